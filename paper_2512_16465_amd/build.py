"""Builds libgemm.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_2512_16465_amd.build            # compile what changed, link
    python -m paper_2512_16465_amd.build --force    # recompile everything
    python -m paper_2512_16465_amd.build --define NAME=VALUE [--define ...] --output /some/where/libgemm_x.so
        # a second build with compile-time switches of the kernels set differently (for A/B measurements:
        # bench.py --library loads it); its objects go to a directory next to the output

Objects go to paper_2512_16465_amd/_build/ (not tracked); the shared library lands next to
this file so that it travels with the source tree.  Every build also compiles
diagnostics/*.hip into libceilings.so, measuring aids that only bench.py loads.
"""
from __future__ import annotations

import concurrent.futures as cf
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgemm.so")

DIAG_SRC = [os.path.join(HERE, "diagnostics", n) for n in ("mfma_ceiling.hip", "hbm_read_ceiling.hip")]
DIAG_LIB = os.path.join(HERE, "libceilings.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-c++20-extensions", "-fPIC", "-fvisibility=hidden",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function", "-Wno-unknown-pragmas",
    # never let the compiler form packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _tile_variant_indices():
    idx = []
    for line in open(os.path.join(CSRC, "tile_variants.def")):
        m = re.match(r"\s*GEMM_TILE_VARIANT\(\s*(\d+)\s*,", line)
        if m:
            idx.append(int(m.group(1)))
    return idx


def _units():
    """(source, object, extra flags) for every translation unit."""
    units = []
    for name in ("gemm_api.hip", "general_kernel.hip", "skinny_kernel.hip", "gemv_f32_kernel.hip", "gemv16_kernel.hip", "tile_dispatch.hip"):
        units.append((os.path.join(CSRC, name), os.path.join(OBJ, name.replace(".hip", ".o")), []))
    for i in _tile_variant_indices():      # one small source file per variant of tile_variants.def
        units.append((os.path.join(CSRC, f"tile_variant_{i}.hip"), os.path.join(OBJ, f"tile_variant_{i}.o"), []))
    return units


def device_assembly(source_name: str, out_path: str) -> str:
    """Compiles the device side of one translation unit of csrc/ to gfx950 assembly text, with the
    flags the library is built with.  For checks that read the generated code."""
    src = os.path.join(CSRC, source_name)
    cmd = [HIPCC, *[f for f in FLAGS if f != "-fPIC"], "--cuda-device-only", "-S", src, "-o", out_path]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed: {' '.join(cmd)}\n{p.stderr}")
    return out_path


def _newest_header():
    t = 0.0
    for root in (CSRC, os.path.join(os.path.dirname(HERE), "include")):
        for f in os.listdir(root):
            if f.endswith((".hpp", ".h", ".def", ".inc")):
                t = max(t, os.path.getmtime(os.path.join(root, f)))
    return t


def _compile(unit):
    src, obj, extra = unit
    cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature", "unknown feature")
    err = "\n".join(l for l in p.stderr.splitlines() if not any(n in l for n in noise))
    return p.returncode, " ".join(cmd), err


def build_diagnostics(force: bool = False) -> str:
    """libceilings.so: the register-only MFMA loops and the plain read kernel bench.py times beside the GEMM."""
    if force or not os.path.exists(DIAG_LIB) or os.path.getmtime(DIAG_LIB) < max(os.path.getmtime(f) for f in DIAG_SRC):
        cmd = [HIPCC, *FLAGS, "-shared", *DIAG_SRC, "-o", DIAG_LIB]
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed: {' '.join(cmd)}\n{p.stderr}")
    return DIAG_LIB


def build_library(force: bool = False, jobs: int = 8, verbose: bool = True, defines=(), output: str = "") -> str:
    global OBJ, LIB, FLAGS
    if output:
        LIB = os.path.abspath(output)
        OBJ = LIB + ".objs"
    if defines:
        FLAGS = FLAGS + ["-D" + d for d in defines]
    os.makedirs(OBJ, exist_ok=True)
    hdr = _newest_header()
    todo = []
    for u in _units():
        src, obj, _ = u
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), hdr):
            todo.append(u)
    if todo:
        with cf.ThreadPoolExecutor(max_workers=max(1, min(jobs, len(todo)))) as ex:
            for rc, cmd, err in ex.map(_compile, todo):
                if verbose and err.strip():
                    print(err, file=sys.stderr)
                if rc != 0:
                    raise RuntimeError(f"hipcc failed: {cmd}\n{err}")
    objs = [u[1] for u in _units()]
    if todo or force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", LIB, *objs]
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"link failed: {' '.join(cmd)}\n{p.stderr}")
    return LIB


if __name__ == "__main__":
    argv = sys.argv[1:]
    defs = [argv[i + 1] for i, x in enumerate(argv) if x == "--define" and i + 1 < len(argv)]
    outp = next((argv[i + 1] for i, x in enumerate(argv) if x == "--output" and i + 1 < len(argv)), "")
    if not outp:
        print(build_diagnostics(force="--force" in argv))
    print(build_library(force="--force" in argv or bool(defs), defines=defs, output=outp))

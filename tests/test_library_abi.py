"""CPU-only: the C-ABI shared library loads and exports every symbol include/gemm.h declares;
the binding marshals arguments only.  No compute call is made here (there is no GPU)."""
import ctypes
import os
import re

import paper_2512_16465_amd as lg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gemm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gemm_[a-z_]+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = declared_functions()
    for must in ("gemm_create", "gemm_run", "gemm_destroy", "gemm_status_string"):
        assert must in names
    assert sorted(lg.EXPORTED_SYMBOLS) == names


def test_library_loads_and_exports_every_declared_symbol():
    lib = lg.load_library()
    for name in declared_functions():
        assert getattr(lib, name) is not None
    # nothing but the declared entry points is exported with a gemm_ prefix
    assert isinstance(lib, ctypes.CDLL)


def test_measuring_aids_of_the_bench_are_built_and_answer_on_the_host():
    """libceilings.so (register-only MFMA loops and a read-only kernel, loaded by bench.py alone) exports its entry
    points; those that make no HIP call answer here, and the launchers refuse bad arguments before any HIP call."""
    path = os.path.join(ROOT, "paper_2512_16465_amd", "libceilings.so")
    assert os.path.exists(path), "run python -m paper_2512_16465_amd.build"
    lib = ctypes.CDLL(path)
    lib.mfma_ceiling_bytes_per_workgroup.restype = ctypes.c_size_t
    lib.mfma_ceiling_flop.restype = ctypes.c_double
    lib.mfma_ceiling_flop.argtypes = [ctypes.c_int, ctypes.c_int]
    assert lib.mfma_ceiling_bytes_per_workgroup() == 16 * 256 * 16
    # 64 instructions of 2*16*16*32 flop (or 32 of 2*32*32*16) per pass and wave, four waves per workgroup
    assert lib.mfma_ceiling_flop(256, 1000) == 256 * 4 * 1000 * 64 * 2 * 16 * 16 * 32
    lib.mfma_ceiling_launch.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.mfma_ceiling_launch(2, 256, 16, 16, 1, 16, 16, None) == -1      # unknown shape
    assert lib.mfma_ceiling_launch(1, 256, 16, None, 1, 16, 16, None) == -1    # no data
    assert lib.mfma_ceiling_launch(1, 256, 0, 16, 1, 16, 16, None) == -1       # no passes
    lib.hbm_read_launch.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert lib.hbm_read_launch(None, 1 << 20, 256, 16, None) == -1             # no data
    assert lib.hbm_read_launch(16, (1 << 20) + 16, 256, 16, None) == -1        # not whole trips
    assert lib.hbm_read_launch(16, 1 << 20, 0, 16, None) == -1                 # no workgroups


def test_host_only_entry_points_answer_without_a_gpu():
    assert lg.gemm_status_string(0) == "success"
    assert "invalid" in lg.gemm_status_string(1)
    assert lg.gemm_status_string(12345) == "unknown status"
    names = []
    i = 0
    while lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, i) is not None:
        names.append(lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, i))
        i += 1
    assert len(names) >= 2 and len(set(names)) == len(names)
    assert lg.gemm_variant_name(lg.GEMM_KERNEL_SKINNY, 0) is not None
    assert lg.gemm_variant_name(lg.GEMM_KERNEL_AUTO, 0) is None
    # argument errors that are detected before any HIP call
    assert lg.gemm_run(0, 1, 1, 1, 0, 0, 0, 1.0, 0, 1, 0, 1, 0.0, 0, 1, None, 0, check=False) == lg.GEMM_ERR_INVALID_ARG
    assert lg.gemm_set_plan(0, lg.GEMM_KERNEL_GENERAL, 0, 0, check=False) == lg.GEMM_ERR_INVALID_ARG


def test_oracle_and_library_share_no_code():
    """Neither side imports the other, and the oracle's sources are not part of the library build."""
    pkg = os.path.join(ROOT, "paper_2512_16465_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".def")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2512_16465_amd" not in text and "gemm.h" not in text and "hip" not in text.lower().replace("relationship", ""), f

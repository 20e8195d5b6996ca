#!/usr/bin/env python3
"""Benchmark of libgemm on one MI355X.

    python bench.py [--gpus 1] [--steps 50] [--warmup 10] [--settle-ms 80] [--configs C3,C5,...] [--no-cpu-baseline]

A "step" is one gemm_run call on the headline workload (C3: bf16 8192^3, row-major A and B,
fp32 output) with operands resident in HBM.  The protocol follows the paper's evaluation
(Section 5.1): warm-up launches, then timed launches, mean latency reported.  Prints ONE JSON
line; `value` is TFLOP/s on C3, `roofline` prices the dominant kernel of C3 against the dense
bf16 MFMA peak, `cpu_baseline` times the CPU oracle on a bounded sample of the same workload,
and `other_configs` carries the remaining configurations (C5 is priced against HBM bandwidth).
`mfma_ceiling` is context for the compute-bound rows: the rate and clock of register-only MFMA
loops on values drawn like the headline's operands and on zeros, measured in the same process;
`hbm_read_ceiling` is the same for the bandwidth-bound rows: what a kernel that only reads gets.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16 matrix-core peak
FP32_VECTOR_PEAK_TFLOPS = 157.3
FP32_MFMA_PEAK_TFLOPS = 157.3      # fp32 matrix-core peak (same figure as the vector ALUs)
HBM_PEAK_GBPS = 8000.0


def kernel_source_hash() -> str:
    """Hash of the kernel sources: counter-derived traffic figures are only quoted while the
    kernels they were measured on are unchanged."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2512_16465_amd", "csrc")
    for f in sorted(os.listdir(csrc)):
        h.update(f.encode())
        h.update(open(os.path.join(csrc, f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(name: str):
    """HBM bytes per launch from the rocprofv3 counter runs recorded in profiles/traffic.json,
    or None when absent or taken on different kernel sources."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    rec = json.load(open(path)).get(name)
    if not rec or rec.get("kernel_source_hash") != kernel_source_hash():
        return None
    return rec.get("hbm_bytes_per_launch")


def classify(cfg) -> str:
    """The paper's roofline rule (Section 4.3): left of the ridge of the slowest unit (fp32
    vector ALUs) is memory-bound, right of the ridge of the fastest unit that can do the work (the
    matrix cores for the operand type) is compute-bound, in between is the middle zone."""
    import workloads as wl
    ai = cfg.flops() / cfg.algorithmic_bytes()
    low = FP32_VECTOR_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBPS * 1e9)
    high = (FP32_MFMA_PEAK_TFLOPS if cfg.dtype == wl.F32 else MFMA_BF16_PEAK_TFLOPS) * 1e12 / (HBM_PEAK_GBPS * 1e9)
    return "memory-bound" if ai < low else ("compute-bound" if ai > high else "middle-zone")


class Resident:
    """Operands of one configuration in HBM; `copies` independent input sets are rotated so that
    a memory-bound call cannot be served from the 256 MB last-level cache."""

    def __init__(self, cfg, seed, copies=1):
        import torch
        import workloads as wl
        self.cfg = cfg
        dev = torch.device("cuda:0")
        self.sets = []
        self.host_inputs = None
        for c in range(copies):
            inp = wl.make_inputs(cfg, seed + c)
            if c == 0:
                self.host_inputs = inp
            A = wl.bits_to_torch(inp["A"], cfg.dtype, dev)
            B = wl.bits_to_torch(inp["B"], cfg.dtype, dev)
            tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[cfg.out_dtype]
            if inp["C"] is not None:
                C = wl.bits_to_torch(inp["C"], cfg.out_dtype, dev)
            else:
                C = torch.empty(cfg.batch * cfg.M * cfg.ld_c(), dtype=tdt, device=dev)
            bias = wl.bits_to_torch(inp["bias"], cfg.bias_dtype, dev) if inp["bias"] is not None else None
            self.sets.append((A, B, C, bias))

    def launch(self, lg, handle, i, stream):
        cfg = self.cfg
        A, B, C, bias = self.sets[i % len(self.sets)]
        epi = lg.make_epilogue(cfg.out_dtype, bias.data_ptr() if bias is not None else 0, cfg.bias_dtype, cfg.act)
        if cfg.batch > 1:
            lg.gemm_run_batched(handle, cfg.batch, cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, cfg.alpha,
                                A.data_ptr(), cfg.ld_a(), cfg.stride_a(), B.data_ptr(), cfg.ld_b(), cfg.stride_b(),
                                cfg.beta, C.data_ptr(), cfg.ld_c(), cfg.stride_c(), epi, stream)
            return
        lg.gemm_run(handle, cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, cfg.alpha,
                    A.data_ptr(), cfg.ld_a(), B.data_ptr(), cfg.ld_b(), cfg.beta, C.data_ptr(), cfg.ld_c(), epi, stream)


def time_config(lg, handle, res: Resident, steps: int, warmup: int, settle_ms: float = 0.0):
    """Returns (wall ms per step over the whole timed region; mean launch duration from HIP events
    on the launch stream around that region; min and std of single launches timed by an event
    pair each; warm-up launches done).

    Warm-up: `warmup` launches, then further launches until `settle_ms` have passed since the
    first one.  After an idle period (input generation, the sampled check) the part needs about
    50 ms of continuous work before launch times stop falling (8192^3: 915 us for the first
    launches, 750 us from the 60th on), so a warm-up counted in launches alone would leave the
    short configurations inside that ramp.  The timed region is exactly `steps` launches."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    t_warm = time.perf_counter()
    done = 0
    while done < warmup or (time.perf_counter() - t_warm) * 1e3 < settle_ms:
        batch = min(10, warmup - done) if done < warmup else 10
        for i in range(batch):
            res.launch(lg, handle, done + i, stream)
        done += batch
        if done >= warmup:
            torch.cuda.synchronize()        # the clock is only read between batches
    # pass 1: the timed region, nothing but the launches between the two syncs; host wall clock
    # around it, and one pair of events on the launch stream around the same launches (the mean
    # launch duration that the roofline figure uses: device time, back to back, no host in it)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for i in range(steps):
        res.launch(lg, handle, i, stream)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    mean = ev0.elapsed_time(ev1) / steps
    # pass 2: launch by launch, for the spread (an event pair per launch costs a few microseconds
    # of its own, which is why the mean comes from pass 1)
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    for i in range(steps):
        starts[i].record()
        res.launch(lg, handle, i, stream)
        stops[i].record()
    torch.cuda.synchronize()
    per = [starts[i].elapsed_time(stops[i]) for i in range(steps)]
    pmean = sum(per) / len(per)
    var = sum((x - pmean) ** 2 for x in per) / len(per)
    return (t1 - t0) * 1e3 / steps, mean, min(per), var ** 0.5, done


def quick_verify(res: Resident, lg, handle):
    """A sampled check of the timed call against the oracle (256 elements), outside the timed region."""
    import numpy as np
    import torch
    import oracle
    import workloads as wl
    cfg = res.cfg
    inp = res.host_inputs
    A, B, C, bias = res.sets[0]
    if inp["C"] is not None:
        C.copy_(wl.bits_to_torch(inp["C"], cfg.out_dtype, C.device))
    res.launch(lg, handle, 0, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    rows, cols = wl.sample_indices(cfg.M, cfg.N, 1, grid=16)
    last = cfg.batch - 1                 # a batch is checked on its last matrix
    flat = (torch.from_numpy(rows).to(C.device) * cfg.ld_c() + torch.from_numpy(cols).to(C.device)) + last * cfg.stride_c()
    got = oracle.decode(cfg.out_dtype, wl.torch_to_bits(C[flat]))
    prob = oracle.Problem(cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, inp["A"][last * cfg.stride_a():], cfg.ld_a(),
                          inp["B"][last * cfg.stride_b():], cfg.ld_b(),
                          alpha=cfg.alpha, beta=cfg.beta, C=None if inp["C"] is None else inp["C"][last * cfg.stride_c():],
                          ldc=cfg.ld_c(), c_dtype=cfg.out_dtype,
                          bias=inp["bias"], bias_dtype=cfg.bias_dtype, act=cfg.act)
    ref, _, mag = oracle.gemm_at(prob, rows, cols)
    tol = (1e-5 * mag + 1e-6) if cfg.dtype == wl.F32 else (4e-3 * mag + 1e-5)
    return bool(np.all(np.abs(got - ref) <= tol))


def cpu_baseline(res: Resident, target_seconds: float = 12.0):
    """The oracle as it stands, on the host cores, over whole rows of C of the same workload (of the
    first matrix of a batch); the time for the whole workload is a projection from that sample."""
    import oracle
    cfg = res.cfg
    inp = res.host_inputs
    prob = oracle.Problem(cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, inp["A"], cfg.ld_a(), inp["B"], cfg.ld_b(),
                          alpha=cfg.alpha, beta=cfg.beta, C=inp["C"], ldc=cfg.ld_c(), c_dtype=cfg.out_dtype,
                          bias=inp["bias"], bias_dtype=cfg.bias_dtype, act=cfg.act)
    cores = oracle.num_threads()
    t0 = time.perf_counter()
    oracle.gemm_rows(prob, 0, 1)                      # calibration: one row
    t_row = time.perf_counter() - t0
    nrows = int(max(1, min(cfg.M, target_seconds / max(t_row, 1e-6))))
    t0 = time.perf_counter()
    oracle.gemm_rows(prob, 0, nrows)
    dt = time.perf_counter() - t0
    flops = 2.0 * nrows * cfg.N * cfg.K
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"rows 0..{nrows - 1} of C ({nrows} x {cfg.N} outputs, K={cfg.K}) in {dt:.1f} s; "
                      f"projected whole workload {dt * cfg.M * cfg.batch / nrows:.1f} s",
            "projected_seconds": dt * cfg.M * cfg.batch / nrows}


def _ceilings_library():
    """The measuring aids of paper_2512_16465_amd/diagnostics/ (a library of their own), or None when not built."""
    import ctypes
    path = os.path.join(ROOT, "paper_2512_16465_amd", "libceilings.so")
    return ctypes.CDLL(path) if os.path.exists(path) else None


def hbm_read_ceiling(torch, sizes_mib=(128, 512), launches: int = 40, settle_ms: float = 30.0):
    """GB/s of a kernel that only reads (paper_2512_16465_amd/diagnostics/hbm_read_ceiling.hip: coalesced 16-byte
    loads, eight per lane in flight) over buffers of the sizes of the streamed weights, 1 GiB of buffers in
    rotation so that the 256 MB last-level cache cannot serve them, best of three grid sizes.  Context for the
    bandwidth-bound rows, whose roofline.frac stays a fraction of the nominal 8 TB/s."""
    import ctypes
    lib = _ceilings_library()
    if lib is None:
        return {"error": "libceilings.so is not built (python -m paper_2512_16465_amd.build)"}
    lib.hbm_read_launch.restype = ctypes.c_int
    lib.hbm_read_launch.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    dev = torch.device("cuda:0")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    out = {"kernel": "grid-stride 16-byte loads, 8 per lane in flight, nothing stored", "peak_gbps": HBM_PEAK_GBPS,
           "launches": launches, "sizes": {}}
    for mib in sizes_mib:
        nbytes = mib << 20
        bufs = [torch.full((nbytes,), 0x5a, dtype=torch.uint8, device=dev) for _ in range(max(2, 1024 // mib))]
        best = None
        for per_cu in (4, 8, 16):
            def launch(i):
                rc = lib.hbm_read_launch(bufs[i % len(bufs)].data_ptr(), nbytes, cus * per_cu, sink.data_ptr(), stream)
                if rc != 0:
                    raise RuntimeError(f"hbm_read_launch returned {rc}")
            t0, i = time.perf_counter(), 0
            while (time.perf_counter() - t0) * 1e3 < settle_ms:
                launch(i)
                i += 1
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for i in range(launches):
                launch(i)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / launches
            gbps = nbytes / (ms * 1e-3) / 1e9
            if best is None or gbps > best["gbps"]:
                best = {"gbps": gbps, "frac_of_peak": gbps / HBM_PEAK_GBPS, "us_per_launch": ms * 1e3, "workgroups_per_cu": per_cu}
        out["sizes"][f"{mib} MiB"] = best
        del bufs
        torch.cuda.empty_cache()
    return out


def mfma_ceiling(torch, cfg, seed: int, settle_ms: float = 150.0, launches: int = 10, passes: int = 16384):
    """Rate and clock of register-only MFMA loops (paper_2512_16465_amd/diagnostics/mfma_ceiling.hip: no
    memory traffic in the timed part, the register blocking of the 256x256 tile) on operand values drawn
    like cfg's A and B, and on zeros.  What the part's power limit leaves of the nominal peak to any
    kernel on such data; context for roofline.frac, which stays a fraction of the nominal peak."""
    import ctypes
    lib = _ceilings_library()
    if lib is None:
        return {"error": "libceilings.so is not built (python -m paper_2512_16465_amd.build)"}
    lib.mfma_ceiling_bytes_per_workgroup.restype = ctypes.c_size_t
    lib.mfma_ceiling_flop.restype = ctypes.c_double
    lib.mfma_ceiling_flop.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.mfma_ceiling_launch.restype = ctypes.c_int
    lib.mfma_ceiling_launch.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    dev = torch.device("cuda:0")
    wgs = torch.cuda.get_device_properties(0).multi_processor_count     # one workgroup of four waves per compute unit
    per_wg = lib.mfma_ceiling_bytes_per_workgroup()
    assert per_wg == 16 * 256 * 16
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    # per workgroup 16 fragments x 256 lanes x 8 values: the first 8 fragments play A, the others B
    def draw(dist):
        if dist[0] == "normal":
            return torch.randn((wgs, 8, 256, 8), generator=gen, device=dev) * dist[1]
        return (torch.rand((wgs, 8, 256, 8), generator=gen, device=dev) * 2.0 - 1.0) * dist[1]
    like = torch.cat([draw(cfg.a_dist), draw(cfg.b_dist)], dim=1).to(torch.bfloat16).contiguous()
    zeros = torch.zeros_like(like)
    assert like.numel() * 2 == wgs * per_wg
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    stamps = torch.zeros(2 * wgs, dtype=torch.int64, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    flop = lib.mfma_ceiling_flop(wgs, passes)
    out = {"kernel": "register-only loops of independent MFMAs, 256 accumulator registers per lane, one wave per SIMD",
           "workgroups": wgs, "passes": passes, "launches": launches, "peak_tflops": MFMA_BF16_PEAK_TFLOPS, "cases": {}}
    for shape, sname in ((1, "v_mfma_f32_16x16x32_bf16"), (0, "v_mfma_f32_32x32x16_bf16")):
        for data, dname in ((like, "values drawn like the operands"), (zeros, "zeros")):
            def launch():
                rc = lib.mfma_ceiling_launch(shape, wgs, passes, data.data_ptr(), wgs, sink.data_ptr(), stamps.data_ptr(), stream)
                if rc != 0:
                    raise RuntimeError(f"mfma_ceiling_launch returned {rc}")
            t0 = time.perf_counter()
            while (time.perf_counter() - t0) * 1e3 < settle_ms:      # the clock settles under the load first
                launch()
                torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(launches):
                launch()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / launches
            st = stamps.cpu().view(wgs, 2).double()
            ghz = float((st[:, 0] / st[:, 1]).mean()) * 0.1          # shader cycles per tick of the 100 MHz constant clock
            tf = flop / (ms * 1e-3) / 1e12
            out["cases"][f"{sname}, {dname}"] = {"tflops": tf, "frac_of_peak": tf / MFMA_BF16_PEAK_TFLOPS, "ghz": ghz,
                                                 "ms_per_launch": ms}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--configs", default="C3,C5,C2,C4,C1,X1,X2,X3,X4,X5,X6,X7,X8,X11,G1,G2,G3,G4,G5,G6,G7,G8",
                    help="first one is the headline workload; X* are the further shapes of workloads.EXTRA_CONFIGS")
    ap.add_argument("--settle-ms", type=float, default=80.0,
                    help="the warm-up keeps launching until this much time has passed (clock ramp after idle); 0 = exactly --warmup launches")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="oracle time spent on the headline workload")
    ap.add_argument("--cpu-seconds-other", type=float, default=1.0,
                    help="oracle time spent on each further configuration (a projection from a few rows of C); 0 = none")
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--no-mfma-ceiling", action="store_true",
                    help="skip the register-only MFMA loops that show what the power limit leaves of the nominal peak")
    ap.add_argument("--no-hbm-ceiling", action="store_true", help="skip the read-only kernel that shows what plain reads get of 8 TB/s")
    ap.add_argument("--kernel", type=int, default=0, help="force a kernel family (gemm_kernel_t); 0 = automatic")
    ap.add_argument("--variant", type=int, default=-1, help="tile variant when --kernel is forced")
    ap.add_argument("--split-k", type=int, default=0, help="split-K factor when --kernel is forced; 0 = automatic")
    ap.add_argument("--library", default="", help="path of another build of libgemm.so to measure (see paper_2512_16465_amd/build.py --output)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy (3 times) so that a counter run can scale "
                         "FETCH_SIZE / WRITE_SIZE by what they read for a transfer of known size")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this library is single-GPU by design; run with --gpus 1 "
              "(one GPU computes the whole product; nothing here shards it)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_16465_amd as lg
    import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.library:
        import paper_2512_16465_amd.binding as binding
        binding.LIB_PATH = os.path.abspath(args.library)
    lg.load_library()          # fails loudly when the HIP library is not built
    seed = wl.DEFAULT_SEED if args.seed is None else args.seed
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    handle = lg.gemm_create()
    if args.kernel:
        lg.gemm_set_plan(handle, args.kernel, args.variant, args.split_k)
    names = [n.strip() for n in args.configs.split(",") if n.strip()]
    results = {}
    headline = None
    for idx, name in enumerate(names):
        cfg = wl.CONFIGS[name] if name in wl.CONFIGS else wl.EXTRA_CONFIGS[name]
        bound = "hbm" if classify(cfg) != "compute-bound" else "mfma"
        res = Resident(cfg, seed, copies=2 if bound == "hbm" and cfg.algorithmic_bytes() > (64 << 20) else 1)
        ok = None if args.no_verify else quick_verify(res, lg, handle)
        wall_ms, ev_mean, ev_min, ev_std, warm_done = time_config(lg, handle, res, args.steps, args.warmup, args.settle_ms)
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        kname = lg.gemm_variant_name(kernel, variant)
        tflops = cfg.flops() / (wall_ms * 1e-3) / 1e12
        gbps = cfg.algorithmic_bytes() / (wall_ms * 1e-3) / 1e9
        if name == "C1":
            roof = None          # launch-latency bound: no roofline is meaningful
        elif bound == "mfma":
            ach = cfg.flops() / (ev_mean * 1e-3) / 1e12
            peak = FP32_MFMA_PEAK_TFLOPS if cfg.dtype == wl.F32 else MFMA_BF16_PEAK_TFLOPS    # the contraction's own type
            roof = {"bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                    "frac": ach / peak, "traffic": measured_traffic(name), "kernel": kname}
        else:
            ach = cfg.algorithmic_bytes() / (ev_mean * 1e-3) / 1e9
            roof = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBPS, "traffic": measured_traffic(name), "kernel": kname}
        results[name] = {
            "workload": cfg.note, "class": classify(cfg), "kernel": kname, "split_k": split,
            "ms_per_step": wall_ms, "launch_ms_mean": ev_mean, "launch_ms_min": ev_min, "launch_ms_std": ev_std,
            "tflops": tflops, "algorithmic_gbps": gbps, "verified_sample": ok, "warmup_launches": warm_done, "roofline": roof,
        }
        if idx > 0 and not args.no_cpu_baseline and args.cpu_seconds_other > 0:
            results[name]["cpu_baseline"] = cpu_baseline(res, args.cpu_seconds_other)
        if idx == 0:
            headline = (name, cfg, res, wall_ms, tflops, roof)
        else:
            del res
            torch.cuda.empty_cache()

    name, cfg, res, wall_ms, tflops, roof = headline
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(res, args.cpu_seconds)
    torch.cuda.synchronize()
    lg.gemm_destroy(handle)
    ceiling = None if args.no_mfma_ceiling or cfg.dtype != wl.BF16 else mfma_ceiling(torch, cfg, seed)
    if ceiling and "cases" in ceiling and roof and roof["bound"] == "mfma":
        like = ceiling["cases"]["v_mfma_f32_16x16x32_bf16, values drawn like the operands"]["tflops"]
        ceiling["headline_over_ceiling"] = roof["achieved"] / like      # the GEMM against the loop of its own instruction
    line = {
        "metric": "gemm_tflops_bf16_8192cubed" if name == "C3" else f"gemm_tflops_{name}",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        # launches before the timed region: at least --warmup, then as many as fill --settle-ms (clock ramp)
        "warmup": results[name]["warmup_launches"], "warmup_requested": args.warmup, "settle_ms": args.settle_ms,
        "ms_per_step": wall_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "clocks": {"value, ms_per_step, tflops, algorithmic_gbps": "host wall clock around the timed launches, between two device synchronisations",
                   "roofline.achieved, launch_ms_*": "HIP events on the launch stream around the same number of launches"},
        "dtype": "bf16" if cfg.dtype == wl.BF16 else ("f16" if cfg.dtype == wl.F16 else "f32"),
        "data": "synthetic",
        "config": {"workload": f"{name}: {cfg.note}", "M": cfg.M, "N": cfg.N, "K": cfg.K,
                   "accumulate": "f32", "out_dtype": {0: "f32", 1: "f16", 2: "bf16"}[cfg.out_dtype], "seed": seed},
        "pct_of_mfma_peak": 100.0 * tflops / MFMA_BF16_PEAK_TFLOPS,
        "roofline": roof,
        "cpu_baseline": cpu,
        "mfma_ceiling": ceiling,
        "hbm_read_ceiling": None if args.no_hbm_ceiling else hbm_read_ceiling(torch),
        "hbm_gbps_at_m32": results["C5"]["algorithmic_gbps"] if "C5" in results else None,
        "other_configs": {k: v for k, v in results.items() if k != name},
        "headline_detail": results[name],
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

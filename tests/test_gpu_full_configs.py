"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (automatic
plan, default leading dimensions): a stratified sample of 4096 output elements against the
oracle, plus properties that involve every output element without an O(MNK) reference --
integer-exact data checked by a Freivalds-style product with random sign vectors, all-ones
inputs, and run-to-run determinism."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import DeviceProblem, check_sampled, decode_c, oracle_problem

pytestmark = pytest.mark.gpu

FULL = ["C2", "C3", "C4", "C5", "X1", "X2", "X3", "X4", "X5", "X6", "X7", "X9", "X10", "X11",
        "G1", "G2", "G3", "G4", "G5", "G6", "G7", "G8"]
ALL = {**wl.CONFIGS, **wl.EXTRA_CONFIGS}
SKINNY = ("C5", "X5", "X7", "G1", "G2", "G4", "G5", "G6", "G7", "G8")      # the streaming kernels (bf16/fp16 skinny, fp32 rows)


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    torch.cuda.synchronize()
    lg.gemm_destroy(h)


def dense(cfg, storage, shape, ld):
    return storage.reshape(shape[0], ld)[:, : shape[1]]


@pytest.mark.parametrize("name", FULL)
def test_sampled_against_oracle(handle, name):
    cfg = ALL[name]
    print(f"{name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg)
    p = DeviceProblem(cfg, inp)
    print(f"{name}: running", flush=True)
    p.run(handle)
    bits = p.result_bits()
    kernel, variant, split = lg.gemm_get_last_plan(handle)
    print(f"{name}: plan kernel={kernel} variant={variant} split={split}; oracle on the sample", flush=True)
    expected_kernel = lg.GEMM_KERNEL_SKINNY if name in SKINNY else lg.GEMM_KERNEL_MFMA_TILE
    assert kernel == expected_kernel
    check_sampled(cfg, inp, bits, wl.DEFAULT_SEED, name)
    # same call again on the same data: same bits
    first = bits.copy()
    p.reset_c()
    p.run(handle)
    assert np.array_equal(first.view(np.uint8), p.result_bits().view(np.uint8))


@pytest.mark.parametrize("name", FULL)
def test_integer_exact_with_full_coverage(handle, name):
    """Entries in {-1, 0, 1}: every partial sum is an exact integer below 2^24, so C is unique.
    With fp32 output, C r = A (B r) and r^T C = (r^T A) B must hold EXACTLY for sign vectors r
    (int64 arithmetic on the host, O(MK + KN + MN)); each output element takes part in both."""
    cfg = wl.scaled(ALL[name], out_dtype=wl.F32, act=wl.ACT_NONE, bias_dist=None)
    inp, vals = wl.make_integer_inputs(cfg, 2024, -1, 1)
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    check_integer_result(cfg, inp, vals, p.result_bits()[:, : cfg.N])


def check_integer_result(cfg, inp, vals, C):
    Ci = np.rint(C).astype(np.int64)
    assert np.array_equal(Ci.astype(np.float32), C), "non-integer output on integer data"
    opA = vals["A"].T if cfg.transA else vals["A"]          # M x K
    opB = vals["B"].T if cfg.transB else vals["B"]          # K x N
    rng = np.random.default_rng(7)
    extra = cfg.beta * vals["C"] if cfg.beta != 0.0 else 0
    for _ in range(2):
        r = rng.choice(np.array([-1, 1], dtype=np.int64), size=cfg.N)
        want = cfg.alpha * (opA @ (opB @ r)) + (extra @ r if cfg.beta != 0.0 else 0)
        assert np.array_equal(Ci @ r, np.asarray(want, dtype=np.int64)), "row check failed"
        l = rng.choice(np.array([-1, 1], dtype=np.int64), size=cfg.M)
        want = cfg.alpha * ((l @ opA) @ opB) + (l @ extra if cfg.beta != 0.0 else 0)
        assert np.array_equal(l @ Ci, np.asarray(want, dtype=np.int64)), "column check failed"
    # and a sample against the oracle, exact
    rows, cols = wl.sample_indices(cfg.M, cfg.N, 5)
    ref, _, _ = oracle.gemm_at(oracle_problem(cfg, inp), rows, cols)
    assert np.array_equal(C[rows, cols].astype(np.float64), ref)


@pytest.mark.parametrize("name,variant,split", [("X4", 5, 1), ("X4", 10, 1), ("X4", 15, 1), ("C5", 15, 4), ("X7", 14, 4), ("X7", 10, 8),
                                                ("X7", 5, 4), ("C2", 14, 1), ("C2", 5, 2)])
def test_forced_tile_plans_at_full_size(handle, name, variant, split):
    """Plans the automatic choice does not take at these shapes, among them the rotated k walks of the
    streaming calls (one row or column of tiles beyond the last-level cache; splits of at most four shares) on
    the 128x128, 256x128, 128x256 and 256x256 tiles, and k slices at full size: same exact checks."""
    cfg = wl.scaled(ALL[name], out_dtype=wl.F32, act=wl.ACT_NONE, bias_dist=None)
    inp, vals = wl.make_integer_inputs(cfg, 2025, -1, 1)
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, variant, split)
    try:
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, variant, split)
    finally:
        lg.gemm_set_plan(handle)
    check_integer_result(cfg, inp, vals, p.result_bits()[:, : cfg.N])


@pytest.mark.parametrize("name", FULL)
def test_all_ones_gives_k(handle, name):
    cfg = wl.scaled(ALL[name], act=wl.ACT_NONE, bias_dist=None)
    one = lambda shape, ld, dt: wl.to_bits(np.ones(shape[0] * ld, np.float32), dt)
    inp = {"A": one(cfg.a_shape(), cfg.ld_a(), cfg.dtype), "B": one(cfg.b_shape(), cfg.ld_b(), cfg.dtype),
           "C": one((cfg.M, cfg.N), cfg.ld_c(), cfg.out_dtype) if cfg.beta != 0.0 else None, "bias": None}
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    got = decode_c(cfg, p.result_bits())
    exact = cfg.alpha * cfg.K + (cfg.beta if cfg.beta != 0.0 else 0.0)
    want = oracle.decode(cfg.out_dtype, oracle.encode(cfg.out_dtype, np.array([exact])))[0]   # e.g. 16385 -> 16384 in bf16
    assert np.all(got == want), f"{name}: {np.sum(got != want)} elements differ from {want}"


def test_operand_beyond_two_gib(handle):
    """Maximum sizes: an A of more than 2 GiB (16392 x 65536 bf16), where 32-bit byte offsets into
    the operand end.  The operand is drawn on the device (integers in {-1, 0, 1}, exact in bf16);
    the rows on both sides of the 2 GiB line, the first and the last rows are copied back and the
    oracle computes exactly those rows of C, which must match bit for bit (every sum is an
    integer below 2^24)."""
    M, N, K = 16392, 264, 65536
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    print("2 GiB operand: drawing", flush=True)
    A = torch.randint(-1, 2, (M, K), generator=gen, device=dev, dtype=torch.int8).to(torch.bfloat16)
    B = torch.randint(-1, 2, (N, K), generator=gen, device=dev, dtype=torch.int8).to(torch.bfloat16)       # stored N x K
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    assert A.numel() * 2 > 2 ** 31
    epi = lg.make_epilogue(wl.F32)
    print("2 GiB operand: running", flush=True)
    lg.gemm_run(handle, M, N, K, 0, 1, wl.BF16, 1.0, A.data_ptr(), K, B.data_ptr(), K, 0.0, C.data_ptr(), N, epi,
                torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    kernel, variant, _ = lg.gemm_get_last_plan(handle)
    name = lg.gemm_variant_name(kernel, variant)
    print(f"2 GiB operand: ran {name}", flush=True)
    assert kernel == lg.GEMM_KERNEL_MFMA_TILE and not name.startswith("dma"), name      # the direct-to-LDS kernels stop at 2 GiB
    line = 2 ** 31 // (2 * K)                                                            # first row wholly past 2 GiB
    rows = np.unique(np.concatenate([np.arange(0, 3), np.arange(line - 4, line + 4), np.arange(M - 9, M),
                                     np.random.default_rng(3).integers(0, M, 40)]))
    a_rows = wl.torch_to_bits(A[torch.from_numpy(rows).to(dev)].reshape(-1))
    prob = oracle.Problem(len(rows), N, K, 0, 1, wl.BF16, a_rows, K, wl.torch_to_bits(B.reshape(-1)), K, c_dtype=wl.F32)
    ref = oracle.gemm_full(prob)
    got = C[torch.from_numpy(rows).to(dev)].cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref), f"{np.sum(got != ref)} elements differ in the sampled rows"
    # every element is a finite integer (no row or tile was skipped)
    assert bool(torch.all(C == torch.round(C)))


def test_batched_full_config_x8(handle):
    """The strided batch of the bench (32 per-head products 2048 x 2048 x 128) at full size, in the automatic plan:
    a stratified sample of every matrix against the oracle, the same call twice gives the same bits, and on
    integer data every matrix satisfies the sign-vector identities exactly."""
    cfg = ALL["X8"]

    def run(c, inp):
        dev = torch.device("cuda:0")
        A, B = wl.bits_to_torch(inp["A"], c.dtype, dev), wl.bits_to_torch(inp["B"], c.dtype, dev)
        tdt = {wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[c.out_dtype]
        C = torch.full((c.batch * c.M * c.ld_c(),), float("nan"), dtype=tdt, device=dev)
        lg.gemm_run_batched(handle, c.batch, c.M, c.N, c.K, c.transA, c.transB, c.dtype, c.alpha, A.data_ptr(), c.ld_a(),
                            c.stride_a(), B.data_ptr(), c.ld_b(), c.stride_b(), c.beta, C.data_ptr(), c.ld_c(), c.stride_c(),
                            lg.make_epilogue(c.out_dtype), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        return wl.torch_to_bits(C).reshape(c.batch, c.M, c.ld_c())

    print("X8: gaussian batch", flush=True)
    inp = wl.make_inputs(cfg)
    bits = run(cfg, inp)
    assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_MFMA_TILE
    one = wl.scaled(cfg, batch=1)
    for b in range(cfg.batch):
        sub = {"A": inp["A"][b * cfg.stride_a():(b + 1) * cfg.stride_a()], "B": inp["B"][b * cfg.stride_b():(b + 1) * cfg.stride_b()],
               "C": None, "bias": None}
        rows, cols = wl.sample_indices(cfg.M, cfg.N, wl.DEFAULT_SEED + b, grid=16)
        ref, _, mag = oracle.gemm_at(oracle_problem(one, sub), rows, cols)
        got = oracle.decode(cfg.out_dtype, np.ascontiguousarray(bits[b][rows, cols]))
        from gpu_harness import assert_close
        assert_close(one, got, ref, mag, f"X8 matrix {b}")
    again = run(cfg, inp)
    assert np.array_equal(bits.view(np.uint8), again.view(np.uint8)), "X8: two runs differ"
    print("X8: integer batch", flush=True)
    icfg = wl.scaled(cfg, out_dtype=wl.F32)
    iinp, vals = wl.make_integer_inputs(icfg, 2026, -1, 1)
    C = run(icfg, iinp)
    ione = wl.scaled(icfg, batch=1)
    for b in range(cfg.batch):
        v = {"A": vals["A"][b * cfg.M:(b + 1) * cfg.M], "B": vals["B"][b * cfg.N:(b + 1) * cfg.N], "C": None}
        sub = {"A": iinp["A"][b * cfg.stride_a():(b + 1) * cfg.stride_a()], "B": iinp["B"][b * cfg.stride_b():(b + 1) * cfg.stride_b()],
               "C": None, "bias": None}
        check_integer_result(ione, sub, v, C[b][:, : cfg.N])

"""GPU parity on the values Gaussian data never produces: subnormal inputs, results below the
normal range, sums that overflow the type of C, and infinities in an operand.

The result contract is IEEE: products of 16-bit inputs are exact, sums are rounded in fp32, the
output is rounded once to nearest even; a value beyond the largest finite number of the type of C
becomes an infinity, Inf times zero is a NaN.  The oracle computes the same thing in fp64 (where
every product and every partial sum of these small cases is exact) and rounds once, so wherever
the fp32 sums are exact too the two must agree bit for bit.  Each case runs in every kernel family
that takes its layout."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import DeviceProblem, decode_c, oracle_problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    torch.cuda.synchronize()
    lg.gemm_destroy(h)


def store(x, dtype):
    return wl.to_bits(np.ascontiguousarray(x, dtype=np.float32).reshape(-1), dtype)


# (kernel family, variant, split) to force; None = automatic
def plans_for(M, dtype, ta):
    if dtype == wl.F32:
        return [None, (lg.GEMM_KERNEL_MFMA_TILE, 11, 1), (lg.GEMM_KERNEL_MFMA_TILE, 13, 1), (lg.GEMM_KERNEL_GENERAL, 0, 1)]
    plans = [None, (lg.GEMM_KERNEL_MFMA_TILE, 10, 1), (lg.GEMM_KERNEL_MFMA_TILE, 5, 1), (lg.GEMM_KERNEL_MFMA_TILE, 0, 1),
             (lg.GEMM_KERNEL_MFMA_TILE, 5, 2), (lg.GEMM_KERNEL_GENERAL, 0, 1)]
    if M <= 64 and not ta:
        plans += [(lg.GEMM_KERNEL_SKINNY, -1, 1), (lg.GEMM_KERNEL_SKINNY, -1, 2)]
    if M <= 8 and not ta:        # few rows: both kernels for a weight stored N x K, by name (each refuses the other layout)
        plans += [(lg.GEMM_KERNEL_SKINNY, 1, 1), (lg.GEMM_KERNEL_SKINNY, 4, 1), (lg.GEMM_KERNEL_SKINNY, 4, 2), (lg.GEMM_KERNEL_SKINNY, 5, 1)]
    return plans


def run_all_plans(handle, cfg, inp):
    """Yields (plan, C as fp64 values) for every plan that takes the call."""
    for plan in plans_for(cfg.M, cfg.dtype, cfg.transA):
        if plan is None:
            lg.gemm_set_plan(handle)
        else:
            lg.gemm_set_plan(handle, *plan)
        try:
            p = DeviceProblem(cfg, inp)
            st = p.run(handle, check=False)
            if st == lg.GEMM_ERR_UNSUPPORTED:
                continue
            assert st == lg.GEMM_OK, (plan, st)
            yield plan, decode_c(cfg, p.result_bits())
        finally:
            lg.gemm_set_plan(handle)


def same_values(got, want):
    """Equal as IEEE values: same finite numbers, same infinities, NaN where NaN."""
    nan_ok = np.isnan(got) == np.isnan(want)
    rest = np.where(np.isnan(want), True, got == want)
    return bool(np.all(nan_ok) and np.all(rest))


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16])
@pytest.mark.parametrize("M,tb", [(48, 0), (48, 1), (264, 1), (264, 0), (4, 1), (8, 1)])
def test_subnormal_inputs_are_multiplied_not_flushed(handle, dtype, M, tb):
    # A holds small integers times the smallest subnormal of the type, B small integers times a power of two
    # that brings every product and every sum back into the normal fp32 range: all arithmetic is exact
    N, K = 136, 64
    tiny = 2.0 ** -24 if dtype == wl.F16 else 2.0 ** -133
    big = 2.0 ** 10 if dtype == wl.F16 else 2.0 ** 40
    rng = np.random.default_rng(5)
    a = rng.integers(-7, 8, (M, K)).astype(np.float64) * tiny
    b = rng.integers(-3, 4, (K, N)).astype(np.float64) * big
    cfg = wl.Config("subnormal_in", M, N, K, 0, tb, dtype, wl.F32)
    inp = {"A": store(a, dtype), "B": store(b.T if tb else b, dtype), "C": None, "bias": None}
    assert np.array_equal(oracle.decode(dtype, inp["A"]).reshape(M, K), a), "the test's inputs must be exact in the type"
    want = oracle.gemm_full(oracle_problem(cfg, inp))
    assert np.array_equal(want, a @ b) and np.any(want != 0)
    ran = 0
    for plan, got in run_all_plans(handle, cfg, inp):
        assert np.array_equal(got, want), f"{plan}: {np.sum(got != want)} of {got.size} elements differ (subnormal inputs flushed?)"
        ran += 1
    assert ran >= 4


@pytest.mark.parametrize("M,tb", [(40, 0), (40, 1), (136, 1), (3, 1), (8, 1)])
def test_results_below_the_normal_range_of_fp32(handle, M, tb):
    # every product is an integer multiple of 2^-149: sums are exact subnormal fp32 numbers
    N, K = 128, 32
    rng = np.random.default_rng(6)
    a = rng.integers(-3, 4, (M, K)).astype(np.float64) * 2.0 ** -70
    b = rng.integers(-3, 4, (K, N)).astype(np.float64) * 2.0 ** -79
    cfg = wl.Config("subnormal_out", M, N, K, 0, tb, wl.BF16, wl.F32)
    inp = {"A": store(a, wl.BF16), "B": store(b.T if tb else b, wl.BF16), "C": None, "bias": None}
    want = oracle.gemm_full(oracle_problem(cfg, inp))
    assert np.array_equal(want, a @ b) and np.any(want != 0) and np.all(np.abs(want) < 2.0 ** -126)
    for plan, got in run_all_plans(handle, cfg, inp):
        assert np.array_equal(got, want), f"{plan}: {np.sum(got != want)} of {got.size} subnormal results differ"


@pytest.mark.parametrize("dtype,limit", [(wl.F16, 65504.0), (wl.BF16, 3.3895313892515355e38)])
@pytest.mark.parametrize("M,tb", [(32, 0), (32, 1), (200, 1), (2, 1), (8, 1)])
def test_sums_beyond_the_output_type_become_infinite(handle, dtype, limit, M, tb):
    # column j of C is j * step: finite below the largest number of the type, an infinity above it, the sign
    # alternating by row
    N, K = 136, 32
    if dtype == wl.F16:
        a = np.where(np.arange(M)[:, None] % 2 == 0, 1.0, -1.0) * np.full((M, K), 32.0)
        b = np.tile((np.arange(N) * 1.0)[None, :], (K, 1))              # C[i][j] = +-32 * 32 * j = +-1024 j: up to 138240
    else:
        a = np.where(np.arange(M)[:, None] % 2 == 0, 1.0, -1.0) * np.full((M, K), 2.0 ** 100)
        b = np.tile((2.0 ** 20 * np.arange(N))[None, :], (K, 1))        # +-2^125 * j: overflows bf16 from j = 8 on
    cfg = wl.Config("overflow", M, N, K, 0, tb, dtype, dtype)
    inp = {"A": store(a, dtype), "B": store(b.T if tb else b, dtype), "C": None, "bias": None}
    want = oracle.decode(dtype, oracle.encode(dtype, oracle.gemm_full(oracle_problem(cfg, inp))))
    assert np.any(np.isinf(want)) and np.any(np.isfinite(want) & (want != 0)) and np.nanmax(np.abs(want[np.isfinite(want)])) <= limit
    for plan, got in run_all_plans(handle, cfg, inp):
        assert same_values(got, want), f"{plan}: overflow handled differently in {np.sum(~(np.isnan(got) | (got == want)))} elements"


@pytest.mark.parametrize("dtype", [wl.F16, wl.BF16, wl.F32])
@pytest.mark.parametrize("M,tb", [(24, 0), (24, 1), (160, 1), (4, 1), (8, 1)])
def test_an_infinite_input_follows_ieee(handle, dtype, M, tb):
    # A[1][3] = +Inf, A[2][5] = -Inf; B small integers with zeros: Inf * positive = Inf, Inf * 0 = NaN, and rows
    # without an infinity stay finite and exact
    N, K = 128, 32
    rng = np.random.default_rng(8)
    a = rng.integers(-2, 3, (M, K)).astype(np.float64)
    b = rng.integers(-2, 3, (K, N)).astype(np.float64)
    a[1, 3], a[2, 5] = np.inf, -np.inf
    cfg = wl.Config("inf_in", M, N, K, 0, tb, dtype, wl.F32)
    inp = {"A": store(a, dtype), "B": store(b.T if tb else b, dtype), "C": None, "bias": None}
    with np.errstate(invalid="ignore"):
        want = oracle.gemm_full(oracle_problem(cfg, inp))
    assert np.any(np.isnan(want[1])) and np.any(np.isinf(want[1])) and np.all(np.isfinite(want[0])) and np.all(np.isfinite(want[3:]))
    for plan, got in run_all_plans(handle, cfg, inp):
        assert same_values(got, want), f"{plan}: infinities handled differently"

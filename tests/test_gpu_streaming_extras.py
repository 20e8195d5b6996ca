"""GPU parity of the streaming (skinny) family beyond row-major 16-bit A: an A stored K x M, which is
gathered into a row-major copy first, and fp32 operands with at most 8 rows, which run on the vector
ALUs (the matrix-vector product that the paper uses as its memory-bound kernel, Section 5.3)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import DeviceProblem, assert_close, decode_c, expected_bits_exact, oracle_problem

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    torch.cuda.synchronize()
    lg.gemm_destroy(h)


def cfg_of(M, N, K, ta, tb, dtype, out=None, **kw):
    return wl.Config("s", M, N, K, ta, tb, dtype, dtype if out is None else out, **kw)


@pytest.mark.parametrize("tb", [0, 1])
@pytest.mark.parametrize("M", [1, 7, 32, 41, 64])
def test_skinny_with_a_stored_k_by_m(handle, M, tb):
    # any M is taken (the copy is gathered element by element); ragged last column group, partial last step, padded lda
    N, K = 776, 2056
    for dtype in (wl.BF16, wl.F16):
        cfg = cfg_of(M, N, K, 1, tb, dtype, alpha=1.0, beta=1.0, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                     c_dist=("normal", 1.0), lda=M + 3, ldb=(K if tb else N) + 24)
        inp = wl.make_inputs(cfg, 60 + M)
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        for s in (1, 4):
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, s)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_SKINNY, tb, s)
            assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"transA skinny M={M} tb={tb} split {s}")
    lg.gemm_set_plan(handle)
    # integer data: the same bits as with the same A stored row-major
    icfg = cfg_of(M, 520, 1032, 1, tb, wl.BF16, wl.F32)
    iinp, vals = wl.make_integer_inputs(icfg, 9, -2, 2)
    want = oracle.decode(wl.F32, expected_bits_exact(icfg, iinp))
    for s in (1, 3):
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, s)
        p = DeviceProblem(icfg, iinp)
        p.run(handle)
        assert np.array_equal(decode_c(icfg, p.result_bits()), want)
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("tb", [0, 1])
@pytest.mark.parametrize("M", [1, 2, 4, 5, 8])
def test_f32_streaming_kernels(handle, M, tb):
    # ragged column groups (1048 = 4*256 + 24 = 32*32 + 24), K no multiple of a step or trip, padded leading dimensions
    N, K = 1048, 2060
    cfg = cfg_of(M, N, K, 0, tb, wl.F32, alpha=0.5, beta=-1.5, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                 c_dist=("normal", 1.0), bias_dist=("normal", 0.3), bias_dtype=wl.F32, act=wl.ACT_GELU_TANH,
                 lda=K + 4, ldb=(K if tb else N) + 12, ldc=N + 5)
    inp = wl.make_inputs(cfg, 80 + M)
    ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
    for s in (1, 2, 5):
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, s)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        assert (kernel, variant) == (lg.GEMM_KERNEL_SKINNY, 2 + tb) and split <= s
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"fp32 streaming M={M} tb={tb} split {s}")
    # integer data: unique answer, whatever the split; agrees with the fp32 tiles
    icfg = cfg_of(M, 264, 4096, 0, tb, wl.F32, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
    iinp, _ = wl.make_integer_inputs(icfg, 17, -3, 3)
    want = oracle.decode(wl.F32, expected_bits_exact(icfg, iinp))
    for plan in [(lg.GEMM_KERNEL_SKINNY, -1, 0), (lg.GEMM_KERNEL_SKINNY, -1, 1), (lg.GEMM_KERNEL_SKINNY, -1, 4),
                 (lg.GEMM_KERNEL_MFMA_TILE, -1, 0)]:
        lg.gemm_set_plan(handle, *plan)
        p = DeviceProblem(icfg, iinp)
        p.run(handle)
        assert np.array_equal(decode_c(icfg, p.result_bits()), want), plan
    lg.gemm_set_plan(handle)


def test_f32_streaming_refusals_and_automatic_choice(handle):
    # more than 8 rows, an A stored K x M, or a K that is no multiple of 4 are not for these kernels
    for (M, N, K, ta) in [(9, 1024, 1024, 0), (4, 1024, 1024, 1), (4, 1024, 1022, 0)]:
        cfg = cfg_of(M, N, K, ta, 0, wl.F32)
        p = DeviceProblem(cfg, wl.make_inputs(cfg, 3))
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, 1)
        assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)
    # the automatic plan streams a matrix-vector product on a weight of 16 MiB or more
    cfg = cfg_of(1, 2048, 2048, 0, 1, wl.F32)
    inp = wl.make_inputs(cfg, 4)
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    assert lg.gemm_get_last_plan(handle)[:2] == (lg.GEMM_KERNEL_SKINNY, 3)
    ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
    assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, "fp32 matrix-vector product, automatic")
    small = cfg_of(1, 512, 512, 0, 0, wl.F32)
    q = DeviceProblem(small, wl.make_inputs(small, 5))
    q.run(handle)
    assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_MFMA_TILE


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 8])
def test_vector_alu_kernel_for_a_16_bit_weight_stored_n_by_k(handle, M, dtype):
    """Variant 4 of the streaming family (at most 8 rows, B stored N x K, the sums on the vector ALUs): ragged last
    group of columns (1048 = 65 * 16 + 8), a K that is no multiple of a trip of 512, padded leading dimensions, every
    epilogue term, and a split of k through the reduction kernel."""
    N, K = 1048, 2072
    cfg = cfg_of(M, N, K, 0, 1, dtype, alpha=0.5, beta=-1.5, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                 c_dist=("normal", 1.0), bias_dist=("normal", 0.3), bias_dtype=wl.F32, act=wl.ACT_GELU_TANH,
                 lda=K + 8, ldb=K + 24, ldc=N + 5)
    inp = wl.make_inputs(cfg, 90 + M)
    # what lies behind the last k of a stored row must not reach the sums: NaN in the padding of both operands
    nan16 = np.uint16(0x7fc0 if dtype == wl.BF16 else 0x7e00)
    inp["A"].reshape(M, K + 8)[:, K:] = nan16
    inp["B"].reshape(N, K + 24)[:, K:] = nan16
    ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
    assert np.isfinite(ref).all()
    for s in (1, 2, 5):
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 4, s)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        assert (kernel, variant) == (lg.GEMM_KERNEL_SKINNY, 4) and split <= s
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"16-bit vector-ALU kernel M={M} split {s}")
        first = p.result_bits().copy()
        p.reset_c()
        p.run(handle)
        assert np.array_equal(first.view(np.uint8), p.result_bits().view(np.uint8)), "two runs differ"
    # integer data: a unique answer, whatever the kernel and the split; short and long k, fp32 and 16-bit C
    for (n, k, out) in [(264, 4096, wl.F32), (40, 8, dtype), (8, 520, wl.F32), (4104, 1032, dtype)]:
        icfg = cfg_of(M, n, k, 0, 1, dtype, out, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
        iinp, _ = wl.make_integer_inputs(icfg, 17, -3, 3)
        want = oracle.decode(out, expected_bits_exact(icfg, iinp))
        for plan in [(lg.GEMM_KERNEL_SKINNY, 4, 0), (lg.GEMM_KERNEL_SKINNY, 4, 1), (lg.GEMM_KERNEL_SKINNY, 4, 3),
                     (lg.GEMM_KERNEL_SKINNY, 1, 0), (0, -1, 0)]:
            lg.gemm_set_plan(handle, *plan)
            p = DeviceProblem(icfg, iinp)
            p.run(handle)
            assert np.array_equal(decode_c(icfg, p.result_bits()), want), (n, k, plan)
    lg.gemm_set_plan(handle)


def test_vector_alu_kernel_refusals_and_automatic_choice(handle):
    # more than 8 rows, an A stored K x M, a row-major B, or a K that is no multiple of 8 are not for variant 4
    for (M, N, K, ta, tb) in [(9, 1024, 1024, 0, 1), (4, 1024, 1024, 1, 1), (4, 1024, 1024, 0, 0), (4, 1024, 1020, 0, 1)]:
        cfg = cfg_of(M, N, K, ta, tb, wl.BF16)
        p = DeviceProblem(cfg, wl.make_inputs(cfg, 3))
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 4, 1)
        assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)
    # the automatic plan: up to four rows on a weight stored N x K take it at every size, more rows do not
    for (M, N, K, expect) in [(1, 4096, 4096, True), (4, 512, 512, True), (1, 8192, 8192, True), (5, 4096, 4096, False)]:
        cfg = cfg_of(M, N, K, 0, 1, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.03))
        inp = wl.make_inputs(cfg, 4)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        kernel, variant, _ = lg.gemm_get_last_plan(handle)
        assert ((kernel, variant) == (lg.GEMM_KERNEL_SKINNY, 4)) == expect, (M, N, K)
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"automatic plan {M}x{N}x{K}")


@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
@pytest.mark.parametrize("N", [1048, 4360])
@pytest.mark.parametrize("M", [1, 5, 8, 13, 16])
def test_mfma_kernel_with_16_columns_per_workgroup(handle, M, N, dtype):
    """Variant 5 of the streaming family (B stored N x K, at most 16 rows, one block of 16 columns per workgroup whose
    waves share the k range), with four visits in flight per wave (N <= 4096) and with two: a ragged last block
    (1048 = 65 * 16 + 8, 4360 = 272 * 16 + 8), a K that is no multiple of a chunk of 256 and gives the four waves 3, 2, 2
    and 2 chunks, padded leading dimensions with NaN behind every row, every epilogue term, and slices of k through
    the reduction kernel."""
    K = 2072
    cfg = cfg_of(M, N, K, 0, 1, dtype, alpha=0.5, beta=-1.5, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                 c_dist=("normal", 1.0), bias_dist=("normal", 0.3), bias_dtype=wl.F32, act=wl.ACT_GELU_TANH,
                 lda=K + 8, ldb=K + 24, ldc=N + 5)
    inp = wl.make_inputs(cfg, 120 + M)
    nan16 = np.uint16(0x7fc0 if dtype == wl.BF16 else 0x7e00)
    inp["A"].reshape(M, K + 8)[:, K:] = nan16
    inp["B"].reshape(N, K + 24)[:, K:] = nan16
    ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
    assert np.isfinite(ref).all()
    for s in (1, 2):
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 5, s)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        assert (kernel, variant) == (lg.GEMM_KERNEL_SKINNY, 5) and split <= s
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"16-column MFMA kernel M={M} split {s}")
        first = p.result_bits().copy()
        p.reset_c()
        p.run(handle)
        assert np.array_equal(first.view(np.uint8), p.result_bits().view(np.uint8)), "two runs differ"
    # integer data: a unique answer, whatever the kernel and the split; one chunk, fewer chunks than waves, many
    for (n, k, out) in [(264, 4096, wl.F32), (40, 8, dtype), (24, 520, wl.F32), (4104, 1032, dtype), (4096, 8192, wl.F32), (6152, 4360, dtype)]:
        icfg = cfg_of(M, n, k, 0, 1, dtype, out, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
        iinp, _ = wl.make_integer_inputs(icfg, 19, -3, 3)
        want = oracle.decode(out, expected_bits_exact(icfg, iinp))
        for plan in [(lg.GEMM_KERNEL_SKINNY, 5, 0), (lg.GEMM_KERNEL_SKINNY, 5, 1), (lg.GEMM_KERNEL_SKINNY, 5, 3),
                     (lg.GEMM_KERNEL_SKINNY, 1, 0), (0, -1, 0)]:
            lg.gemm_set_plan(handle, *plan)
            p = DeviceProblem(icfg, iinp)
            p.run(handle)
            assert np.array_equal(decode_c(icfg, p.result_bits()), want), (n, k, plan)
    lg.gemm_set_plan(handle)


def test_mfma_kernel_with_16_columns_refusals_and_automatic_choice(handle):
    # more than 16 rows, a row-major B or fp32 operands are not for variant 5
    for (M, N, K, tb, dtype) in [(17, 1024, 2048, 1, wl.BF16), (8, 1024, 2048, 0, wl.BF16), (8, 1024, 2048, 1, wl.F32)]:
        cfg = cfg_of(M, N, K, 0, tb, dtype)
        p = DeviceProblem(cfg, wl.make_inputs(cfg, 3))
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 5, 1)
        assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)
    for (M, N, K, expect) in [(8, 4096, 4096, True), (16, 2048, 4096, True), (17, 4096, 4096, False), (8, 8192, 4096, True), (8, 8192, 512, False)]:
        cfg = cfg_of(M, N, K, 0, 1, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.03))
        inp = wl.make_inputs(cfg, 4)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        kernel, variant, _ = lg.gemm_get_last_plan(handle)
        assert ((kernel, variant) == (lg.GEMM_KERNEL_SKINNY, 5)) == expect, (M, N, K)
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"automatic plan {M}x{N}x{K}")

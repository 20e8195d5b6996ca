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

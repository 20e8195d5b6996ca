"""GPU parity of the persistent short-k tile kernel (K <= 128 in whole 32-wide slabs, C write-only):
every layout, input and output type, ragged M and N,
activations, strided batches, and grids with several tiles per workgroup, which is where its pipeline across tiles runs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import BatchedDeviceProblem, DeviceProblem, assert_close, decode_c, expected_bits_exact, oracle_problem

pytestmark = pytest.mark.gpu

SHORTK = next(v for v in range(64) if (lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, v) or "").startswith("shortk"))


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    torch.cuda.synchronize()
    lg.gemm_destroy(h)


def cfg_of(M, N, K, ta, tb, dtype, out, **kw):
    return wl.Config("shortk", M, N, K, ta, tb, dtype, out, **kw)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
@pytest.mark.parametrize("K", [32, 64, 96, 128])
def test_shortk_layouts_types_and_epilogues(handle, ta, tb, K):
    # 5 x 4 tiles with ragged last row and column of tiles; padded leading dimensions
    M, N = 520, 392
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, SHORTK, 1)
    try:
        for dtype, out, act, bias in [(wl.BF16, wl.BF16, wl.ACT_NONE, None), (wl.F16, wl.F16, wl.ACT_GELU_ERF, None),
                                      (wl.BF16, wl.F32, wl.ACT_SILU, None)]:
            cfg = cfg_of(M, N, K, ta, tb, dtype, out, alpha=0.75, a_dist=("normal", 1.0), b_dist=("normal", 0.3), bias_dist=bias,
                         bias_dtype=wl.F32, act=act, lda=(M if ta else K) + 8, ldb=(K if tb else N) + 16, ldc=N + 8)
            inp = wl.make_inputs(cfg, 300 + K)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, SHORTK, 1)
            ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
            assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"shortk K={K} {ta}{tb} out={out}")
            # the padding columns of C stay as they were (NaN fill of a write-only C)
            pad = p.result_bits()[:-1, cfg.N:]
            assert np.all(np.isnan(oracle.decode(out, np.ascontiguousarray(pad))))
    finally:
        lg.gemm_set_plan(handle)


@pytest.mark.parametrize("tb", [1, 0])
def test_shortk_many_tiles_per_workgroup_integer_exact(handle, tb):
    # 3 x 17 x 17 = 867 tiles: up to four per workgroup on 256 compute units; integer data, unique answer
    cfg = cfg_of(2176, 2176, 64, 0, tb, wl.BF16, wl.BF16, alpha=1.0)
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, SHORTK, 1)
    try:
        p = BatchedDeviceProblem(cfg, 3, cfg.stride_a() + 8, cfg.stride_b(), cfg.stride_c() + 16, seed=21, integer=True)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle)[:2] == (lg.GEMM_KERNEL_MFMA_TILE, SHORTK)
        p.check("shortk, several tiles per workgroup", exact=True)
        first = wl.torch_to_bits(p.C).copy()
        p.run(handle)
        torch.cuda.synchronize()
        assert np.array_equal(first.view(np.uint8), wl.torch_to_bits(p.C).view(np.uint8)), "two runs differ"
    finally:
        lg.gemm_set_plan(handle)


@pytest.mark.parametrize("K,ta,tb,out", [(128, 0, 1, wl.BF16), (96, 0, 0, wl.F32), (64, 1, 1, wl.F16), (32, 1, 0, wl.BF16), (128, 0, 1, wl.F32), (32, 0, 0, wl.F32)])
def test_shortk_runs_of_tiles_with_ragged_edges(handle, K, ta, tb, out):
    # 6 x 17 x 17 = 1734 tiles on 512 workgroups: runs of four tiles that cross the ragged last row of tiles
    # (fewer stores than a whole tile), the end of a column of tiles (B changes) and the end of a matrix;
    # integer data, unique answer in every output type
    M, N = 2104, 2088
    dtype = wl.F16 if out == wl.F16 else wl.BF16
    cfg = cfg_of(M, N, K, ta, tb, dtype, out, alpha=1.0, lda=(M if ta else K) + 8, ldb=(K if tb else N) + 8, ldc=N + 8)
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, SHORTK, 1)
    try:
        p = BatchedDeviceProblem(cfg, 6, cfg.stride_a() + 8, cfg.stride_b() + 16, cfg.stride_c() + 8, seed=51 + K, integer=True)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle)[:2] == (lg.GEMM_KERNEL_MFMA_TILE, SHORTK)
        p.check(f"shortk, runs with edges K={K} {ta}{tb} out={out}", exact=True)
    finally:
        lg.gemm_set_plan(handle)


def test_shortk_refusals_and_automatic_choice(handle):
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, SHORTK, 1)
    try:
        for cfg in (cfg_of(256, 256, 160, 0, 1, wl.BF16, wl.BF16),                              # five slabs
                    cfg_of(256, 256, 72, 0, 1, wl.BF16, wl.BF16),                               # a partial slab
                    cfg_of(256, 256, 64, 0, 1, wl.BF16, wl.BF16, beta=1.0),                     # C is read
                    cfg_of(256, 256, 64, 0, 1, wl.BF16, wl.BF16, bias_dist=("normal", 1.0)),    # a bias
                    cfg_of(256, 256, 64, 0, 1, wl.BF16, wl.BF16, ldc=259)):                     # rows of C off 16-byte boundaries
            p = DeviceProblem(cfg, wl.make_inputs(cfg, 1))
            assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED, cfg
    finally:
        lg.gemm_set_plan(handle)
    # the automatic plan takes it for a batch of short products with a tile or more per compute unit ...
    cfg = cfg_of(1024, 1024, 128, 0, 1, wl.BF16, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.1))
    p = BatchedDeviceProblem(cfg, 8, cfg.stride_a(), cfg.stride_b(), cfg.stride_c(), seed=33)
    p.run(handle)
    assert lg.gemm_get_last_plan(handle)[:2] == (lg.GEMM_KERNEL_MFMA_TILE, SHORTK)
    p.check("shortk, automatic")
    # ... and not when C is read
    cfg2 = cfg_of(1024, 1024, 128, 0, 1, wl.BF16, wl.BF16, beta=1.0, a_dist=("normal", 1.0), b_dist=("normal", 0.1))
    q = BatchedDeviceProblem(cfg2, 8, cfg2.stride_a(), cfg2.stride_b(), cfg2.stride_c(), seed=34)
    q.run(handle)
    assert lg.gemm_get_last_plan(handle)[1] != SHORTK
    q.check("short products with beta, automatic")

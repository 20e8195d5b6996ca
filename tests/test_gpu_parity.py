"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle, element by
element on seeded inputs at sizes the oracle finishes in seconds.  Shapes span several macro
tiles and leave ragged tails in every dimension."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import (BatchedDeviceProblem, DeviceProblem, assert_close, c_bits_as_uint, check_full, decode_c,
                         expected_bits_exact, oracle_problem, stream_ptr)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    torch.cuda.synchronize()
    lg.gemm_destroy(h)


def base_cfg(M, N, K, ta, tb, dtype=wl.BF16, out=None, **kw):
    return wl.Config("t", M, N, K, ta, tb, dtype, dtype if out is None else out, **kw)


def all_tile_variants():
    n = 0
    while lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, n) is not None:
        n += 1
    return n


def tile_variants(f32=False, every=False):
    """Indices of the tile variants for 16-bit (default) or fp32 operands that take any shape (the persistent
    short-k kernel has tests of its own).  Unless `every` is set, only the variants an automatic plan can pick:
    the older pipelines (variants 1, 2, 4, 6, 7, 8) are kept as alternatives for forced plans and run in the
    integer-exact test alone."""
    names = [lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, v) for v in range(all_tile_variants())]
    picked = [v for v, n in enumerate(names) if n.startswith("f32_") == f32 and not n.startswith("shortk")]
    return picked if every or f32 else [v for v in picked if v not in (1, 2, 4, 6, 7, 8)]


# ------------------------------------------------------------------ C1: the fp32 parity configuration

def test_c1_fp32_full_matrix(handle):
    cfg = wl.CONFIGS["C1"]
    inp = wl.make_inputs(cfg)
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    check_full(cfg, inp, p.result_bits(), "C1")


# ------------------------------------------------------------------ macro-tile kernels, every variant

@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_tile_variants_gaussian(handle, ta, tb, dtype):
    # 3 x 3 tiles of 256 with ragged tails; K leaves a masked partial slab (K % 64 = 40)
    M, N, K = 520, 584, 424
    for out in (dtype, wl.F32):
        cfg = base_cfg(M, N, K, ta, tb, dtype, out, a_dist=("normal", 1.0), b_dist=("normal", 0.5))
        inp = wl.make_inputs(cfg, 31 + ta * 2 + tb)
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        for v in tile_variants():
            print(f"tile variant {v} ta={ta} tb={tb} dtype={dtype} out={out}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            assert lg.gemm_get_last_plan(handle)[:2] == (lg.GEMM_KERNEL_MFMA_TILE, v)
            assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"variant {v}")
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
def test_tile_variants_integer_exact(handle, ta, tb):
    # integer entries: every partial sum is exact in fp32, the answer is unique -> equal values required
    M, N, K = 264, 776, 1096
    for out in (wl.BF16, wl.F32):
        cfg = base_cfg(M, N, K, ta, tb, wl.BF16, out, alpha=2.0, beta=-1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32,
                       lda=(M if ta else K) + 8, ldb=(K if tb else N) + 16, ldc=N + 3)
        inp, _ = wl.make_integer_inputs(cfg, 77, -2, 2)
        want = oracle.decode(out, expected_bits_exact(cfg, inp))
        for v in tile_variants(every=True):
            print(f"integer tile variant {v} ta={ta} tb={tb} out={out}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            got = decode_c(cfg, p.result_bits())
            assert np.array_equal(got, want), f"variant {v}: {np.sum(got != want)} wrong elements"
            # the padding columns of C (ldc > N) must be untouched
            pad_got = p.result_bits()[:-1, cfg.N:]
            pad_want = inp["C"].reshape(M, cfg.ld_c())[:-1, cfg.N:]
            assert np.array_equal(pad_got, pad_want)
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0)])
def test_tile_variants_every_small_slab_count(handle, ta, tb):
    # 1 .. 13 k slabs of 32 (and the matching counts of 64), with and without a partial last slab:
    # every entry into and exit from the software pipelines, whatever their depth
    M, N = 72, 136
    for K in (16, 32, 40, 64, 96, 104, 128, 160, 168, 192, 224, 256, 264, 288, 320, 352, 384, 416):
        cfg = base_cfg(M, N, K, ta, tb, wl.BF16, wl.F32, alpha=1.0, beta=0.0)
        inp, _ = wl.make_integer_inputs(cfg, 100 + K, -2, 2)
        want = oracle.decode(wl.F32, expected_bits_exact(cfg, inp))
        for v in tile_variants():
            print(f"slab-count sweep K={K} variant {v} ta={ta} tb={tb}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            got = decode_c(cfg, p.result_bits())
            assert np.array_equal(got, want), f"K={K} variant {v}: {np.sum(got != want)} wrong elements"
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 1), (1, 0)])
@pytest.mark.parametrize("dtype", [wl.BF16, wl.F16])
def test_whole_tiles_without_epilogue_terms(handle, ta, tb, dtype):
    # C = alpha * A * B on whole tiles (beta = 0, no bias, no activation): the direct-to-LDS kernels with the
    # 32x32x16 MFMA then store straight from the accumulator layout, 16-bit results two to a 32-bit word after
    # a trade between neighbouring lanes.  Integer data -> every element exact, in each output type; a C whose
    # rows start on odd elements takes the staged epilogue instead and must agree.
    M, N, K = 512, 768, 200
    for out in (dtype, wl.F32):
        for ldc in (N, N + 6, N + 3):
            cfg = base_cfg(M, N, K, ta, tb, dtype, out, alpha=-3.0, ldc=ldc)
            inp, _ = wl.make_integer_inputs(cfg, 87, -3, 3)
            want = oracle.decode(out, expected_bits_exact(cfg, inp))
            for v in tile_variants():
                print(f"whole tiles variant {v} ta={ta} tb={tb} dtype={dtype} out={out} ldc={ldc}", flush=True)
                lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
                p = DeviceProblem(cfg, inp)
                p.run(handle)
                got = decode_c(cfg, p.result_bits())
                assert np.array_equal(got, want), f"variant {v}: {np.sum(got != want)} wrong elements"
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
def test_tile_split_of_the_trailing_round(handle, ta, tb):
    # nine 256x256 tiles, fewer than compute units: a forced split cuts every tile's k range into shares
    # whose fp32 partial tiles a second kernel adds (in order) before the epilogue; integer data -> exact.
    # K = 1096 leaves a partial last slab in the last share; parts = 5 gives shares of unequal length,
    # parts = 64 more shares than the 35 slabs (clamped)
    M, N, K = 520, 584, 1096
    cfg = base_cfg(M, N, K, ta, tb, wl.BF16, wl.BF16, alpha=2.0, beta=-1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32,
                   act=wl.ACT_RELU, ldc=N + 5)
    inp, _ = wl.make_integer_inputs(cfg, 78, -2, 2)
    want = oracle.decode(wl.BF16, expected_bits_exact(cfg, inp))
    splitting = [v for v in tile_variants() if "dma16" in lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, v)]
    assert splitting
    for v in splitting:
        for parts in (2, 5, 64):
            print(f"split variant {v} parts {parts} ta={ta} tb={tb}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v, parts)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            kernel, variant, used = lg.gemm_get_last_plan(handle)
            assert (kernel, variant) == (lg.GEMM_KERNEL_MFMA_TILE, v) and used == min(parts, 35)
            got = decode_c(cfg, p.result_bits())
            assert np.array_equal(got, want), f"variant {v} parts {parts}: {np.sum(got != want)} wrong elements"
            pad_got = p.result_bits()[:-1, cfg.N:]
            assert np.array_equal(pad_got, inp["C"].reshape(M, cfg.ld_c())[:-1, cfg.N:])
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
def test_tile_k_slices(handle, ta, tb):
    # Every tile variant without the split above cuts K into slices instead: consecutive ranges of whole
    # slabs, computed side by side into fp32 partial results that a second kernel adds in order before the
    # epilogue.  Integer data -> exact.  K = 1096: 35 slabs, the last one partial; 3 slices of 12 / 12 / 11
    # slabs, 16 slices of 3 / ... / 2 (12 ranges in all), 64 -> one slab each (35).  Edge tiles in both
    # directions, padded ldc whose padding must stay untouched.
    M, N, K = 392, 328, 1096
    cfg = base_cfg(M, N, K, ta, tb, wl.BF16, wl.BF16, alpha=2.0, beta=-1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32,
                   act=wl.ACT_RELU, ldc=N + 5)
    inp, _ = wl.make_integer_inputs(cfg, 81, -2, 2)
    want = oracle.decode(wl.BF16, expected_bits_exact(cfg, inp))
    slicing = [v for v in tile_variants() if "dma16" not in lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, v)]
    assert slicing
    for v in slicing:
        for slices, used_want in ((3, 3), (16, 12), (64, 35)):
            print(f"k slices variant {v} slices {slices} ta={ta} tb={tb}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v, slices)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, v, used_want)
            got = decode_c(cfg, p.result_bits())
            assert np.array_equal(got, want), f"variant {v} slices {slices}: {np.sum(got != want)} wrong elements"
            pad_got = p.result_bits()[:-1, cfg.N:]
            assert np.array_equal(pad_got, inp["C"].reshape(M, cfg.ld_c())[:-1, cfg.N:])
    lg.gemm_set_plan(handle)


def test_tile_k_slices_fp32_refusals_and_automatic_choice(handle):
    # fp32 tile kernels slice the same way (Gaussian data to the fp32 tolerance, integer data exactly)
    for v in tile_variants(f32=True):
        cfg = base_cfg(200, 264, 1000, 0, 1, wl.F32, wl.F32, alpha=0.5, beta=2.0, a_dist=("normal", 1.0), b_dist=("normal", 0.5),
                       c_dist=("normal", 1.0), bias_dist=("normal", 1.0), bias_dtype=wl.F32, act=wl.ACT_GELU_TANH)
        inp = wl.make_inputs(cfg, 82)
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v, 5)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, v, 5)
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"fp32 k slices variant {v}")
    # slices need N to be a multiple of 8 (the adding kernel works on groups of 8 columns), and one matrix
    cfg = base_cfg(256, 132, 1024, 0, 1, wl.BF16, wl.F32, beta=1.0)
    inp, _ = wl.make_integer_inputs(cfg, 83, -2, 2)
    before = inp["C"].copy()
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, 5, 4)
    p = DeviceProblem(cfg, inp)
    assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    assert np.array_equal(p.result_bits().reshape(-1), before.reshape(-1))
    lg.gemm_set_plan(handle)
    # automatic choice: 16 tiles of 128 x 128 with a long k loop are sliced; exact on integer data,
    # within the bounds on Gaussian data, the same bits on a second run
    cfg = base_cfg(512, 512, 4096, 0, 0, wl.BF16, wl.BF16, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.BF16)
    inp, _ = wl.make_integer_inputs(cfg, 84, -1, 1)
    want = oracle.decode(wl.BF16, expected_bits_exact(cfg, inp))
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    kernel, variant, slices = lg.gemm_get_last_plan(handle)
    assert kernel == lg.GEMM_KERNEL_MFMA_TILE and slices > 1
    assert "dma16" not in lg.gemm_variant_name(kernel, variant)
    assert np.array_equal(decode_c(cfg, p.result_bits()), want)
    gcfg = base_cfg(512, 512, 4096, 0, 1, wl.BF16, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.05))
    ginp = wl.make_inputs(gcfg, 85)
    gref, _, gmag = oracle.gemm_full(oracle_problem(gcfg, ginp), want_bounds=True)
    g = DeviceProblem(gcfg, ginp)
    g.run(handle)
    first = g.result_bits().copy()
    assert lg.gemm_get_last_plan(handle)[2] > 1
    assert_close(gcfg, decode_c(gcfg, first), gref, gmag, "automatic k slices")
    g2 = DeviceProblem(gcfg, ginp)
    g2.run(handle)
    assert np.array_equal(first, g2.result_bits())
    # fp32 operands: a few tiles with a long k loop are sliced as well; integer data -> exact
    fcfg = base_cfg(256, 264, 8192, 1, 0, wl.F32, wl.F32, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
    finp, _ = wl.make_integer_inputs(fcfg, 88, -2, 2)
    fwant = oracle.decode(wl.F32, expected_bits_exact(fcfg, finp))
    f = DeviceProblem(fcfg, finp)
    f.run(handle)
    kernel, variant, slices = lg.gemm_get_last_plan(handle)
    assert kernel == lg.GEMM_KERNEL_MFMA_TILE and slices > 1 and lg.gemm_variant_name(kernel, variant).startswith("f32_")
    assert np.array_equal(decode_c(fcfg, f.result_bits()), fwant)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
def test_tile_split_with_rotated_k_walk(handle, ta, tb):
    # K = 2048 in whole slabs and rows of the k-contiguous operands 4096 bytes apart: a split call
    # then walks k from a different slab in every workgroup and wraps around.  Integer data -> the
    # order of the sum does not show, every element is exact; Gaussian data within the bounds.
    M, N, K = 520, 584, 2048
    cfg = base_cfg(M, N, K, ta, tb, wl.BF16, wl.F32, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
    inp, _ = wl.make_integer_inputs(cfg, 79, -2, 2)
    want = oracle.decode(wl.F32, expected_bits_exact(cfg, inp))
    gcfg = base_cfg(M, N, K, ta, tb, wl.BF16, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.05))
    ginp = wl.make_inputs(gcfg, 80)
    gref, _, gmag = oracle.gemm_full(oracle_problem(gcfg, ginp), want_bounds=True)
    splitting = [v for v in tile_variants() if "dma16" in lg.gemm_variant_name(lg.GEMM_KERNEL_MFMA_TILE, v)]
    for v in splitting:
        for parts in (2, 3, 4, 7):       # 3 and 7: odd slab counts in some shares (those walk unrotated)
            print(f"rotated split variant {v} parts {parts} ta={ta} tb={tb}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v, parts)
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, v, parts)
            got = decode_c(cfg, p.result_bits())
            assert np.array_equal(got, want), f"variant {v} parts {parts}: {np.sum(got != want)} wrong elements"
            g = DeviceProblem(gcfg, ginp)
            g.run(handle)
            assert_close(gcfg, decode_c(gcfg, g.result_bits()), gref, gmag, f"rotated split variant {v} parts {parts}")
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 1), (0, 0), (1, 1), (1, 0)])
def test_f32_tile_variants(handle, ta, tb):
    # fp32 operands on the fp32 matrix instruction: 3 x 5 tiles of 128 with ragged tails, K leaves a partial slab
    # (K % 16 = 12); Gaussian data to the fp32 tolerance, integer data exactly; wrong operand type is refused
    assert tile_variants(f32=True)
    M, N, K = 300, 520, 172
    for v in tile_variants(f32=True):
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
        cfg = base_cfg(M, N, K, ta, tb, wl.F32, wl.F32, alpha=0.5, beta=2.0, a_dist=("normal", 1.0), b_dist=("normal", 0.5),
                       c_dist=("normal", 1.0), bias_dist=("normal", 1.0), bias_dtype=wl.F32, act=wl.ACT_GELU_TANH,
                       lda=(M if ta else K) + 4, ldb=(K if tb else N) + 8, ldc=N + 1)
        inp = wl.make_inputs(cfg, 61 + 2 * ta + tb)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle)[:2] == (lg.GEMM_KERNEL_MFMA_TILE, v)
        check_full(cfg, inp, p.result_bits(), f"f32 variant {v}")
        cfg = base_cfg(M, N, K, ta, tb, wl.F32, wl.F32, alpha=3.0, beta=-1.0)
        inp, _ = wl.make_integer_inputs(cfg, 62, -3, 3)
        want = oracle.decode(wl.F32, expected_bits_exact(cfg, inp))
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        assert np.array_equal(decode_c(cfg, p.result_bits()), want)
        # a 16-bit problem cannot run on it, nor an fp32 problem on a 16-bit variant
        cfg16 = base_cfg(64, 64, 64, ta, tb, wl.BF16, wl.BF16)
        assert DeviceProblem(cfg16, wl.make_inputs(cfg16, 1)).run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, tile_variants()[0])
    cfg = base_cfg(64, 64, 64, ta, tb, wl.F32, wl.F32)
    assert DeviceProblem(cfg, wl.make_inputs(cfg, 1)).run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)


def test_f32_automatic_choice(handle):
    # aligned -> an fp32 tile kernel, whatever the size; unaligned -> general kernel
    big = base_cfg(512, 640, 64, 0, 0, wl.F32, wl.F32)
    small = base_cfg(256, 256, 256, 0, 0, wl.F32, wl.F32)
    tiny = base_cfg(24, 40, 12, 0, 1, wl.F32, wl.F32)
    odd = base_cfg(512, 642, 64, 0, 0, wl.F32, wl.F32)
    for cfg, family in ((big, lg.GEMM_KERNEL_MFMA_TILE), (small, lg.GEMM_KERNEL_MFMA_TILE), (tiny, lg.GEMM_KERNEL_MFMA_TILE),
                        (odd, lg.GEMM_KERNEL_GENERAL)):
        inp = wl.make_inputs(cfg, 8)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle)[0] == family
        check_full(cfg, inp, p.result_bits(), "f32 auto")


def test_tile_epilogue_bias_gelu_beta(handle):
    M, N, K = 300, 392, 256
    cfg = base_cfg(M, N, K, 0, 1, wl.BF16, wl.BF16, alpha=0.5, beta=1.5, a_dist=("normal", 1.0),
                   b_dist=("normal", 0.1), c_dist=("normal", 1.0), bias_dist=("normal", 0.5),
                   bias_dtype=wl.BF16, act=wl.ACT_GELU_ERF)
    inp = wl.make_inputs(cfg, 5)
    for v in tile_variants():
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        check_full(cfg, inp, p.result_bits(), f"epilogue variant {v}")
    lg.gemm_set_plan(handle)


def test_small_tile_problem_single_partial_slab(handle):
    # K smaller than one slab; M, N smaller than one tile
    cfg = base_cfg(40, 24, 8, 0, 1, wl.F16, wl.F16)
    inp = wl.make_inputs(cfg, 9)
    for v in tile_variants():
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        check_full(cfg, inp, p.result_bits(), f"tiny variant {v}")
    lg.gemm_set_plan(handle)


# ------------------------------------------------------------------ skinny split-K kernels (B row-major, B stored N x K)

@pytest.mark.parametrize("tb", [0, 1])
@pytest.mark.parametrize("M", [1, 5, 16, 17, 32, 33, 49, 64])
def test_skinny_gaussian_and_split_agreement(handle, M, tb):
    # 4 column groups with a ragged last one (776 = 3*256 + 8); K % 16 = 8 and K % 32 = 8 leave a
    # partly filled last step in either kernel; padded leading dimensions
    N, K = 776, 2056
    for dtype in (wl.BF16, wl.F16):
        cfg = base_cfg(M, N, K, 0, tb, dtype, dtype, alpha=1.0, beta=1.0, a_dist=("normal", 1.0),
                       b_dist=("normal", 0.02), c_dist=("normal", 1.0), lda=K + 8, ldb=(K if tb else N) + 24)
        inp = wl.make_inputs(cfg, 40 + M)
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        for s in (1, 2, 3, 8):
            print(f"skinny M={M} tb={tb} dtype={dtype} split={s}", flush=True)
            lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, tb, s)      # the MFMA kernel of the layout, also where few rows would go to the vector ALUs
            p = DeviceProblem(cfg, inp)
            p.run(handle)
            assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_SKINNY, tb, s)
            assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, f"skinny tb={tb} split {s}")
    # a variant forced against the layout of the call is refused
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 1 - tb, 1)
    p = DeviceProblem(cfg, inp)
    assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("tb", [0, 1])
@pytest.mark.parametrize("out", [wl.BF16, wl.F32])
@pytest.mark.parametrize("M", [19, 57])
def test_skinny_integer_exact_all_splits_equal(handle, out, tb, M):
    N, K = 1032, 4104
    cfg = base_cfg(M, N, K, 0, tb, wl.BF16, out, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.BF16,
                   ldc=N + 8)
    inp, _ = wl.make_integer_inputs(cfg, 123, -1, 1)
    want = oracle.decode(out, expected_bits_exact(cfg, inp))
    for s in (0, 1, 2, 4, 7, 16):
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, s)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        got = decode_c(cfg, p.result_bits())
        assert np.array_equal(got, want), f"split {s}: {np.sum(got != want)} wrong"
    # the other kernel families agree bit for bit on integer data
    for kern in (lg.GEMM_KERNEL_MFMA_TILE, lg.GEMM_KERNEL_GENERAL):
        lg.gemm_set_plan(handle, kern, -1 if kern == lg.GEMM_KERNEL_MFMA_TILE else 0)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        assert np.array_equal(decode_c(cfg, p.result_bits()), want)
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("tb", [0, 1])
def test_skinny_short_k_unaligned_c_and_stale_neighbours(handle, tb):
    # fewer steps than pipeline stages (K = 40), a C whose rows allow no vector access (ldc = 203),
    # bias and activation; B stored N x K is followed in memory by NaN (what lies behind the last
    # k of a row must not reach the sums), and the padding columns of C keep their contents
    for out in (wl.BF16, wl.F32):
        cfg = base_cfg(7, 200, 40, 0, tb, wl.BF16, out, alpha=0.5, beta=-1.0, a_dist=("normal", 1.0), b_dist=("normal", 1.0),
                       c_dist=("normal", 1.0), bias_dist=("normal", 1.0), bias_dtype=wl.F32, act=wl.ACT_SILU, ldc=203,
                       lda=48, ldb=(48 if tb else 208))
        inp = wl.make_inputs(cfg, 77)
        nan16 = np.uint16(0x7fc0)
        a2 = inp["A"].reshape(7, 48); a2[:, 40:] = nan16
        b2 = inp["B"].reshape(-1, cfg.ld_b()); b2[:, (40 if tb else 200):] = nan16
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inp), want_bounds=True)
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, 1)
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        bits = p.result_bits()
        assert_close(cfg, decode_c(cfg, bits), ref, mag, f"skinny short K tb={tb}")
        assert np.array_equal(bits[:-1, cfg.N:], inp["C"].reshape(cfg.M, cfg.ld_c())[:-1, cfg.N:])
    lg.gemm_set_plan(handle)


def test_skinny_fp16_gelu(handle):
    cfg = base_cfg(8, 512, 1024, 0, 0, wl.F16, wl.F16, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                   bias_dist=("normal", 0.5), bias_dtype=wl.F16, act=wl.ACT_GELU_ERF)
    inp = wl.make_inputs(cfg, 3)
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, -1, 0)      # a weight this small goes to the tile family by itself
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_SKINNY
    lg.gemm_set_plan(handle)
    check_full(cfg, inp, p.result_bits(), "skinny fp16 gelu")


@pytest.mark.parametrize("M,N,K,tb", [(8, 512, 1024, 0), (24, 512, 1024, 1), (32, 2048, 2048, 1), (40, 768, 2048, 1), (64, 1024, 4096, 0)])
def test_few_rows_small_weight_automatic_choice(handle, M, N, K, tb):
    # the streaming kernels are for weights of 128 MiB and more; below that, and above 32 rows, the call goes
    # to the tile family (sliced along K where that fills the chip).  Integer data -> exact.
    cfg = base_cfg(M, N, K, 0, tb, wl.BF16, wl.BF16, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
    inp, _ = wl.make_integer_inputs(cfg, 86, -2, 2)
    want = oracle.decode(wl.BF16, expected_bits_exact(cfg, inp))
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_MFMA_TILE
    assert np.array_equal(decode_c(cfg, p.result_bits()), want)


@pytest.mark.parametrize("M,N,K,tb", [(128, 264, 40960, 0), (200, 520, 16392, 1)])
def test_long_k_on_few_tiles_takes_the_quarter_tile_with_its_split(handle, M, N, K, tb):
    # a handful of 128 x 128 tiles with k of 16384 or more: the 16x16x32 tile of that size, its one round cut
    # into shares along k (32 and 24 of them here, added up by the generic reduction), with partly filled tiles and
    # a k that ends inside a slab.  Integers -> exact.
    cfg = base_cfg(M, N, K, 0, tb, wl.BF16, wl.F32, alpha=1.0, beta=1.0, bias_dist=("normal", 1.0), bias_dtype=wl.F32)
    inp, _ = wl.make_integer_inputs(cfg, 87, -2, 2)
    print(f"long k {M}x{N}x{K}: oracle", flush=True)
    want = oracle.decode(wl.F32, expected_bits_exact(cfg, inp))
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    kernel, variant, shares = lg.gemm_get_last_plan(handle)
    assert kernel == lg.GEMM_KERNEL_MFMA_TILE and lg.gemm_variant_name(kernel, variant) == "dma16p_128x128x32_w2x2_s5" and shares > 1
    assert np.array_equal(decode_c(cfg, p.result_bits()), want)


def test_plan_query_agrees_with_the_plan_that_ran(handle):
    # the host-only query and the call itself go through the same choice
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for (M, N, K, ta, tb, dtype, out) in [(512, 512, 4096, 0, 0, wl.BF16, wl.BF16), (64, 1024, 4096, 0, 1, wl.F16, wl.F32),
                                          (300, 520, 192, 1, 1, wl.BF16, wl.BF16), (256, 264, 8192, 0, 0, wl.F32, wl.F32),
                                          (2048, 128, 2048, 0, 0, wl.BF16, wl.BF16), (37, 29, 53, 1, 0, wl.F32, wl.F32)]:
        cfg = base_cfg(M, N, K, ta, tb, dtype, out, a_dist=("normal", 1.0), b_dist=("normal", 0.05))
        p = DeviceProblem(cfg, wl.make_inputs(cfg, 89))
        p.run(handle)
        torch.cuda.synchronize()
        assert lg.gemm_get_last_plan(handle) == lg.gemm_plan_query(cus, 1, M, N, K, ta, tb, dtype, out, cfg.ld_a(), cfg.ld_b(), cfg.ld_c())


# ------------------------------------------------------------------ every activation through every kernel family

@pytest.mark.parametrize("act", [wl.ACT_RELU, wl.ACT_SILU, wl.ACT_GELU_TANH, wl.ACT_GELU_ERF])
def test_activations_in_every_kernel_family(handle, act):
    # pre-activation values of order 1 on both sides of zero (bias shifts a third of the columns far negative
    # and far positive, where the activations saturate)
    cases = [
        ("tile", base_cfg(300, 520, 192, 0, 1, wl.BF16, wl.BF16, alpha=0.25, beta=0.5, a_dist=("normal", 1.0),
                          b_dist=("normal", 0.3), c_dist=("normal", 1.0), bias_dist=("normal", 4.0), bias_dtype=wl.F32, act=act),
         lg.GEMM_KERNEL_MFMA_TILE),
        ("tile fp32 out", base_cfg(264, 264, 96, 0, 0, wl.F16, wl.F32, a_dist=("normal", 1.0), b_dist=("normal", 0.2),
                                   bias_dist=("normal", 2.0), bias_dtype=wl.F16, act=act), lg.GEMM_KERNEL_MFMA_TILE),
        ("skinny", base_cfg(8, 512, 1024, 0, 0, wl.BF16, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                            bias_dist=("normal", 2.0), bias_dtype=wl.BF16, act=act), lg.GEMM_KERNEL_SKINNY),
        ("skinny nt", base_cfg(24, 512, 1024, 0, 1, wl.F16, wl.F32, a_dist=("normal", 1.0), b_dist=("normal", 0.05),
                               bias_dist=("normal", 2.0), bias_dtype=wl.F32, act=act), lg.GEMM_KERNEL_SKINNY),
        ("general", base_cfg(37, 29, 53, 1, 0, wl.F32, wl.F32, bias_dist=("normal", 2.0), bias_dtype=wl.F32, act=act),
         lg.GEMM_KERNEL_GENERAL),
    ]
    for name, cfg, family in cases:
        inp = wl.make_inputs(cfg, 40 + act)
        if family == lg.GEMM_KERNEL_SKINNY:
            lg.gemm_set_plan(handle, family, -1, 0)      # small weights: forced, the automatic choice is the tile family
        p = DeviceProblem(cfg, inp)
        p.run(handle)
        lg.gemm_set_plan(handle)
        assert lg.gemm_get_last_plan(handle)[0] == family, name
        check_full(cfg, inp, p.result_bits(), f"{name} act {act}")


def test_relu_keeps_nan_and_is_exact(handle):
    # integer data: the pre-activation values are exact, so ReLU's output is unique
    cfg = base_cfg(264, 520, 160, 0, 1, wl.BF16, wl.F32, alpha=1.0, beta=0.0, act=wl.ACT_RELU)
    inp, _ = wl.make_integer_inputs(cfg, 5, -3, 3)
    want = oracle.decode(wl.F32, expected_bits_exact(cfg, inp))
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    got = decode_c(cfg, p.result_bits())
    assert np.array_equal(got, want) and (want == 0).mean() > 0.3 and (want > 0).mean() > 0.3


def test_unknown_activation_is_rejected(handle):
    cfg = base_cfg(64, 64, 64, 0, 1)
    inp = wl.make_inputs(cfg, 1)
    p = DeviceProblem(cfg, inp)
    epi = lg.make_epilogue(cfg.out_dtype, act=9)
    st = lg.gemm_run(handle, cfg.M, cfg.N, cfg.K, 0, 1, cfg.dtype, 1.0, p.A.data_ptr(), cfg.ld_a(), p.B.data_ptr(), cfg.ld_b(),
                     0.0, p.C.data_ptr(), cfg.ld_c(), epi, stream_ptr(), check=False)
    assert st == lg.GEMM_ERR_INVALID_ARG


# ------------------------------------------------------------------ general kernel: any shape, any alignment

@pytest.mark.parametrize("dtype", [wl.F32, wl.F16, wl.BF16])
def test_edge_shapes_through_the_boundary(handle, dtype):
    rng = np.random.default_rng(17)
    sizes = [1, 7, 31, 33, 255, 257]
    combos = [(1, 1, 1), (7, 33, 31), (33, 7, 257), (255, 31, 7), (257, 1, 33), (1, 257, 255), (31, 255, 1)]
    for (M, N, K) in combos:
        assert M in sizes and N in sizes and K in sizes
        ta, tb = int(rng.integers(2)), int(rng.integers(2))
        cfg = base_cfg(M, N, K, ta, tb, dtype, dtype, alpha=1.25, beta=0.5, c_dist=("normal", 1.0),
                       bias_dist=("normal", 1.0), bias_dtype=dtype,
                       lda=(M if ta else K) + 3, ldb=(K if tb else N) + 1, ldc=N + 2)
        inp = wl.make_inputs(cfg, 1000 + M + N + K)
        p = DeviceProblem(cfg, inp, a_offset_elems=1, b_offset_elems=1)     # base pointers off by one element
        p.run(handle)
        assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_GENERAL
        check_full(cfg, inp, p.result_bits(), f"edge {M}x{N}x{K} ta={ta} tb={tb}")


def test_general_kernel_matches_on_aligned_shape(handle):
    cfg = base_cfg(136, 264, 512, 0, 0, wl.BF16, wl.F32)
    inp = wl.make_inputs(cfg, 2)
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_GENERAL, 0)
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    lg.gemm_set_plan(handle)
    check_full(cfg, inp, p.result_bits(), "general")


# ------------------------------------------------------------------ degenerate cases of the definition

def test_empty_sum_and_zero_alpha(handle):
    M, N = 37, 53
    # K = 0: C = act(beta*C + bias)
    cfg = base_cfg(M, N, 0, 0, 0, wl.BF16, wl.BF16, beta=2.0, c_dist=("normal", 1.0), bias_dist=("normal", 1.0),
                   bias_dtype=wl.F32, act=wl.ACT_GELU_ERF, lda=8, ldb=N)
    inp = wl.make_inputs(cfg, 4)
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    check_full(cfg, inp, p.result_bits(), "K=0")
    # alpha = 0 with NaN in A: the product term is dropped altogether
    cfg = base_cfg(M, N, 64, 0, 0, wl.BF16, wl.BF16, alpha=0.0, beta=1.0, c_dist=("normal", 1.0))
    inp = wl.make_inputs(cfg, 6)
    inp_nan = dict(inp)
    inp_nan["A"] = wl.to_bits(np.full(inp["A"].shape, np.nan, np.float32), wl.BF16)
    p = DeviceProblem(cfg, inp_nan)
    p.run(handle)
    got = decode_c(cfg, p.result_bits())
    assert np.array_equal(got, oracle.decode(wl.BF16, inp["C"]).reshape(M, N))
    # M = 0 or N = 0: nothing happens, status OK
    ptr = p.A.data_ptr()
    assert lg.gemm_run(handle, 0, N, 8, 0, 0, wl.BF16, 1.0, 0, 8, ptr, N, 0.0, 0, N, None, stream_ptr()) == lg.GEMM_OK
    assert lg.gemm_run(handle, M, 0, 8, 0, 0, wl.BF16, 1.0, ptr, 8, 0, 1, 0.0, 0, 1, None, stream_ptr()) == lg.GEMM_OK


def test_beta_zero_ignores_stale_c_and_is_deterministic(handle):
    for (M, N, K, ta, tb) in [(512, 512, 512, 0, 1), (16, 1024, 2048, 0, 0), (100, 100, 100, 1, 0)]:
        cfg = base_cfg(M, N, K, ta, tb, wl.BF16, wl.F32)
        inp = wl.make_inputs(cfg, 8)
        p = DeviceProblem(cfg, inp)            # C starts as NaN
        p.run(handle)
        first = c_bits_as_uint(cfg, p.result_bits()).copy()
        assert np.all(np.isfinite(decode_c(cfg, p.result_bits())))
        p.reset_c()
        p.run(handle)
        assert np.array_equal(first, c_bits_as_uint(cfg, p.result_bits()))      # same bits run to run


def test_linearity_in_beta(handle):
    cfg0 = base_cfg(32, 512, 1024, 0, 0, wl.BF16, wl.F32, beta=0.0)
    cfg1 = wl.scaled(cfg0, beta=1.0, c_dist=("normal", 1.0))
    inp0, inp1 = wl.make_inputs(cfg0, 21), wl.make_inputs(cfg1, 21)
    p0, p1 = DeviceProblem(cfg0, inp0), DeviceProblem(cfg1, inp1)
    p0.run(handle)
    p1.run(handle)
    diff = decode_c(cfg1, p1.result_bits()) - decode_c(cfg0, p0.result_bits())
    c0 = oracle.decode(wl.F32, inp1["C"]).reshape(32, 512)
    assert np.all(np.abs(diff - c0) <= 1e-5 * (np.abs(c0) + 1.0))


# ------------------------------------------------------------------ error behaviour

def test_invalid_arguments_leave_c_untouched(handle):
    cfg = base_cfg(64, 64, 64, 0, 0, wl.BF16, wl.BF16)
    inp = wl.make_inputs(cfg, 1)
    p = DeviceProblem(cfg, inp)
    before = p.result_bits().copy()
    A, B, C, s = p.A.data_ptr(), p.B.data_ptr(), p.C.data_ptr(), stream_ptr()
    run = lambda *a, **k: lg.gemm_run(*a, **k, check=False)
    E = lg.GEMM_ERR_INVALID_ARG
    assert run(0, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 64, None, s) == E           # null handle
    assert run(handle, -1, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 64, None, s) == E      # negative size
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 63, B, 64, 0.0, C, 64, None, s) == E      # lda < K
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 63, 0.0, C, 64, None, s) == E      # ldb < N
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 63, None, s) == E      # ldc < N
    assert run(handle, 64, 64, 64, 2, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 64, None, s) == E      # bad op
    assert run(handle, 64, 64, 64, 0, 0, 7, 1.0, A, 64, B, 64, 0.0, C, 64, None, s) == E            # bad dtype
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, 0, 64, B, 64, 0.0, C, 64, None, s) == E      # null A
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, 0, 64, None, s) == E      # null C
    bad_act = lg.make_epilogue(wl.BF16, 0, wl.BF16, 9)
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 64, bad_act, s) == E
    f16_out = lg.make_epilogue(wl.F16, 0, wl.BF16, 0)
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 64, f16_out, s) == lg.GEMM_ERR_UNSUPPORTED
    # a forced plan that cannot run the call is refused, not silently replaced
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 0, 2)
    assert run(handle, 8, 64, 64, 1, 0, wl.F32, 1.0, A, 8, B, 64, 0.0, C, 64, None, s) == lg.GEMM_ERR_UNSUPPORTED   # fp32 A stored K x M
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_SKINNY, 1, 2)
    assert run(handle, 64, 64, 64, 0, 0, wl.BF16, 1.0, A, 64, B, 64, 0.0, C, 64, None, s) == lg.GEMM_ERR_UNSUPPORTED   # variant against the layout
    lg.gemm_set_plan(handle)
    assert lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, 99, 0, check=False) == E
    assert "invalid" in lg.gemm_status_string(E)
    after = p.result_bits()
    assert np.array_equal(before.view(np.uint16), after.view(np.uint16))


# ------------------------------------------------------------------ strided batches

def test_batched_tile_variants(handle):
    # three products of 2 x 2 ragged tiles per matrix, padded strides, beta, bias and activation
    cfg = base_cfg(300, 264, 72, 0, 1, wl.BF16, wl.BF16, alpha=0.5, beta=1.0, a_dist=("normal", 1.0), b_dist=("normal", 0.3),
                   c_dist=("normal", 1.0), bias_dist=("normal", 1.0), bias_dtype=wl.F32, act=wl.ACT_GELU_TANH, lda=80, ldc=272)
    for v in tile_variants():
        print(f"batched tile variant {v}", flush=True)
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, v, 1)
        p = BatchedDeviceProblem(cfg, 3, 300 * 80 + 16, 264 * 72 + 8, 300 * 272 + 4, seed=60)
        p.run(handle)
        assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, v, 1)
        p.check(f"batched tile variant {v}")
    # a split of the k range is refused for a batch
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, 10, 2)
    p = BatchedDeviceProblem(cfg, 3, 300 * 80 + 16, 264 * 72 + 8, 300 * 272 + 4, seed=60)
    assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)


@pytest.mark.parametrize("ta,tb", [(0, 0), (1, 0), (1, 1)])
def test_batched_layouts_shared_operand_and_automatic_choice(handle, ta, tb):
    # B shared by the whole batch (stride 0), fp16 in and fp32 out, automatic plan
    cfg = base_cfg(136, 520, 200, ta, tb, wl.F16, wl.F32, a_dist=("normal", 1.0), b_dist=("normal", 0.2))
    p = BatchedDeviceProblem(cfg, 5, cfg.stride_a() + 8, 0, cfg.stride_c(), seed=70 + 2 * ta + tb)
    p.run(handle)
    assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_MFMA_TILE
    p.check(f"batched layout {ta}{tb}")


def test_batched_integer_exact_in_every_family(handle):
    cases = [
        ("tile", base_cfg(264, 136, 328, 0, 1, wl.BF16, wl.F32, alpha=1.0, beta=1.0), 4, lg.GEMM_KERNEL_MFMA_TILE),
        ("f32 tile", base_cfg(136, 264, 52, 0, 0, wl.F32, wl.F32), 9, lg.GEMM_KERNEL_MFMA_TILE),
        ("skinny", base_cfg(8, 512, 1024, 0, 0, wl.BF16, wl.BF16, alpha=1.0, beta=1.0), 3, lg.GEMM_KERNEL_SKINNY),
        ("skinny nt", base_cfg(20, 512, 1024, 0, 1, wl.F16, wl.F32), 3, lg.GEMM_KERNEL_SKINNY),
        ("general", base_cfg(37, 29, 53, 1, 0, wl.F32, wl.F32, alpha=1.0, beta=1.0), 6, lg.GEMM_KERNEL_GENERAL),
    ]
    for name, cfg, batch, family in cases:
        print(f"batched integer {name}", flush=True)
        p = BatchedDeviceProblem(cfg, batch, cfg.stride_a(), cfg.stride_b(), cfg.stride_c() + 8, seed=80, integer=True)
        if family == lg.GEMM_KERNEL_SKINNY:
            lg.gemm_set_plan(handle, family, -1, 0)
        p.run(handle)
        lg.gemm_set_plan(handle)
        assert lg.gemm_get_last_plan(handle)[0] == family, name
        p.check(f"batched integer {name}", exact=True)


def test_batched_unaligned_strides_take_the_general_kernel(handle):
    cfg = base_cfg(130, 72, 40, 0, 1, wl.BF16, wl.BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.5))
    p = BatchedDeviceProblem(cfg, 3, cfg.stride_a() + 3, cfg.stride_b() + 1, cfg.stride_c() + 1, seed=90)
    p.run(handle)
    assert lg.gemm_get_last_plan(handle)[0] == lg.GEMM_KERNEL_GENERAL
    p.check("batched unaligned")
    # the tile family refuses such strides when forced
    lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, -1, 0)
    assert p.run(handle, check=False) == lg.GEMM_ERR_UNSUPPORTED
    lg.gemm_set_plan(handle)


def test_batched_argument_errors_and_empty_batch(handle):
    cfg = base_cfg(64, 64, 64, 0, 0, wl.BF16, wl.BF16)
    p = BatchedDeviceProblem(cfg, 2, cfg.stride_a(), cfg.stride_b(), cfg.stride_c(), seed=1)
    before = wl.torch_to_bits(p.C).copy()
    args = dict(handle=handle, M=64, N=64, K=64, transA=0, transB=0, dtype=wl.BF16, alpha=1.0, A=p.A.data_ptr(), lda=64,
                B=p.B.data_ptr(), ldb=64, beta=0.0, C=p.C.data_ptr(), ldc=64, epilogue=None, stream=stream_ptr(), check=False)
    ok = dict(batch=2, strideA=4096, strideB=4096, strideC=4096)
    assert lg.gemm_run_batched(**{**args, **ok, "batch": -1}) == lg.GEMM_ERR_INVALID_ARG
    assert lg.gemm_run_batched(**{**args, **ok, "strideA": -1}) == lg.GEMM_ERR_INVALID_ARG
    assert lg.gemm_run_batched(**{**args, **ok, "strideC": 4095}) == lg.GEMM_ERR_INVALID_ARG      # results would overlap
    assert lg.gemm_run_batched(**{**args, **ok, "batch": 0}) == lg.GEMM_OK
    torch.cuda.synchronize()
    assert np.array_equal(wl.torch_to_bits(p.C).view(np.uint8), before.view(np.uint8))


# ------------------------------------------------------------------ handles, streams, workspace

def test_two_handles_on_two_streams_and_a_growing_workspace(handle):
    # Distinct handles own distinct workspaces and may run side by side on two streams; within one handle a call
    # that needs more workspace than the calls before it takes a new buffer and leaves the old one to the
    # launches queued ahead of it, while the other handle's work goes on.  Integer data -> every result exact.
    other = lg.gemm_create()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    sliced = base_cfg(392, 328, 1096, 0, 1, wl.BF16, wl.F32)                   # 3 slices: 1.5 MiB of partial results
    grown = base_cfg(1024, 1024, 1024, 0, 0, wl.BF16, wl.F32)                  # 16 slices: 64 MiB, beyond the first buffer
    streamed = base_cfg(32, 2048, 4096, 0, 0, wl.BF16, wl.BF16)                # split-K of the streaming kernels
    inputs = {id(c): wl.make_integer_inputs(c, 90 + i, -2, 2)[0] for i, c in enumerate((sliced, grown, streamed))}
    wants = {id(c): oracle.decode(c.out_dtype, expected_bits_exact(c, inputs[id(c)])) for c in (sliced, grown, streamed)}
    first = [DeviceProblem(sliced, inputs[id(sliced)]) for _ in range(6)]
    beside = [DeviceProblem(streamed, inputs[id(streamed)]) for _ in range(6)]
    big, last = DeviceProblem(grown, inputs[id(grown)]), DeviceProblem(sliced, inputs[id(sliced)])
    torch.cuda.synchronize()
    try:
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, 5, 3)
        lg.gemm_set_plan(other, lg.GEMM_KERNEL_SKINNY, -1, 4)
        for p, q in zip(first, beside):
            with torch.cuda.stream(s1):
                p.run(handle)
            with torch.cuda.stream(s2):
                q.run(other)
        assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, 5, 3) and lg.gemm_get_last_plan(other)[0] == lg.GEMM_KERNEL_SKINNY
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, 5, 16)
        with torch.cuda.stream(s1):
            big.run(handle)                      # the workspace grows with six launches queued ahead of it
        assert lg.gemm_get_last_plan(handle) == (lg.GEMM_KERNEL_MFMA_TILE, 5, 16)
        lg.gemm_set_plan(handle, lg.GEMM_KERNEL_MFMA_TILE, 5, 3)
        with torch.cuda.stream(s1):
            last.run(handle)
        torch.cuda.synchronize()
    finally:
        lg.gemm_set_plan(handle)
        torch.cuda.synchronize()
        lg.gemm_destroy(other)
    for p in first + [last]:
        assert np.array_equal(decode_c(sliced, p.result_bits()), wants[id(sliced)])
    for q in beside:
        assert np.array_equal(decode_c(streamed, q.result_bits()), wants[id(streamed)])
    assert np.array_equal(decode_c(grown, big.result_bits()), wants[id(grown)])


def test_a_growing_workspace_does_not_wait_for_the_stream(handle):
    # gemm_run never synchronises: a call that needs a larger workspace than the handle holds returns while the
    # work queued ahead of it (which uses the old buffer) is still running, and both results are exact.
    h = lg.gemm_create()
    queued = base_cfg(392, 328, 1096, 0, 1, wl.BF16, wl.F32)                   # 3 slices: uses the first (32 MiB) buffer
    grown = base_cfg(1024, 1024, 1024, 0, 0, wl.BF16, wl.F32)                  # 16 slices: 64 MiB
    filler = base_cfg(4096, 4096, 4096, 0, 1, wl.BF16, wl.BF16)                # ~0.1 ms each, no workspace
    iq, ig = wl.make_integer_inputs(queued, 31, -2, 2)[0], wl.make_integer_inputs(grown, 32, -2, 2)[0]
    want_q = oracle.decode(queued.out_dtype, expected_bits_exact(queued, iq))
    want_g = oracle.decode(grown.out_dtype, expected_bits_exact(grown, ig))
    pq, pg = DeviceProblem(queued, iq), DeviceProblem(grown, ig)
    pf = DeviceProblem(filler, wl.make_integer_inputs(filler, 33, -1, 1)[0])
    stream = torch.cuda.Stream()
    done = torch.cuda.Event()
    torch.cuda.synchronize()
    try:
        with torch.cuda.stream(stream):
            lg.gemm_set_plan(h, lg.GEMM_KERNEL_MFMA_TILE, 5, 3)
            pq.run(h)
            assert lg.gemm_workspace_size(h) == 32 << 20
            lg.gemm_set_plan(h)
            for _ in range(300):                                               # some 30 ms of work on the stream
                pf.run(h)
            lg.gemm_set_plan(h, lg.GEMM_KERNEL_MFMA_TILE, 5, 3)
            pq.run(h)                                                          # still on the first buffer
            done.record(stream)
            lg.gemm_set_plan(h, lg.GEMM_KERNEL_MFMA_TILE, 5, 16)
            pg.run(h)
            returned_early = not done.query()
            assert lg.gemm_workspace_size(h) >= 64 << 20
        torch.cuda.synchronize()
        assert returned_early, "the growing call waited for the work queued ahead of it"
        assert np.array_equal(decode_c(queued, pq.result_bits()), want_q)
        assert np.array_equal(decode_c(grown, pg.result_bits()), want_g)
        # with every stream idle, a reservation frees what the growth set aside and keeps the size
        lg.gemm_reserve_workspace(h, 0)
        assert lg.gemm_workspace_size(h) >= 64 << 20
        lg.gemm_reserve_workspace(h, 200 << 20)
        assert lg.gemm_workspace_size(h) >= 200 << 20
        with torch.cuda.stream(stream):
            pg.run(h)
        torch.cuda.synchronize()
        assert np.array_equal(decode_c(grown, pg.result_bits()), want_g)
    finally:
        torch.cuda.synchronize()
        lg.gemm_destroy(h)

"""CPU-only: the host logic that picks kernel family, tile, split and slices, through
gemm_plan_query (host arithmetic, no device).  Pins the choice for the benchmark configurations and for
the shapes each rule was made for, on a device with 256 compute units."""
import pytest

import paper_2512_16465_amd as lg
import workloads as wl

CUS = 256
TILE, SKINNY, GENERAL = lg.GEMM_KERNEL_MFMA_TILE, lg.GEMM_KERNEL_SKINNY, lg.GEMM_KERNEL_GENERAL


def plan(M, N, K, ta=0, tb=0, dtype=wl.BF16, out=None, batch=1, lda=None, ldb=None, ldc=None, cus=CUS):
    out = dtype if out is None else out
    lda = (M if ta else K) if lda is None else lda
    ldb = (K if tb else N) if ldb is None else ldb
    ldc = N if ldc is None else ldc
    kernel, variant, split = lg.gemm_plan_query(cus, batch, M, N, K, ta, tb, dtype, out, lda, ldb, ldc)
    return kernel, lg.gemm_variant_name(kernel, variant), split


def plan_of(name):
    c = {**wl.CONFIGS, **wl.EXTRA_CONFIGS}[name]
    return plan(c.M, c.N, c.K, c.transA, c.transB, c.dtype, c.out_dtype, c.batch, c.ld_a(), c.ld_b(), c.ld_c())


def test_benchmark_configurations():
    big = "dma16p_256x256x32_w2x2_s5"
    assert plan_of("C1") == (TILE, "f32_64x64x32_w2x2", 1)
    for name in ("C2", "C3", "C4", "X1", "X2"):
        assert plan_of(name) == (TILE, big, 1), name
    assert plan_of("C5") == (SKINNY, "skinny_nn_32x256_w4", 4)
    assert plan_of("X5") == (SKINNY, "skinny_nn_32x256_w4", 4)
    assert plan_of("X7") == (SKINNY, "skinny_nt_32x256_w4", 4)
    assert plan_of("X4") == (TILE, "dma16p_256x128x32_w2x2_s5", 1)       # N = 128: every full tile would be half empty
    assert plan_of("X6") == (TILE, "f32_128x128x32_w2x2", 1)
    assert plan_of("X11") == (TILE, "dma16p_128x256x32_w2x2_s5", 4)   # 64 tiles in 4 shares: one workgroup per unit
    assert plan_of("X8") == (TILE, "shortk_128x128_w2x2_persistent", 1)  # batched, K = 128, 32 tiles per unit: persistent workgroups
    # made in two: 8000 x 8192 on whole tiles (four full rounds), then the strip of 8 columns
    assert plan_of("X3") == (TILE, big, 1)
    assert plan_of("X9") == (TILE, big, 1) and plan_of("X10") == (TILE, big, 1)
    # ... whereas one more tile column that is half full stays one call with a split trailing round
    kernel, name, split = plan(8192, 8192 + 128, 8192, 0, 1)
    assert (kernel, name) == (TILE, big) and split > 1


def test_few_rows_on_a_16_bit_weight_stored_n_by_k_take_the_vector_alu_kernel():
    """Up to four rows, B stored N x K, A row-major, one matrix: variant 4 of the streaming family in one launch at
    every size (two slices only where N gives between a quarter and one workgroup per compute unit); more rows, the
    other layouts, fp32 and batches keep their kernels."""
    valu = "gemv16_nt_8x32_w4"
    assert plan_of("G1") == (SKINNY, valu, 1) and plan_of("G7") == (SKINNY, valu, 1) and plan_of("G8") == (SKINNY, valu, 1)
    for (M, N, K) in [(1, 512, 512), (2, 4096, 4096), (3, 16384, 16384), (4, 32000, 4096), (4, 128, 128)]:
        for dtype in (wl.BF16, wl.F16):
            assert plan(M, N, K, 0, 1, dtype=dtype)[:2] == (SKINNY, valu), (M, N, K)
    assert plan(1, 1536, 8192, 0, 1) == (SKINNY, valu, 2)           # 96 groups of 16 columns on 256 units
    assert plan(17, 8192, 8192, 0, 1)[:2] == (SKINNY, "skinny_nt_32x256_w4") and plan(8, 16384, 8192, 0, 1)[:2] == (SKINNY, "skinny_nt_32x256_w4")
    # 5 to 16 rows on a weight of 128 MiB at most with a long k: the MFMA kernel with 16 columns per workgroup, in
    # one launch (two slices where N leaves half the units idle), up to 4096 stored rows, and up to 12288 where K >= 4096
    narrow = "skinny_nt_16x16_w4"
    assert plan(5, 4096, 4096, 0, 1) == (SKINNY, narrow, 1) and plan(16, 4096, 14336, 0, 1) == (SKINNY, narrow, 1)
    assert plan_of("G4") == (SKINNY, narrow, 1)
    assert plan(8, 1024, 8192, 0, 1) == (SKINNY, narrow, 2) and plan(16, 2048, 2048, 0, 1) == (SKINNY, narrow, 1)      # at least four visits per wave and slice
    for (M, N, K) in [(8, 8192, 8192), (8, 4096, 16384), (16, 11008, 4096), (8, 4104, 4096), (5, 12288, 5120)]:
        assert plan(M, N, K, 0, 1) == (SKINNY, narrow, 1), (M, N, K)
    assert plan(8, 4096, 1024, 0, 1)[:2] == (SKINNY, narrow) and plan(12, 8192, 2048, 0, 1)[:2] == (SKINNY, narrow)      # a short k does not hurt it
    # 9 to 16 rows beyond one round: only where the last round is 65 % full (320 and 576 workgroups on 512 places are not, 688 are)
    assert plan(16, 5120, 5120, 0, 1)[0] == TILE and plan(12, 9216, 4608, 0, 1)[0] == TILE and plan(8, 5120, 5120, 0, 1)[:2] == (SKINNY, narrow)
    for (M, N, K) in [(17, 4096, 4096), (8, 4096, 128), (8, 8192, 512), (8, 12296, 4096)]:
        assert plan(M, N, K, 0, 1)[0] == TILE, (M, N, K)
    assert plan(8, 4096, 4096, 1, 1)[1] != narrow and plan(8, 4096, 4096, 0, 0)[1] != narrow
    assert plan(1, 4096, 4096, 0, 0)[0] == TILE                       # row-major B
    assert plan(1, 4096, 4096, 1, 1)[1] != valu                       # A stored K x M
    assert plan(4, 4096, 4100, 0, 1)[1] != valu                       # K no multiple of 8
    c = wl.Config("b", 2, 512, 512, 0, 1, wl.BF16, wl.BF16, batch=3)
    assert plan(c.M, c.N, c.K, 0, 1, c.dtype, c.out_dtype, c.batch, c.ld_a(), c.ld_b(), c.ld_c())[1] != valu


def test_family_by_rows_and_weight_size():
    # the streaming kernels: up to 32 rows on a B of 128 MiB or more with K and N of 4096 or more
    assert plan(32, 8192, 8192)[0] == SKINNY and plan(1, 16384, 4096, 0, 1)[0] == SKINNY
    assert plan(33, 16384, 16384)[:2] == (TILE, "dma16p_128x256x32_w2x2_s5")
    assert plan(64, 16384, 16384, 0, 1) == (TILE, "dma16p_128x256x32_w2x2_s5", 4)
    assert plan(32, 4096, 4096)[0] == TILE                      # 32 MiB of weights
    # up to 64 rows on cache-resident weights: the quartered 16x16x32 tile with its split
    kernel, name, shares = plan(48, 4096, 4096, 0, 1)
    assert (kernel, name) == (TILE, "dma16p_128x128x32_w2x2_s5") and shares > 1
    assert plan(64, 1024, 1024)[1] == "dma16p_128x128x32_w2x2_s5" and plan(65, 1024, 1024)[1] != "dma16p_128x128x32_w2x2_s5"
    assert plan(16, 2048, 32768)[0] == TILE                     # too few column groups
    assert plan(16, 65536, 2048)[0] == TILE                     # short k
    assert plan(8, 8192, 8192, ta=1)[0] == TILE                 # A stored K x M: the tiles take 8 rows ...
    assert plan(5, 8192, 8192, ta=1)[0] == SKINNY and plan(1, 512, 1024, ta=1, tb=1)[0] == SKINNY    # ... but no other count below it
    # 112 column groups: two slices fill 224 of 256 units in one round
    assert plan(32, 28672, 8192) == (SKINNY, "skinny_nn_32x256_w4", 2)
    # anything the vector loads cannot take goes to the general kernel
    assert plan(37, 29, 53, 1, 0, wl.F32)[0] == GENERAL
    assert plan(128, 128, 132)[0] == GENERAL                    # K not a multiple of 8
    assert plan(128, 128, 128, lda=132)[0] == GENERAL           # rows of A off the 16-byte grid


def test_roofline_rule_of_section_4_3():
    """The class every bench row gets from the library equals the one the bench computes for it from the
    workload's own flop and byte counts; the ridge points are where the rule puts them; and the class
    gates the family: compute-bound calls never stream, whatever their shape."""
    import bench
    names = {lg.GEMM_MEMORY_BOUND: "memory-bound", lg.GEMM_MIDDLE_ZONE: "middle-zone", lg.GEMM_COMPUTE_BOUND: "compute-bound"}
    for name, c in {**wl.CONFIGS, **wl.EXTRA_CONFIGS}.items():
        cls, ai = lg.gemm_roofline_class(c.batch, c.M, c.N, c.K, c.dtype, c.out_dtype, c.beta != 0.0,
                                         c.bias_dtype if c.bias_dist is not None else None)
        assert names[cls] == bench.classify(c), name
        assert abs(ai - c.flops() / c.algorithmic_bytes()) <= 1e-9 * ai, name
    expect = {"C1": "compute-bound", "C2": "compute-bound", "C3": "compute-bound", "C4": "compute-bound", "C5": "middle-zone",
              "X5": "memory-bound", "X7": "middle-zone", "X8": "middle-zone", "X4": "middle-zone", "X11": "middle-zone",
              "G1": "memory-bound", "G2": "memory-bound", "G5": "memory-bound", "G6": "memory-bound", "X6": "compute-bound"}
    for name, want in expect.items():
        assert bench.classify({**wl.CONFIGS, **wl.EXTRA_CONFIGS}[name]) == want, name
    # ridge points: 157.3e12 / 8e12 = 19.66 flop/byte and 2.5e15 / 8e12 = 312.5 (bf16, fp16); fp32 has one ridge
    # bf16 M x N x N with N large: intensity -> M flop/byte
    big = 1 << 15
    assert lg.gemm_roofline_class(1, 19, big, big, wl.BF16, wl.BF16)[0] == lg.GEMM_MEMORY_BOUND
    assert lg.gemm_roofline_class(1, 20, big, big, wl.BF16, wl.BF16)[0] == lg.GEMM_MIDDLE_ZONE
    assert lg.gemm_roofline_class(1, 316, big, big, wl.BF16, wl.BF16)[0] == lg.GEMM_MIDDLE_ZONE
    assert lg.gemm_roofline_class(1, 324, big, big, wl.BF16, wl.BF16)[0] == lg.GEMM_COMPUTE_BOUND
    assert lg.gemm_roofline_class(1, 39, big, big, wl.F32, wl.F32)[0] == lg.GEMM_MEMORY_BOUND       # M / 2 flop per byte
    assert lg.gemm_roofline_class(1, 40, big, big, wl.F32, wl.F32)[0] == lg.GEMM_COMPUTE_BOUND
    # the streaming family is a candidate only left of the matrix-core ridge; it is chosen for long streams of B
    assert plan(1, 8192, 8192)[0] == SKINNY and plan(8, 8192, 8192, 0, 1)[0] == SKINNY
    assert plan(1, 8192, 8192, dtype=wl.F32) == (SKINNY, "gemv_f32_nn_8x256_w4", 8)
    assert plan(8, 8192, 8192, 0, 1, dtype=wl.F32) == (SKINNY, "gemv_f32_nt_8x32_w4", 1)
    assert plan(8, 4096, 4096, dtype=wl.F32)[0] == TILE and plan(8, 4096, 4096, 0, 1, dtype=wl.F32)[0] == SKINNY
    assert plan(9, 8192, 8192, dtype=wl.F32)[0] == TILE and plan(1, 512, 512, dtype=wl.F32)[0] == TILE


def test_tile_split_and_slices():
    small = "dma_128x128x32_w2x2_s4"
    # 16 tiles of 128 x 128 with a long k loop: k slices
    kernel, name, slices = plan(512, 512, 4096)
    assert (kernel, name) == (TILE, small) and slices > 1
    assert plan(1024, 1024, 1024) == (TILE, small, 1)           # 64 tiles, short k: whole
    assert plan(512, 512, 4104)[2] > 1                           # a last slice shorter than the others
    kernel, name, split = plan(512, 516, 4096, tb=1)             # slices need N to be a multiple of 8 ...
    assert kernel == TILE and (split == 1 or name.startswith("dma16"))   # ... the split of the 16x16x32 tiles does not
    # one partly filled round of 256 x 256 tiles: split shares; a grid the half tile fills better
    kernel, name, shares = plan(4096, 4224, 4096)
    assert (kernel, name) == (TILE, "dma16p_256x256x32_w2x2_s5") and shares > 1
    assert plan(2048, 4096, 4096) == (TILE, "dma16p_128x256x32_w2x2_s5", 1)
    assert plan(4096, 2048, 2048) == (TILE, "dma16p_256x128x32_w2x2_s5", 1)
    # a few 128 x 128 tiles with k of 16384 or more: the 16x16x32 tile of that size with its split, not slices
    for shape in ((256, 1024, 32768), (512, 1024, 16384), (128, 512, 65536)):
        kernel, name, shares = plan(*shape)
        assert (kernel, name) == (TILE, "dma16p_128x128x32_w2x2_s5") and shares > 1, shape
    assert plan(128, 1024, 8192)[1] == small
    # ... and on grids of 30 to 200 small tiles inside the cache when its estimate is 8 % ahead of the sliced 32x32x16 tile
    assert plan(128, 4096, 4096) == (TILE, "dma16p_128x128x32_w2x2_s5", 6) and plan(512, 4096, 4096) == (TILE, "dma16p_128x128x32_w2x2_s5", 2)
    # weights beyond the last-level cache stay on the full tile with its split
    assert plan(640, 16384, 16384)[1] == "dma16p_256x256x32_w2x2_s5"
    # batched calls: no split, no slices, no half tiles
    for shape in ((2048, 128, 2048), (512, 512, 4096), (4096, 128, 4096)):
        kernel, name, split = plan(*shape, batch=8)
        assert kernel == TILE and split == 1 and not name.startswith("dma16p_256x128") and not name.startswith("dma16p_128x256")
    # short k loops over several rounds take the ring of three; one round of large tiles with K = 512 beats four of small ones (21 against 25 us)
    assert plan(8192, 8192, 256)[1] == "dma_128x128x32_w2x2_s3" and plan(4096, 4096, 512)[1] == "dma16p_256x256x32_w2x2_s5"


def test_fp32_tiles_and_slices():
    assert plan(1024, 1024, 1024, dtype=wl.F32) == (TILE, "f32_64x64x32_w2x2", 1)
    assert plan(4096, 4096, 4096, dtype=wl.F32) == (TILE, "f32_128x128x32_w2x2", 1)
    assert plan(3072, 3072, 3072, dtype=wl.F32) == (TILE, "f32_64x64x32_w2x2", 1)
    kernel, name, slices = plan(256, 256, 65536, dtype=wl.F32)
    assert (kernel, name, slices) == (TILE, "f32_64x64x32_w2x2", 16)
    assert plan(64, 1024, 1024, dtype=wl.F32)[2] > 1


def test_fewer_compute_units_change_the_choice():
    # the same 256 tiles are two rounds on 128 units: no share of a last round to split
    assert plan(4096, 4096, 4096, cus=128) == (TILE, "dma16p_256x256x32_w2x2_s5", 1)
    assert plan(32, 16384, 16384, cus=128)[2] == 2              # 64 column groups x 2 slices = 128 workgroups


def test_query_argument_errors():
    q = lambda *args: lg.gemm_plan_query(*args, check=False)
    ok = (CUS, 1, 64, 64, 64, 0, 0, wl.BF16, wl.BF16, 64, 64, 64)
    assert isinstance(q(*ok), tuple)
    assert q(0, *ok[1:]) == lg.GEMM_ERR_INVALID_ARG
    assert q(CUS, 1, 0, 64, 64, 0, 0, wl.BF16, wl.BF16, 64, 64, 64) == lg.GEMM_ERR_INVALID_ARG
    assert q(CUS, 1, 64, 64, 64, 0, 0, wl.BF16, wl.BF16, 63, 64, 64) == lg.GEMM_ERR_INVALID_ARG
    assert q(CUS, 1, 64, 64, 64, 2, 0, wl.BF16, wl.BF16, 64, 64, 64) == lg.GEMM_ERR_INVALID_ARG
    assert q(CUS, 1, 64, 64, 64, 0, 0, wl.BF16, wl.F16, 64, 64, 64) == lg.GEMM_ERR_UNSUPPORTED


def test_invariants_over_random_shapes():
    """Whatever the shape: a valid plan; the general kernel exactly when an operand cannot be read in 16-byte
    vectors (but for an A stored K x M with at most 64 rows, which the streaming kernels copy element by element);
    the streaming kernels only for few rows; no split inside a batch."""
    import random
    rng = random.Random(5)
    dims = [1, 7, 8, 24, 32, 33, 64, 100, 128, 136, 256, 520, 1024, 2056, 4096, 8192, 16384, 28672, 65536]
    for _ in range(3000):
        M, N, K = rng.choice(dims), rng.choice(dims), rng.choice(dims)
        ta, tb = rng.randint(0, 1), rng.randint(0, 1)
        dtype = rng.choice([wl.BF16, wl.F16, wl.F32])
        out = rng.choice([dtype, wl.F32])
        batch = rng.choice([1, 1, 1, 4])
        pad = lambda: rng.choice([0, 0, 0, 8, 3])
        lda, ldb, ldc = (M if ta else K) + pad(), (K if tb else N) + pad(), N + pad()
        kernel, variant, split = lg.gemm_plan_query(CUS, batch, M, N, K, ta, tb, dtype, out, lda, ldb, ldc)
        what = (batch, M, N, K, ta, tb, dtype, out, lda, ldb, ldc)
        assert kernel in (TILE, SKINNY, GENERAL) and split >= 1, what
        assert lg.gemm_variant_name(kernel, variant) is not None, what
        vec = 4 if dtype == wl.F32 else 8
        # rows of both operands start on 16-byte boundaries and hold whole vectors
        loadable = lda % vec == 0 and ldb % vec == 0 and (M if ta else K) % vec == 0 and (K if tb else N) % vec == 0
        copied_a = (ta and dtype != wl.F32 and M <= 64 and not loadable
                    and ldb % 8 == 0 and (K if tb else N) % 8 == 0 and K % 8 == 0 and N % 8 == 0
                    and (N if tb else K + 16) * ldb * 2 < 0x7ffffff0 and M * K * 2 < 0x7ffffff0)      # 32-bit offsets into B and the copy
        if copied_a and batch > 1:
            assert kernel in (SKINNY, GENERAL), what          # (the strides of the batch may break the alignment of B)
        elif copied_a:
            assert kernel == SKINNY, what
        else:
            assert (kernel == GENERAL) == (not loadable), what
        if kernel == SKINNY and dtype == wl.F32:
            assert M <= 8 and not ta, what
        elif kernel == SKINNY:
            assert (M <= 32 and not ta) or copied_a, what
        if batch > 1:
            assert split == 1 or kernel == SKINNY, what

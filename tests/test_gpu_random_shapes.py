"""GPU parity on seeded random calls in the automatic plan: shapes drawn around the tile edges (one
below, on, one vector above), both layouts of each operand, all element types, padded leading
dimensions, alpha / beta / bias / ReLU drawn per case.  Operands are small integers, so every
partial sum is exact in fp32 and the result is unique: the library must match the oracle's value,
rounded once to the output type, bit for bit, and must leave the padding columns of C alone."""
import numpy as np
import pytest

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import DeviceProblem, c_bits_as_uint, expected_bits_exact

pytestmark = pytest.mark.gpu

ROWS = [1, 8, 31, 32, 33, 48, 64, 72, 128, 136, 200, 256, 264, 384, 520]
COLS = [8, 24, 120, 128, 136, 256, 264, 512, 520, 1024, 1032]
DEPTH = [8, 32, 40, 200, 256, 512, 1024, 2048, 4104, 8192, 16392]
MAX_MACS = 3 << 28          # bounds the oracle's time per case (about a second)


def draw_case(rng):
    while True:
        M, N, K = (int(rng.choice(ROWS)), int(rng.choice(COLS)), int(rng.choice(DEPTH)))
        if M * N * K <= MAX_MACS:
            break
    ta, tb = int(rng.integers(2)), int(rng.integers(2))
    dtype = int(rng.choice([wl.BF16, wl.BF16, wl.F16, wl.F32]))
    out = dtype if rng.random() < 0.5 else wl.F32
    pad = lambda: int(rng.choice([0, 0, 8, 24]))
    a_cols, b_cols = (M if ta else K), (K if tb else N)
    return wl.Config("random", M, N, K, ta, tb, dtype, out,
                     alpha=float(rng.choice([1.0, 1.0, 2.0, -0.5])), beta=float(rng.choice([0.0, 0.0, 1.0, -2.0])),
                     bias_dist=("normal", 1.0) if rng.random() < 0.4 else None, bias_dtype=wl.F32,
                     act=int(rng.choice([wl.ACT_NONE, wl.ACT_NONE, wl.ACT_RELU])),
                     lda=a_cols + pad(), ldb=b_cols + pad(), ldc=N + int(rng.choice([0, 0, 8, 5])))


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    lg.gemm_destroy(h)


@pytest.mark.parametrize("seed", range(8))
def test_random_calls_match_the_oracle_exactly(handle, seed):
    rng = np.random.default_rng([2718, seed])
    seen = set()
    for i in range(10):
        cfg = draw_case(rng)
        # K <= 16384 and |a|, |b| <= 2: |sum| <= 2^16, times |alpha| <= 2, plus |beta| * 4 + 8: far below 2^24
        inp, _ = wl.make_integer_inputs(cfg, 100 * seed + i, -2, 2)
        what = (f"seed {seed} case {i}: {cfg.M}x{cfg.N}x{cfg.K} ta={cfg.transA} tb={cfg.transB} dtype={cfg.dtype} out={cfg.out_dtype} "
                f"ld=({cfg.ld_a()},{cfg.ld_b()},{cfg.ld_c()}) alpha={cfg.alpha} beta={cfg.beta} bias={cfg.bias_dist is not None} act={cfg.act}")
        print(what, flush=True)
        want = expected_bits_exact(cfg, inp)
        p = DeviceProblem(cfg, inp)
        before = p.result_bits().copy()
        p.run(handle)
        after = p.result_bits()
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        seen.add((lg.gemm_variant_name(kernel, variant), split > 1))
        got, ref = c_bits_as_uint(cfg, after), c_bits_as_uint(cfg, want.reshape(cfg.M, cfg.N))
        # +0 and -0 are the same value (ReLU of a negative, a sum that cancels): compare values, then NaN-freeness
        g, r = oracle.decode(cfg.out_dtype, got), oracle.decode(cfg.out_dtype, ref)
        assert np.array_equal(g, r), f"{what}: {np.sum(g != r)} elements differ ({lg.gemm_variant_name(kernel, variant)}, split {split})"
        if cfg.ld_c() > cfg.N and cfg.M > 1:
            assert np.array_equal(before[:-1, cfg.N:].view(np.uint8), after[:-1, cfg.N:].view(np.uint8)), f"{what}: padding of C written"
    assert len(seen) >= 3, seen       # the draw reaches several kernels


@pytest.mark.parametrize("seed", range(4))
def test_random_few_row_calls_on_weights_stored_n_by_k_match_the_oracle_exactly(handle, seed):
    """1 to 16 rows on a 16-bit weight stored N x K, A row-major, shapes drawn around the edges of the one-launch
    kernels (16 columns per workgroup, trips of 512 and chunks of 256 along k): the automatic plan's vector-ALU kernel
    and 16-column MFMA kernel, exact on integer data like every other call."""
    rng = np.random.default_rng([1618, seed])
    seen = set()
    for i in range(12):
        M = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16]))
        N = int(rng.choice([8, 24, 136, 520, 1032, 4104, 6152]))
        K = int(rng.choice([8, 40, 256, 520, 2048, 4104, 8192]))
        dtype = int(rng.choice([wl.BF16, wl.F16]))
        cfg = wl.Config("few", M, N, K, 0, 1, dtype, dtype if rng.random() < 0.5 else wl.F32,
                        alpha=float(rng.choice([1.0, 2.0, -0.5])), beta=float(rng.choice([0.0, 1.0, -2.0])),
                        bias_dist=("normal", 1.0) if rng.random() < 0.4 else None, bias_dtype=wl.F32,
                        act=int(rng.choice([wl.ACT_NONE, wl.ACT_RELU])),
                        lda=K + int(rng.choice([0, 8, 24])), ldb=K + int(rng.choice([0, 8, 24])), ldc=N + int(rng.choice([0, 8, 5])))
        inp, _ = wl.make_integer_inputs(cfg, 1000 * seed + i, -2, 2)
        what = (f"seed {seed} case {i}: {M}x{N}x{K} dtype={dtype} out={cfg.out_dtype} ld=({cfg.ld_a()},{cfg.ld_b()},{cfg.ld_c()}) "
                f"alpha={cfg.alpha} beta={cfg.beta} bias={cfg.bias_dist is not None} act={cfg.act}")
        print(what, flush=True)
        want = expected_bits_exact(cfg, inp)
        p = DeviceProblem(cfg, inp)
        before = p.result_bits().copy()
        p.run(handle)
        after = p.result_bits()
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        name = lg.gemm_variant_name(kernel, variant)
        seen.add(name)
        g = oracle.decode(cfg.out_dtype, c_bits_as_uint(cfg, after))
        r = oracle.decode(cfg.out_dtype, c_bits_as_uint(cfg, want.reshape(cfg.M, cfg.N)))
        assert np.array_equal(g, r), f"{what}: {np.sum(g != r)} elements differ ({name}, split {split})"
        if cfg.ld_c() > cfg.N and cfg.M > 1:
            assert np.array_equal(before[:-1, cfg.N:].view(np.uint8), after[:-1, cfg.N:].view(np.uint8)), f"{what}: padding of C written"
    assert "gemv16_nt_8x32_w4" in seen and "skinny_nt_16x16_w4" in seen, seen


@pytest.mark.parametrize("seed", range(4))
def test_random_batches_of_short_products_match_the_oracle_exactly(handle, seed):
    """Strided batches with K <= 128 and a tile or more per compute unit, shapes drawn around the tile edges: the
    automatic plan's persistent short-k kernel where C is write-only, the other tile kernels where it is not."""
    from gpu_harness import BatchedDeviceProblem
    rng = np.random.default_rng([31415, seed])
    seen = set()
    for i in range(4):
        M = int(rng.choice([1024, 1032, 1160, 1536, 2040, 2176]))
        N = int(rng.choice([1024, 1032, 1288, 1536, 2056]))
        K = int(rng.choice([32, 64, 96, 128]))
        batch = int(rng.integers(2, 7))
        ta, tb = int(rng.integers(2)), int(rng.integers(2))
        dtype = int(rng.choice([wl.BF16, wl.F16]))
        out = dtype if rng.random() < 0.6 else wl.F32
        plain = rng.random() < 0.75                      # write-only C, no bias: what the short-k kernel takes
        pad = lambda: int(rng.choice([0, 8, 24]))
        cfg = wl.Config("random", M, N, K, ta, tb, dtype, out, alpha=float(rng.choice([1.0, 2.0, -0.5])),
                        beta=0.0 if plain else float(rng.choice([1.0, -2.0])),
                        bias_dist=None if plain else ("normal", 1.0), bias_dtype=wl.F32,
                        act=int(rng.choice([wl.ACT_NONE, wl.ACT_RELU])),
                        lda=(M if ta else K) + pad(), ldb=(K if tb else N) + pad(), ldc=N + int(rng.choice([0, 8, 16])))
        what = (f"seed {seed} case {i}: {batch} x {M}x{N}x{K} ta={ta} tb={tb} dtype={dtype} out={out} "
                f"ld=({cfg.ld_a()},{cfg.ld_b()},{cfg.ld_c()}) alpha={cfg.alpha} beta={cfg.beta} act={cfg.act}")
        print(what, flush=True)
        p = BatchedDeviceProblem(cfg, batch, cfg.stride_a() + 8 * int(rng.integers(3)), cfg.stride_b() + 8 * int(rng.integers(3)),
                                 cfg.stride_c() + 8 * int(rng.integers(3)), seed=1000 * seed + 10 * i, integer=True)
        p.run(handle)
        kernel, variant, split = lg.gemm_get_last_plan(handle)
        seen.add(lg.gemm_variant_name(kernel, variant))
        p.check(what + f" ({lg.gemm_variant_name(kernel, variant)}, split {split})", exact=True)
    assert any("shortk" in name for name in seen), seen

"""CPU-only pins of the oracle: each test fixes a part of ``oracle/gemm_oracle.c`` to a fact that
does not come from that file -- a closed form, an integer or rational computation done another
way, a library routine applied to a special case, or a constant from a table.

The mistakes they are chosen against: a dropped or doubled term (all-ones, integer matmul), a
wrong sign (integer matmul, GELU antisymmetry), a wrong index or leading dimension (padded,
non-square integer cases), a transposed operand (permutation and transposition tests), a wrong
rounding (codec ties and exhaustive round trips), a mis-ordered epilogue (rational brute force).
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import ACT_GELU_ERF, ACT_NONE, BF16, F16, F32, Problem
from workloads import to_bits

DTYPES = [F32, F16, BF16]
TRANS = [(0, 0), (0, 1), (1, 0), (1, 1)]


def store(vals2d, ld, dtype):
    """2-D float values -> padded 1-D storage; padding is NaN so that any stray read poisons the result."""
    rows, cols = vals2d.shape
    full = np.full((rows, ld), np.nan, dtype=np.float32)
    full[:, :cols] = vals2d
    return to_bits(full, dtype).reshape(-1)


def problem_from(a_mk, b_kn, dtype, ta, tb, pad=(0, 0), **kw):
    """Build a Problem from logical op(A) (M x K) and op(B) (K x N) value matrices."""
    M, K = a_mk.shape
    _, N = b_kn.shape
    a_st = a_mk.T if ta else a_mk
    b_st = b_kn.T if tb else b_kn
    lda, ldb = a_st.shape[1] + pad[0], b_st.shape[1] + pad[1]
    return Problem(M, N, K, ta, tb, dtype, store(np.asarray(a_st, np.float32), lda, dtype), lda,
                   store(np.asarray(b_st, np.float32), ldb, dtype), ldb, **kw)


# ---------------------------------------------------------------- codecs

def test_codec_golden_patterns(golden_dir):
    code = {"f32": F32, "f16": F16, "bf16": BF16}
    n = 0
    for line in open(os.path.join(golden_dir, "float_patterns.txt")):
        if line.startswith("#") or not line.strip():
            continue
        fmt, hexbits, expr = line.split()
        bits = int(hexbits, 16)
        value = Fraction(eval(expr, {"__builtins__": {}}, {}))   # every quotient here is exact in fp64
        arr = np.array([bits], dtype=np.uint32 if fmt == "f32" else np.uint16)
        got = oracle.decode(code[fmt], arr)[0]
        assert Fraction(got) == value, (fmt, hexbits)
        assert int(oracle.encode(code[fmt], np.array([got]))[0]) == bits
        n += 1
    assert n >= 15


@pytest.mark.parametrize("dtype,tdtype", [(BF16, torch.bfloat16), (F16, torch.float16)])
def test_codec_all_16bit_patterns_against_torch(dtype, tdtype):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    dec = oracle.decode(dtype, bits)
    want = torch.from_numpy(bits.view(np.int16)).view(tdtype).to(torch.float64).numpy()
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(dec), nan)
    assert np.array_equal(dec[~nan], want[~nan])
    assert np.array_equal(np.signbit(dec[~nan]), np.signbit(want[~nan]))
    # decode -> encode is the identity on every non-NaN pattern; NaNs stay NaN
    back = oracle.encode(dtype, dec)
    assert np.array_equal(back[~nan], bits[~nan])
    assert np.all(np.isnan(oracle.decode(dtype, back[nan])))


@pytest.mark.parametrize("dtype,tdtype", [(BF16, torch.bfloat16), (F16, torch.float16)])
def test_codec_rounding_against_torch(dtype, tdtype):
    rng = np.random.default_rng(5)
    x = np.concatenate([
        rng.standard_normal(60000).astype(np.float32),
        (rng.standard_normal(20000) * 1e-6).astype(np.float32),
        (rng.standard_normal(20000) * 3e4).astype(np.float32),
        np.exp(rng.uniform(-100, 88, 30000)).astype(np.float32),
        # exact ties and their neighbours around many binades
        np.array([(1 + (2 * m + 1) * 2.0 ** -(9 if dtype == BF16 else 12)) * 2.0 ** e
                  for m in range(64) for e in (-20, -3, 0, 5, 14)], dtype=np.float32),
        np.array([0.0, -0.0, np.inf, -np.inf, 65504.0, 65520.0, 65519.0, 3.3895314e38, 3.4e38,
                  2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -25, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -134],
                 dtype=np.float32),
    ])
    want = torch.from_numpy(x).to(tdtype).view(torch.int16).numpy().view(np.uint16)
    got = oracle.encode(dtype, x.astype(np.float64))
    assert np.array_equal(got, want)


def test_codec_tie_pins():
    # nearest-even at bf16: 1 + 2^-8 lies halfway between 1 and 1 + 2^-7 -> even significand 1.0
    assert int(oracle.encode(BF16, np.array([1 + 2.0 ** -8]))[0]) == 0x3F80
    # 1 + 3*2^-8 lies halfway between 1 + 2^-7 (odd) and 1 + 2^-6 (even)
    assert int(oracle.encode(BF16, np.array([1 + 3 * 2.0 ** -8]))[0]) == 0x3F82
    # the largest finite bf16 plus half a unit in the last place overflows to infinity
    big = 255 * 2.0 ** 120
    assert int(oracle.encode(BF16, np.array([big + 2.0 ** 119]))[0]) == 0x7F80
    assert int(oracle.encode(BF16, np.array([big + 2.0 ** 118]))[0]) == 0x7F7F
    # integers: 257 -> 256 (tie, even), 259 -> 260, 16385 -> 16384
    for v, w in [(257.0, 256.0), (259.0, 260.0), (16385.0, 16384.0), (4096.0, 4096.0)]:
        assert oracle.decode(BF16, oracle.encode(BF16, np.array([v])))[0] == w
    # fp32 encode agrees with numpy's own double -> float conversion
    x = np.random.default_rng(1).standard_normal(5000) * 10.0 ** np.random.default_rng(2).integers(-30, 30, 5000)
    assert np.array_equal(oracle.encode(F32, x), x.astype(np.float32).view(np.uint32))


# ---------------------------------------------------------------- activation

def test_gelu_closed_forms(golden_dir):
    for line in open(os.path.join(golden_dir, "normal_cdf.txt")):
        if line.startswith("#") or not line.strip():
            continue
        x, phi = map(float, line.split())
        assert abs(oracle.gelu_erf(x) - x * phi) < 6e-10 * max(1.0, x)
        # Phi(-x) = 1 - Phi(x)
        assert abs(oracle.gelu_erf(-x) - (-x) * (1 - phi)) < 6e-10 * max(1.0, x)
    assert oracle.gelu_erf(0.0) == 0.0
    for x in [0.1, 0.7, 1.3, 2.9, 4.4, 7.0]:
        assert abs(oracle.gelu_erf(-x) - (oracle.gelu_erf(x) - x)) < 1e-15 * max(1, x)
    for x in [6.0, 8.0, 33.0]:     # x*Phi(x) equals x to bf16 precision from 6 upwards
        assert int(oracle.encode(BF16, np.array([oracle.gelu_erf(x)]))[0]) == int(oracle.encode(BF16, np.array([x]))[0])
    assert oracle.gelu_erf(-40.0) == 0.0 or abs(oracle.gelu_erf(-40.0)) < 1e-300


def test_gelu_inside_gemm():
    # K=1, A=[x], B=[1] -> act(x + bias)
    for x, b in [(1.0, 0.0), (0.5, 0.5), (-2.0, 1.0)]:
        p = problem_from(np.array([[x]]), np.array([[1.0]]), F32, 0, 0,
                         bias=np.array([b], np.float32), bias_dtype=F32, act=ACT_GELU_ERF)
        assert oracle.gemm_full(p)[0, 0] == oracle.gelu_erf(x + b)


def test_relu_silu_gelu_tanh_closed_forms_and_library():
    import math
    import torch
    relu = lambda x: oracle.act(oracle.ACT_RELU, x)
    silu = lambda x: oracle.act(oracle.ACT_SILU, x)
    gtanh = lambda x: oracle.act(oracle.ACT_GELU_TANH, x)
    # ReLU: exact
    for x in [0.0, 1.0, -1.0, 3.5, -3.5, 1e-30, -1e-30, 65504.0, -65504.0]:
        assert relu(x) == (x if x > 0 else 0.0)
    assert math.isnan(relu(float("nan")))
    # SiLU: sigmoid(ln 3) = 3/4, sigmoid(ln 9) = 9/10, sigmoid(-ln 3) = 1/4 (closed forms), silu(0) = 0,
    # silu(x) - silu(-x) = x, silu(x) -> x for large x and -> 0 for large -x
    for r, sig in [(3.0, 0.75), (9.0, 0.9), (1.0 / 3.0, 0.25), (99.0, 0.99), (1.0, 0.5)]:
        x = math.log(r)
        assert abs(silu(x) - x * sig) < 1e-15 * max(1.0, abs(x))
    for x in [0.1, 0.9, 2.5, 7.0, 30.0]:
        assert abs((silu(x) - silu(-x)) - x) < 1e-15 * max(1.0, x)
    assert silu(0.0) == 0.0 and silu(800.0) == 800.0 and abs(silu(-800.0)) < 1e-300
    # GELU, tanh form: g(x) - g(-x) = x (tanh is odd), g(0) = 0, within 5e-4 of the exact (erf) GELU everywhere
    # (the known quality of that approximation) and equal to it to 1e-6 relative for |x| < 0.01
    for x in [0.1, 0.9, 2.5, 7.0]:
        assert abs((gtanh(x) - gtanh(-x)) - x) < 1e-15 * max(1.0, x)
    assert gtanh(0.0) == 0.0
    worst = max(abs(gtanh(x) - oracle.gelu_erf(x)) for x in np.linspace(-8.0, 8.0, 3201))
    assert 1e-4 < worst < 5e-4        # a different constant or a dropped cubic term leaves this window
    for x in [1e-3, -5e-3, 9e-3]:
        assert abs(gtanh(x) - oracle.gelu_erf(x)) < 1e-6 * abs(x)
    # an independent library's routines, in fp64
    xs = torch.tensor(np.concatenate([np.linspace(-12.0, 12.0, 2001), [1e-8, -1e-8, 40.0, -40.0]]), dtype=torch.float64)
    for code, fn in [(oracle.ACT_RELU, torch.nn.functional.relu), (oracle.ACT_SILU, torch.nn.functional.silu),
                     (oracle.ACT_GELU_TANH, lambda t: torch.nn.functional.gelu(t, approximate="tanh")),
                     (oracle.ACT_GELU_ERF, torch.nn.functional.gelu)]:
        want = fn(xs).numpy()
        got = np.array([oracle.act(code, float(x)) for x in xs.numpy()])
        assert np.all(np.abs(got - want) <= 4e-16 * np.maximum(1.0, np.abs(want))), code
    assert oracle.act(oracle.ACT_NONE, -2.5) == -2.5


def test_every_activation_inside_gemm():
    # K=1, A=[x], B=[1] -> act(x + bias); an unknown activation code is an error
    for code in (oracle.ACT_RELU, oracle.ACT_SILU, oracle.ACT_GELU_TANH, oracle.ACT_GELU_ERF, oracle.ACT_NONE):
        for x, b in [(1.0, 0.0), (0.5, 0.5), (-2.0, 1.0), (-0.25, -0.5)]:
            p = problem_from(np.array([[x]]), np.array([[1.0]]), F32, 0, 0,
                             bias=np.array([b], np.float32), bias_dtype=F32, act=code)
            assert oracle.gemm_full(p)[0, 0] == oracle.act(code, x + b)
    p = problem_from(np.array([[1.0]]), np.array([[1.0]]), F32, 0, 0, act=7)
    with pytest.raises(Exception):
        oracle.gemm_full(p)


# ---------------------------------------------------------------- closed forms of the product

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("ta,tb", TRANS)
def test_identity(dtype, ta, tb):
    rng = np.random.default_rng(3)
    n, m = 9, 6
    X = oracle.decode(dtype, to_bits(rng.standard_normal((n, m)).astype(np.float32), dtype))  # representable values
    I = np.eye(n)
    got = oracle.gemm_full(problem_from(I, X, dtype, ta, tb, pad=(2, 3)))       # I * X
    assert np.array_equal(got, X)
    got = oracle.gemm_full(problem_from(X.T, I, dtype, ta, tb, pad=(1, 0)))     # X^T * I
    assert np.array_equal(got, X.T)


@pytest.mark.parametrize("ta,tb", TRANS)
def test_permutation(ta, tb):
    rng = np.random.default_rng(4)
    n, m = 11, 7
    X = oracle.decode(BF16, to_bits(rng.standard_normal((n, m)).astype(np.float32), BF16))
    perm = rng.permutation(n)
    P = np.zeros((n, n))
    P[np.arange(n), perm] = 1.0            # (P X)[i] = X[perm[i]]
    assert np.array_equal(oracle.gemm_full(problem_from(P, X, BF16, ta, tb, pad=(4, 4))), X[perm])
    # (X^T P)[:, j] = X^T[:, i] where perm[i] = j
    inv = np.argsort(perm)
    assert np.array_equal(oracle.gemm_full(problem_from(X.T, P, BF16, ta, tb)), X.T[:, inv])


@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("K", [1, 17, 257, 259, 4096])
def test_all_ones_gives_K(dtype, K):
    M, N = 3, 5
    ref = oracle.gemm_full(problem_from(np.ones((M, K)), np.ones((K, N)), dtype, 0, 1))
    assert np.all(ref == float(K))


# ---------------------------------------------------------------- integer matmul done another way

@pytest.mark.parametrize("dtype", DTYPES)
@pytest.mark.parametrize("ta,tb", TRANS)
def test_small_integers_against_int64(dtype, ta, tb):
    rng = np.random.default_rng(100 + 10 * ta + tb)
    M, N, K = 13, 7, 29                      # all different: a swapped dimension cannot pass
    A = rng.integers(-3, 4, (M, K))
    B = rng.integers(-3, 4, (K, N))
    C = rng.integers(-5, 6, (M, N))
    bias = rng.integers(-4, 5, (N,))
    want = 2 * (A.astype(np.int64) @ B.astype(np.int64)) - 3 * C + bias[None, :]
    ldc = N + 5
    p = problem_from(A.astype(np.float64), B.astype(np.float64), dtype, ta, tb, pad=(3, 1),
                     alpha=2.0, beta=-3.0, C=store(C.astype(np.float32), ldc, dtype), ldc=ldc, c_dtype=dtype,
                     bias=to_bits(bias.astype(np.float32), dtype), bias_dtype=dtype)
    ref, sumabs, mag = oracle.gemm_full(p, want_bounds=True)
    assert np.array_equal(ref, want.astype(np.float64))
    want_sa = np.abs(A).astype(np.int64) @ np.abs(B).astype(np.int64)
    assert np.array_equal(sumabs, want_sa.astype(np.float64))
    assert np.array_equal(mag, (2 * want_sa + 3 * np.abs(C) + np.abs(bias)[None, :]).astype(np.float64))


def test_mixed_operand_types_for_c_and_bias():
    # bf16 A, B with fp32 C_in and fp16 bias: each operand is decoded with its own type
    rng = np.random.default_rng(8)
    M, N, K = 4, 6, 5
    A, B = rng.integers(-2, 3, (M, K)), rng.integers(-2, 3, (K, N))
    C, bias = rng.integers(-9, 10, (M, N)), rng.integers(-9, 10, (N,))
    p = problem_from(A.astype(float), B.astype(float), BF16, 0, 0, alpha=1.0, beta=1.0,
                     C=store(C.astype(np.float32), N, F32), ldc=N, c_dtype=F32,
                     bias=to_bits(bias.astype(np.float32), F16), bias_dtype=F16)
    assert np.array_equal(oracle.gemm_full(p), (A @ B + C + bias[None, :]).astype(float))


# ---------------------------------------------------------------- exact rational brute force

def test_tiny_shapes_against_fractions():
    rng = np.random.default_rng(6)
    scal = [0.0, 1.0, -2.0, 0.5]
    cases = 0
    for (M, N, K), (ta, tb), dtype in itertools.product(
            [(1, 1, 1), (2, 3, 4), (5, 2, 3), (3, 5, 1), (4, 4, 5)], TRANS, DTYPES):
        alpha, beta = scal[rng.integers(4)], scal[rng.integers(4)]
        # dyadic values with few bits: every product and sum is exact in fp64
        A = rng.integers(-8, 9, (M, K)) / 8.0
        B = rng.integers(-8, 9, (K, N)) / 4.0
        C = rng.integers(-8, 9, (M, N)) / 2.0
        bias = rng.integers(-8, 9, (N,)) / 8.0
        ldc = N + 2
        p = problem_from(A, B, dtype, ta, tb, pad=(1, 2), alpha=alpha, beta=beta,
                         C=store(C.astype(np.float32), ldc, dtype), ldc=ldc, c_dtype=dtype,
                         bias=to_bits(bias.astype(np.float32), dtype), bias_dtype=dtype)
        ref = oracle.gemm_full(p)
        for i in range(M):
            for j in range(N):
                acc = sum(Fraction(A[i, k]) * Fraction(B[k, j]) for k in range(K))
                want = Fraction(alpha) * acc + Fraction(beta) * Fraction(C[i, j]) + Fraction(bias[j])
                assert Fraction(ref[i, j]) == want, (M, N, K, ta, tb, dtype, i, j)
        cases += 1
    assert cases == 60


def test_non_dyadic_against_fractions_within_one_ulp():
    rng = np.random.default_rng(7)
    M, N, K = 3, 4, 5
    A = oracle.decode(F32, to_bits(rng.standard_normal((M, K)).astype(np.float32), F32))
    B = oracle.decode(F32, to_bits(rng.standard_normal((K, N)).astype(np.float32), F32))
    ref = oracle.gemm_full(problem_from(A, B, F32, 0, 0))
    for i in range(M):
        for j in range(N):
            want = sum(Fraction(A[i, k]) * Fraction(B[k, j]) for k in range(K))
            scale = sum(abs(Fraction(A[i, k]) * Fraction(B[k, j])) for k in range(K))
            assert abs(Fraction(ref[i, j]) - want) <= K * Fraction(2) ** -52 * scale


# ---------------------------------------------------------------- algebraic invariants

def test_outer_product_and_power_of_two_scaling():
    rng = np.random.default_rng(9)
    a = oracle.decode(BF16, to_bits(rng.standard_normal((6, 1)).astype(np.float32), BF16))
    b = oracle.decode(BF16, to_bits(rng.standard_normal((1, 4)).astype(np.float32), BF16))
    ref = oracle.gemm_full(problem_from(a, b, BF16, 0, 0))
    assert np.array_equal(ref, a * b)            # one exact product per entry
    ref8 = oracle.gemm_full(problem_from(a, b, BF16, 0, 0, alpha=8.0))
    assert np.array_equal(ref8, 8.0 * ref)
    refm = oracle.gemm_full(problem_from(a, b, BF16, 0, 0, alpha=-0.25))
    assert np.array_equal(refm, -0.25 * ref)


def test_transpose_identity():
    # (A B)^T = B^T A^T, obtained by swapping operands and flipping both flags: same k order, same bits
    rng = np.random.default_rng(10)
    M, N, K = 5, 8, 37
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    for ta, tb in TRANS:
        ref = oracle.gemm_full(problem_from(A, B, F32, ta, tb))
        ref_t = oracle.gemm_full(problem_from(B.T.copy(), A.T.copy(), F32, tb, ta))
        assert np.array_equal(ref.T, ref_t)
        # all four storage variants of the same logical product agree bit for bit
        assert np.array_equal(ref, oracle.gemm_full(problem_from(A, B, F32, 0, 0)))


def test_beta_semantics():
    rng = np.random.default_rng(11)
    M, N, K = 4, 5, 6
    Cv = rng.standard_normal((M, N)).astype(np.float32)
    zero = np.zeros((M, K))
    B = rng.standard_normal((K, N))
    # A = 0, beta = 1: C unchanged
    p = problem_from(zero, B, F32, 0, 0, beta=1.0, C=store(Cv, N, F32), ldc=N, c_dtype=F32)
    assert np.array_equal(oracle.gemm_full(p), Cv.astype(np.float64))
    # beta = 0: C is never read, NaN there cannot leak; C may even be absent
    A = rng.standard_normal((M, K))
    nanC = np.full((M, N), np.nan, np.float32)
    r0 = oracle.gemm_full(problem_from(A, B, F32, 0, 0, beta=0.0, C=store(nanC, N, F32), ldc=N, c_dtype=F32))
    r1 = oracle.gemm_full(problem_from(A, B, F32, 0, 0))
    assert np.all(np.isfinite(r0)) and np.array_equal(r0, r1)
    # K = 0: the sum is empty
    pe = Problem(M, N, 0, 0, 0, F32, np.zeros(0, np.float32), 1, np.zeros(0, np.float32), N,
                 beta=2.0, C=store(Cv, N, F32), ldc=N, c_dtype=F32)
    assert np.array_equal(oracle.gemm_full(pe), 2.0 * Cv.astype(np.float64))


@pytest.mark.parametrize("dtype", DTYPES)
def test_against_numpy_fp64_matmul(dtype):
    # a library contraction on the decoded operands: equal up to summation order
    rng = np.random.default_rng(12)
    M, N, K = 33, 47, 129
    A = oracle.decode(dtype, to_bits(rng.standard_normal((M, K)).astype(np.float32), dtype))
    B = oracle.decode(dtype, to_bits(rng.standard_normal((K, N)).astype(np.float32), dtype))
    for ta, tb in TRANS:
        ref, sumabs, _ = oracle.gemm_full(problem_from(A, B, dtype, ta, tb, pad=(5, 7)), want_bounds=True)
        assert np.all(np.abs(ref - A @ B) <= 1e-13 * (np.abs(A) @ np.abs(B)))
        assert np.allclose(sumabs, np.abs(A) @ np.abs(B), rtol=1e-13, atol=0)


def test_sampled_and_row_entry_points_match_full():
    rng = np.random.default_rng(13)
    M, N, K = 21, 34, 19
    A = rng.standard_normal((M, K)).astype(np.float32)
    B = rng.standard_normal((K, N)).astype(np.float32)
    Cv = rng.standard_normal((M, N)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    p = problem_from(A, B, BF16, 0, 1, alpha=0.5, beta=1.5, C=store(Cv, N + 1, BF16), ldc=N + 1, c_dtype=BF16,
                     bias=to_bits(bias, BF16), bias_dtype=BF16, act=ACT_GELU_ERF)
    ref, sa, mag = oracle.gemm_full(p, want_bounds=True)
    rows = rng.integers(0, M, 200)
    cols = rng.integers(0, N, 200)
    r2, s2, m2 = oracle.gemm_at(p, rows, cols)
    assert np.array_equal(r2, ref[rows, cols]) and np.array_equal(s2, sa[rows, cols]) and np.array_equal(m2, mag[rows, cols])
    assert np.array_equal(oracle.gemm_rows(p, 3, 7), ref[3:10])
    with pytest.raises(ValueError):
        oracle.gemm_at(p, np.array([M]), np.array([0]))


def test_activation_applies_after_the_whole_affine_part():
    # act(alpha*AB + beta*C + bias), checked against a scalar evaluation with math.erf
    import math
    a, b, c, bias, alpha, beta = 0.75, -1.5, 2.0, 0.25, 2.0, 0.5
    p = problem_from(np.array([[a]]), np.array([[b]]), F32, 0, 0, alpha=alpha, beta=beta,
                     C=np.array([c], np.float32), ldc=1, c_dtype=F32,
                     bias=np.array([bias], np.float32), bias_dtype=F32, act=ACT_GELU_ERF)
    x = alpha * a * b + beta * c + bias
    assert abs(oracle.gemm_full(p)[0, 0] - 0.5 * x * (1 + math.erf(x / math.sqrt(2)))) < 1e-15


def test_strided_batch_against_int64_einsum():
    """A strided batch is `batch` independent products whose matrices lie b * stride elements into
    their arrays: integer data against numpy's int64 einsum, with padded strides, a shared A
    (stride 0), beta and bias."""
    rng = np.random.default_rng(5)
    batch, M, N, K = 5, 3, 4, 6
    lda, ldb, ldc = K + 2, N + 1, N + 3
    sB, sC = K * ldb + 7, M * ldc + 5
    A = rng.integers(-3, 4, size=(M, K))
    B = rng.integers(-3, 4, size=(batch, K, N))
    C0 = rng.integers(-3, 4, size=(batch, M, N))
    bias = rng.integers(-2, 3, size=N)
    a_st = np.full(M * lda, 9.0, np.float32); a_st.reshape(M, lda)[:, :K] = A
    b_st = np.full(batch * sB, 9.0, np.float32)
    c_st = np.full(batch * sC, 9.0, np.float32)
    for b in range(batch):
        b_st[b * sB: b * sB + K * ldb].reshape(K, ldb)[:, :N] = B[b]
        c_st[b * sC: b * sC + M * ldc].reshape(M, ldc)[:, :N] = C0[b]
    prob = oracle.Problem(M, N, K, 0, 0, oracle.F32, a_st, lda, b_st, ldb, alpha=2.0, beta=-1.0, C=c_st, ldc=ldc,
                          c_dtype=oracle.F32, bias=bias.astype(np.float32), bias_dtype=oracle.F32)
    got = oracle.gemm_strided_batched(prob, batch, 0, sB, sC)
    want = 2 * np.einsum("mk,bkn->bmn", A, B) - C0 + bias[None, None, :]
    assert got.shape == (batch, M, N) and np.array_equal(got, want.astype(np.float64))

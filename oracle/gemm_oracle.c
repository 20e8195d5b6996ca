/*
 * CPU oracle for the dense GEMM with fused epilogue.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition against which the GPU library is
 * checked.  It is not part of the product: only the test-suite, the smoke
 * check and the benchmark's CPU-baseline leg may link or call it, and it shares
 * no code (headers, codecs, tables, helpers) with the GPU side.
 *
 * What it computes (the operation the paper's GEMM case study optimises,
 * Section 5.4 and Table 1; the paper never writes the formula, so the plain
 * BLAS statement is used):
 *
 *   acc(i,j) = sum_{k=0}^{K-1} op(A)(i,k) * op(B)(k,j)        fp64, k ascending
 *   pre(i,j) = alpha*acc(i,j) + (beta==0 ? 0 : beta*C_in(i,j)) + (bias ? bias[j] : 0)
 *   ref(i,j) = act(pre(i,j))            act = identity | x*Phi(x) (erf form) | ReLU | SiLU | GELU (tanh form)
 *
 * Storage is row-major: op(A)(i,k) is A[i*lda+k] (transA=0) or A[k*lda+i]
 * (transA=1); op(B)(k,j) is B[k*ldb+j] (transB=0) or B[j*ldb+k] (transB=1);
 * C_in(i,j) is C[i*ldc+j].  Inputs are decoded from the very bit patterns the
 * GPU receives (binary32, binary16, bfloat16), widened exactly to fp64.
 *
 * Every function here is pinned by CPU-only tests to facts that do not come
 * from this file: closed forms (identity, permutation, all-ones), an int64
 * matmul, exact rational arithmetic on tiny shapes, an independent library
 * float codec, and known values of the normal CDF.  Nothing is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* element type codes (an interface constant shared with callers by value only) */
enum { ORACLE_F32 = 0, ORACLE_F16 = 1, ORACLE_BF16 = 2 };
enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_GELU_ERF = 1, ORACLE_ACT_RELU = 2, ORACLE_ACT_SILU = 3, ORACLE_ACT_GELU_TANH = 4 };

typedef struct {
    int64_t M, N, K;
    int32_t transA, transB;
    int32_t ab_dtype;      /* type of A and B */
    int32_t c_dtype;       /* type of C_in (read only when beta != 0) */
    int32_t bias_dtype;    /* type of bias (read only when bias != NULL) */
    int32_t act;
    double alpha, beta;
    const void *A; int64_t lda;
    const void *B; int64_t ldb;
    const void *C; int64_t ldc;   /* may be NULL when beta == 0 */
    const void *bias;             /* length N or NULL */
} oracle_problem_t;

/* ---------- a generic IEEE-style binary format, described by its field widths ---------- */

typedef struct { int mant_bits, exp_bits; } fmt_t;

static fmt_t fmt_of(int dtype) {
    fmt_t f;
    if (dtype == ORACLE_F32)       { f.mant_bits = 23; f.exp_bits = 8; }
    else if (dtype == ORACLE_F16)  { f.mant_bits = 10; f.exp_bits = 5; }
    else                           { f.mant_bits = 7;  f.exp_bits = 8; }
    return f;
}

static int bytes_of(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

/* value of a bit pattern, by the textbook rule (-1)^s * 2^(e-bias) * (1.m), exact in fp64 */
static double decode_bits(fmt_t f, uint32_t bits) {
    const uint32_t mant_mask = (1u << f.mant_bits) - 1u;
    const uint32_t exp_mask = (1u << f.exp_bits) - 1u;
    const uint32_t m = bits & mant_mask;
    const uint32_t e = (bits >> f.mant_bits) & exp_mask;
    const uint32_t s = (bits >> (f.mant_bits + f.exp_bits)) & 1u;
    const int bias = (1 << (f.exp_bits - 1)) - 1;
    double v;
    if (e == exp_mask) v = (m == 0) ? INFINITY : NAN;
    else if (e == 0)   v = ldexp((double)m, 1 - bias - f.mant_bits);              /* subnormal or zero */
    else               v = ldexp((double)(m | (1u << f.mant_bits)), (int)e - bias - f.mant_bits);
    return s ? -v : v;
}

/* nearest representable value, ties to the even significand; overflow to infinity */
static uint32_t encode_bits(fmt_t f, double v) {
    const uint32_t exp_mask = (1u << f.exp_bits) - 1u;
    const int bias = (1 << (f.exp_bits - 1)) - 1;
    const int emin = 1 - bias, emax = bias;
    const uint32_t sign = signbit(v) ? (1u << (f.mant_bits + f.exp_bits)) : 0u;
    if (isnan(v)) return sign | (exp_mask << f.mant_bits) | (1u << (f.mant_bits - 1));
    double a = fabs(v);
    if (isinf(a)) return sign | (exp_mask << f.mant_bits);
    if (a == 0.0) return sign;
    int e2;
    frexp(a, &e2);               /* a = frac * 2^e2, frac in [0.5,1)  =>  a in [2^(e2-1), 2^e2) */
    int E = e2 - 1;
    if (E < emin) E = emin;      /* the subnormal range shares the quantum of emin */
    /* scale so that one unit in the last place is 1.0, then round to integer (ties to even:
       rint under the default rounding mode; the scaling by a power of two is exact) */
    double q = rint(ldexp(a, f.mant_bits - E));
    double r = ldexp(q, E - f.mant_bits);
    if (r == 0.0) return sign;
    frexp(r, &e2);
    E = e2 - 1;                  /* rounding may have carried into the next binade */
    if (E > emax) return sign | (exp_mask << f.mant_bits);
    if (E < emin) {              /* subnormal result: exponent field 0, significand without hidden bit */
        uint32_t m = (uint32_t)ldexp(r, f.mant_bits - emin);
        return sign | m;
    }
    uint32_t m = (uint32_t)(ldexp(r, f.mant_bits - E)) - (1u << f.mant_bits);
    return sign | ((uint32_t)(E + bias) << f.mant_bits) | m;
}

static inline uint32_t load_bits(const void *p, int dtype, int64_t idx) {
    if (dtype == ORACLE_F32) { uint32_t u; memcpy(&u, (const char *)p + 4 * idx, 4); return u; }
    uint16_t h; memcpy(&h, (const char *)p + 2 * idx, 2); return h;
}

static inline double load_value(const void *p, int dtype, int64_t idx) {
    return decode_bits(fmt_of(dtype), load_bits(p, dtype, idx));
}

/* ---------- exported codec entry points ---------- */

double oracle_decode(int dtype, uint32_t bits) { return decode_bits(fmt_of(dtype), bits); }
uint32_t oracle_encode(int dtype, double v) { return encode_bits(fmt_of(dtype), v); }

void oracle_decode_array(int dtype, const void *src, int64_t n, double *dst) {
    for (int64_t i = 0; i < n; ++i) dst[i] = load_value(src, dtype, i);
}

void oracle_encode_array(int dtype, const double *src, int64_t n, void *dst) {
    for (int64_t i = 0; i < n; ++i) {
        uint32_t b = encode_bits(fmt_of(dtype), src[i]);
        if (bytes_of(dtype) == 4) memcpy((char *)dst + 4 * i, &b, 4);
        else { uint16_t h = (uint16_t)b; memcpy((char *)dst + 2 * i, &h, 2); }
    }
}

/* x * Phi(x), Phi the standard normal CDF written with erf */
double oracle_gelu_erf(double x) { return 0.5 * x * (1.0 + erf(x / sqrt(2.0))); }

/* The other activations that a fused epilogue may apply (activation kernels are one of the
 * benchmark families of Section 5.2).  Each is its textbook definition:
 *   ReLU       max(x, 0); a NaN stays a NaN
 *   SiLU       x * sigmoid(x) = x / (1 + exp(-x))
 *   GELU-tanh  x/2 * (1 + tanh( sqrt(2/pi) * (x + 0.044715 x^3) ))   (the tanh approximation of GELU) */
double oracle_relu(double x) { return x != x ? x : (x > 0.0 ? x : 0.0); }
double oracle_silu(double x) { return x / (1.0 + exp(-x)); }
double oracle_gelu_tanh(double x) {
    const double pi = 3.14159265358979323846;
    return 0.5 * x * (1.0 + tanh(sqrt(2.0 / pi) * (x + 0.044715 * x * x * x)));
}
/* act applied to one value; unknown codes are the identity's responsibility of check_problem */
double oracle_act(int act, double x) {
    switch (act) {
        case ORACLE_ACT_GELU_ERF: return oracle_gelu_erf(x);
        case ORACLE_ACT_RELU: return oracle_relu(x);
        case ORACLE_ACT_SILU: return oracle_silu(x);
        case ORACLE_ACT_GELU_TANH: return oracle_gelu_tanh(x);
        default: return x;
    }
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------- the definition, one output element ---------- */

static int check_problem(const oracle_problem_t *p) {
    if (!p || p->M < 0 || p->N < 0 || p->K < 0) return 1;
    if ((p->M > 0 && p->K > 0 && !p->A) || (p->N > 0 && p->K > 0 && !p->B)) return 1;
    if (p->beta != 0.0 && !p->C) return 1;
    if (p->act < ORACLE_ACT_NONE || p->act > ORACLE_ACT_GELU_TANH) return 1;
    return 0;
}

static void element(const oracle_problem_t *p, int64_t i, int64_t j,
                    double *ref, double *sumabs, double *mag) {
    double acc = 0.0, sa = 0.0;
    for (int64_t k = 0; k < p->K; ++k) {
        const int64_t ia = p->transA ? k * p->lda + i : i * p->lda + k;
        const int64_t ib = p->transB ? j * p->ldb + k : k * p->ldb + j;
        const double a = load_value(p->A, p->ab_dtype, ia);
        const double b = load_value(p->B, p->ab_dtype, ib);
        acc += a * b;
        sa += fabs(a * b);
    }
    double pre = p->alpha * acc;
    double m = fabs(p->alpha) * sa;
    if (p->beta != 0.0) {
        const double c = load_value(p->C, p->c_dtype, i * p->ldc + j);
        pre += p->beta * c;
        m += fabs(p->beta * c);
    }
    if (p->bias) {
        const double bj = load_value(p->bias, p->bias_dtype, j);
        pre += bj;
        m += fabs(bj);
    }
    const double out = oracle_act(p->act, pre);
    if (ref) *ref = out;
    if (sumabs) *sumabs = sa;
    if (mag) *mag = m;
}

/*
 * Whole matrix.  ref, sumabs, mag: M*N doubles each, dense row-major (leading
 * dimension N); sumabs and mag may be NULL.
 *   sumabs(i,j) = sum_k |a_ik b_kj|
 *   mag(i,j)    = |alpha| sumabs + |beta C_in| + |bias_j|   (scale of the error bound)
 * Returns 0, or 1 on an invalid problem.
 */
int oracle_gemm_full(const oracle_problem_t *p, double *ref, double *sumabs, double *mag) {
    if (check_problem(p) || !ref) return 1;
    const int64_t total = p->M * p->N;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        const int64_t i = e / p->N, j = e % p->N;
        element(p, i, j, ref + e, sumabs ? sumabs + e : NULL, mag ? mag + e : NULL);
    }
    return 0;
}

/* Listed elements only: (rows[t], cols[t]) for t < n. */
int oracle_gemm_at(const oracle_problem_t *p, const int64_t *rows, const int64_t *cols, int64_t n,
                   double *ref, double *sumabs, double *mag) {
    if (check_problem(p) || !ref || !rows || !cols) return 1;
    for (int64_t t = 0; t < n; ++t)
        if (rows[t] < 0 || rows[t] >= p->M || cols[t] < 0 || cols[t] >= p->N) return 1;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < n; ++t)
        element(p, rows[t], cols[t], ref + t, sumabs ? sumabs + t : NULL, mag ? mag + t : NULL);
    return 0;
}

/* Rows [row0, row0+nrows) of the result, all N columns; ref is nrows*N doubles. */
int oracle_gemm_rows(const oracle_problem_t *p, int64_t row0, int64_t nrows, double *ref) {
    if (check_problem(p) || !ref || row0 < 0 || nrows < 0 || row0 + nrows > p->M) return 1;
    const int64_t total = nrows * p->N;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < total; ++e) {
        const int64_t i = row0 + e / p->N, j = e % p->N;
        element(p, i, j, ref + e, NULL, NULL);
    }
    return 0;
}

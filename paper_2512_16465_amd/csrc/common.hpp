// Internal declarations shared by the kernels of libgemm (device code for gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gemm {

// numeric codes of the public enums (include/gemm.h)
enum : int { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };
enum : int { ACT_NONE = 0, ACT_GELU_ERF = 1, ACT_RELU = 2, ACT_SILU = 3, ACT_GELU_TANH = 4 };

struct Args {
    int64_t M, N, K;
    int32_t transA, transB;
    int32_t dtype, out_dtype, bias_dtype, act;
    float alpha, beta;
    const void* A; int64_t lda;
    const void* B; int64_t ldb;
    void* C; int64_t ldc;
    const void* bias;
    // strided batch: matrix b of each operand starts b * stride elements after the first one;
    // a launch covers `batch` matrices with blockIdx.y (batch == 1: strides unused)
    int64_t strideA, strideB, strideC;
    int32_t batch;
    // k slices: when nonzero, the batch entries are consecutive ranges of K elements of one product
    // whose k extent is k_total (the last range may be shorter); the strides step along k
    int64_t k_total;
};

__host__ __device__ __forceinline__ int elem_bytes(int dtype) { return dtype == DT_F32 ? 4 : 2; }

// First statement of every kernel that takes a batch: point the operands at the matrices of
// this workgroup's batch entry.
__device__ __forceinline__ void select_batch(Args& a) {
    const int64_t b = blockIdx.y;
    a.A = (const char*)a.A + b * a.strideA * elem_bytes(a.dtype);
    a.B = (const char*)a.B + b * a.strideB * elem_bytes(a.dtype);
    a.C = (char*)a.C + b * a.strideC * elem_bytes(a.out_dtype);
    if (a.k_total) {
        const int64_t left = a.k_total - b * a.K;
        a.K = left < a.K ? left : a.K;
    }
}

// Rows of C can be read and written with vectors of four elements (16 bytes of fp32, 8 bytes of a
// 16-bit type) in every matrix of the batch.
inline int c_rows_take_vec4(const Args& a) {
    const int64_t align = a.out_dtype == DT_F32 ? 16 : 8;
    if (a.ldc % 4 != 0 || (uintptr_t)a.C % align != 0) return 0;
    if (a.batch > 1 && (a.strideC * elem_bytes(a.out_dtype)) % align != 0) return 0;
    return 1;
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// ---- scalar conversions (round to nearest even on the way down) ----

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);                                               // ties to even
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) {
    _Float16 h;
    __builtin_memcpy(&h, &b, 2);
    return (float)h;
}

__device__ __forceinline__ uint16_t f32_to_f16_bits(float x) {
    _Float16 h = (_Float16)x;     // v_cvt_f16_f32, round to nearest even
    uint16_t b;
    __builtin_memcpy(&b, &h, 2);
    return b;
}

// element idx of an array whose type is known only at run time (wave-uniform branch)
__device__ __forceinline__ float load_elem(const void* p, int dtype, int64_t idx) {
    if (dtype == DT_F32) return ((const float*)p)[idx];
    const uint16_t b = ((const uint16_t*)p)[idx];
    return dtype == DT_BF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
}

__device__ __forceinline__ void store_elem(void* p, int dtype, int64_t idx, float v) {
    if (dtype == DT_F32) ((float*)p)[idx] = v;
    else if (dtype == DT_BF16) ((uint16_t*)p)[idx] = f32_to_bf16_bits(v);
    else ((uint16_t*)p)[idx] = f32_to_f16_bits(v);
}

// GELU in its exact form x * Phi(x) = x/2 * (1 + erf(x / sqrt 2)).  erf is evaluated with the
// rational approximation 7.1.26 of Abramowitz & Stegun, |error| <= 1.5e-7 over the whole line,
// branch-free (one reciprocal, one exponential, a degree-5 polynomial): two orders of magnitude
// below one rounding of a 16-bit output and far inside the fp32 tolerance, at a quarter of the
// instructions of a libm-grade erff.
__device__ __forceinline__ float gelu_erf(float x) {
    const float z = x * 0.70710678118654752440f;
    const float az = fabsf(z);
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, az, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f(-az * az * 1.44269504088896340736f);
    const float erf_abs = fmaf(-p, e, 1.0f);
    const float erf_z = __builtin_copysignf(erf_abs, z);
    return 0.5f * x * (1.0f + erf_z);
}

// max(x, 0) that keeps a NaN
__device__ __forceinline__ float relu(float x) { return (x > 0.0f || x != x) ? x : 0.0f; }

// x * sigmoid(x) = x / (1 + exp(-x)); exp(-x) overflows to +inf for x < -88 and the quotient
// becomes -0, the limit
__device__ __forceinline__ float silu(float x) {
    const float e = __builtin_amdgcn_exp2f(-x * 1.44269504088896340736f);
    return x * __builtin_amdgcn_rcpf(1.0f + e);
}

// x/2 * (1 + tanh(u)), u = sqrt(2/pi) * (x + 0.044715 x^3), with tanh(u) = 1 - 2 / (1 + exp(2u)):
// one exponential and one reciprocal, saturating correctly at both ends; the cancellation near
// u = 0 costs absolute, not relative, accuracy of tanh and 1 + tanh(u) is near 1 there
__device__ __forceinline__ float gelu_tanh(float x) {
    const float u = 0.7978845608028654f * fmaf(0.044715f * x * x, x, x);
    const float e = __builtin_amdgcn_exp2f(u * 2.88539008177792681472f);
    const float t = fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + e), 1.0f);
    return 0.5f * x * (1.0f + t);
}

__device__ __forceinline__ float apply_act(float x, int act) {
    switch (act) {
        case ACT_GELU_ERF: return gelu_erf(x);
        case ACT_RELU: return relu(x);
        case ACT_SILU: return silu(x);
        case ACT_GELU_TANH: return gelu_tanh(x);
        default: return x;
    }
}

// the activation applied to G vectors of four values, the (wave-uniform) choice made once
template <int G>
__device__ __forceinline__ void apply_act4(f32x4 (&s)[G], int act) {
#define GEMM_ACT_LOOP(F)                    \
    _Pragma("unroll") for (int g = 0; g < G; ++g) \
        _Pragma("unroll") for (int e = 0; e < 4; ++e) s[g][e] = F(s[g][e])
    switch (act) {
        case ACT_GELU_ERF: GEMM_ACT_LOOP(gelu_erf); break;
        case ACT_RELU: GEMM_ACT_LOOP(relu); break;
        case ACT_SILU: GEMM_ACT_LOOP(silu); break;
        case ACT_GELU_TANH: GEMM_ACT_LOOP(gelu_tanh); break;
        default: break;
    }
#undef GEMM_ACT_LOOP
}

// Everything after the contraction, for one element: act(alpha*acc + beta*C_in + bias_j).
// c_in and bias_j are passed already widened; beta == 0 callers pass c_in = 0 without loading it.
__device__ __forceinline__ float epilogue_value(float acc, float alpha, float beta, float c_in, float bias_j, int act) {
    float v = alpha * acc;
    if (beta != 0.0f) v = fmaf(beta, c_in, v);
    v += bias_j;
    return apply_act(v, act);
}

// ---- host-side launchers, one per kernel family; each returns a hipError_t ----

struct TileVariantInfo { const char* name; int BM, BN, BK, threads, kind; };

int tile_num_variants();
const TileVariantInfo* tile_variant_info(int variant);
// true if the call satisfies the alignment/shape preconditions of the macro-tile kernels
bool tile_supports(const Args& a);
// further preconditions of one variant (beyond tile_supports)
bool tile_variant_supports(const Args& a, int variant);
bool shortk_call_fits(const Args& a);
// Split of the trailing tiles along K.  Tiles are numbered in launch order; those with number >=
// first_tile are computed by `parts` workgroups each, every one over a contiguous share of the k
// slabs, which write raw fp32 partial tiles to `partials` ([tile - first_tile][part][BM][BN]);
// launch_tile_split_reduce then adds the parts in order and applies the epilogue.  parts <= 1
// means no split.  It serves grids that fill only a fraction of the last round of workgroups
// (or of the only one).
struct TileSplit { int first_tile; int parts; float* partials; };
bool tile_variant_splits(int variant);
// Variants without that split can still divide K: the launch runs `slices` consecutive k ranges of
// the product as a strided batch (Args::k_total) into fp32 partial results, and
// launch_splitk_reduce adds them.
bool tile_variant_slices(int variant);
hipError_t launch_tile(const Args& a, int variant, int group_m, const TileSplit& split, hipStream_t stream);
hipError_t launch_tile_split_reduce(const Args& a, int variant, int group_m, const TileSplit& split, hipStream_t stream);

bool skinny_supports(const Args& a);
const char* skinny_variant_name(int variant);
// the variant the family prefers for the call, whether `variant` can serve it as well (a call with at most
// 8 rows on a 16-bit weight stored N x K has two), and the largest split factor a variant takes;
// variant < 0 stands for skinny_variant_of(a) everywhere below
int skinny_variant_of(const Args& a);
bool skinny_variant_serves(const Args& a, int variant);
int skinny_max_split(const Args& a, int variant = -1);
// bytes of fp32 workspace the skinny kernel needs for this split factor (0 when split_k == 1)
size_t skinny_workspace_bytes(const Args& a, int split_k);
int skinny_default_split(const Args& a, int num_cus, int variant = -1);
hipError_t launch_skinny(const Args& a, int split_k, float* workspace, hipStream_t stream, int variant = -1);
// Adds `split_k` fp32 partial results `partials[s][M][N]` (rows N apart) in the order of s and applies
// the epilogue of `a` into C.  N must be a multiple of 8.
hipError_t launch_splitk_reduce(const Args& a, int split_k, const float* partials, hipStream_t stream);

// fp32 operands, at most 8 rows: the streaming kernels on the vector ALUs (part of the skinny family)
bool gemv_f32_supports(const Args& a);
int gemv_f32_max_split(const Args& a);
int gemv_f32_default_split(const Args& a, int num_cus);
hipError_t launch_gemv_f32(const Args& a, int split_k, float* workspace, hipStream_t stream);

// bf16 / fp16 operands, at most 8 rows, B stored N x K: the matrix-vector kernel on the vector ALUs (part of the
// skinny family)
bool gemv16_supports(const Args& a);
int gemv16_max_split(const Args& a);
int gemv16_default_split(const Args& a, int num_cus);
hipError_t launch_gemv16(const Args& a, int split_k, float* workspace, hipStream_t stream);

hipError_t launch_general(const Args& a, hipStream_t stream);

}  // namespace gemm

// The general kernel: one thread per output element, any shape, leading dimension, alignment
// and element type.  It is the correctness floor under the matrix-core kernels (calls whose
// operands are not 16-byte aligned, or whose contiguous dimension is not a multiple of 8,
// land here), and it also serves K == 0 and alpha == 0 where only the epilogue is left.
#include "common.hpp"

namespace gemm {

namespace {

constexpr int GT = 16;   // 16 x 16 threads per workgroup

// A small LDS-tiled contraction in fp32: each workgroup computes a 16 x 16 block of C, staging
// 16 x 16 blocks of op(A) and op(B).  Partial sums are folded every 16 terms, which keeps the
// rounding error of long fp32 sums near sqrt-like growth rather than linear in K.
__global__ __launch_bounds__(GT * GT) void general_kernel(Args a) {
    __shared__ float sa[GT][GT + 1];
    __shared__ float sb[GT][GT + 1];
    select_batch(a);
    const int tx = threadIdx.x, ty = threadIdx.y;
    const int64_t tiles_n = (a.N + GT - 1) / GT;
    const int64_t tiles_m = (a.M + GT - 1) / GT;
    const bool skip_product = (a.alpha == 0.0f);
    for (int64_t t = blockIdx.x; t < tiles_m * tiles_n; t += gridDim.x) {
        const int64_t i0 = (t / tiles_n) * GT, j0 = (t % tiles_n) * GT;
        const int64_t i = i0 + ty, j = j0 + tx;
        float acc = 0.0f;
        if (!skip_product) {
            for (int64_t k0 = 0; k0 < a.K; k0 += GT) {
                // sa[r][c] = op(A)(i0 + r, k0 + c); sb[r][c] = op(B)(k0 + r, j0 + c)
                {
                    const int64_t ai = i0 + ty, ak = k0 + tx;
                    float v = 0.0f;
                    if (ai < a.M && ak < a.K)
                        v = load_elem(a.A, a.dtype, a.transA ? ak * a.lda + ai : ai * a.lda + ak);
                    sa[ty][tx] = v;
                    const int64_t bk = k0 + ty, bj = j0 + tx;
                    float w = 0.0f;
                    if (bk < a.K && bj < a.N)
                        w = load_elem(a.B, a.dtype, a.transB ? bj * a.ldb + bk : bk * a.ldb + bj);
                    sb[ty][tx] = w;
                }
                __syncthreads();
                float s = 0.0f;
#pragma unroll
                for (int kk = 0; kk < GT; ++kk) s = fmaf(sa[ty][kk], sb[kk][tx], s);
                acc += s;
                __syncthreads();
            }
        }
        if (i < a.M && j < a.N) {
            const int64_t ci = i * a.ldc + j;
            const float c_in = (a.beta != 0.0f) ? load_elem(a.C, a.out_dtype, ci) : 0.0f;
            const float bj = a.bias ? load_elem(a.bias, a.bias_dtype, j) : 0.0f;
            store_elem(a.C, a.out_dtype, ci, epilogue_value(acc, a.alpha, a.beta, c_in, bj, a.act));
        }
    }
}

}  // namespace

hipError_t launch_general(const Args& a, hipStream_t stream) {
    const int64_t tiles = ((a.M + GT - 1) / GT) * ((a.N + GT - 1) / GT);
    if (tiles == 0) return hipSuccess;
    const int64_t grid = tiles < (1 << 20) ? tiles : (1 << 20);
    hipLaunchKernelGGL(general_kernel, dim3((unsigned)grid, (unsigned)a.batch), dim3(GT, GT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace gemm

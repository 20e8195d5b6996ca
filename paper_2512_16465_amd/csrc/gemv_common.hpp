// Pieces shared by the streaming kernels that run on the vector ALUs (gemv_f32_kernel.hip for fp32
// operands, gemv16_kernel.hip for bf16 / fp16 operands on a weight stored N x K): buffer
// addressing with a masked offset, and the store of one output element.
#pragma once
#include "common.hpp"

namespace gemm {
namespace {

// A byte offset no operand reaches (gemv_*_supports refuse larger ones): a lane that must read
// nothing fetches at this offset and gets zero from the buffer's range check.
constexpr uint32_t GV_MASKED = 0x7ffffff0u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t gv_rsrc(const void* base, int64_t bytes) {
    const int64_t cap = 0xffffffffll;
    const uint32_t n = (uint32_t)(bytes < 0 ? 0 : (bytes > cap ? cap : bytes));
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)n, 0x00020000);
}

__device__ __forceinline__ f32x4 gv_load4(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
}

// 16 bytes with a wave-uniform part of the address in a scalar register.  The range check of the
// buffer looks at `lane_off` alone: GV_MASKED there reads as zero whatever `uniform_off` holds.
__device__ __forceinline__ u32x4 gv_load16(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t uniform_off) {
    return __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, __builtin_amdgcn_readfirstlane(uniform_off), 0));
}

// one output element: the epilogue of the call, or a raw partial sum of slice `slice`
__device__ __forceinline__ void gv_store(const Args& a, int split_k, int slice, float* ws, int64_t row, int64_t col, float x) {
    if (split_k > 1) {
        ws[((int64_t)slice * a.M + row) * a.N + col] = x;
        return;
    }
    const int64_t ci = row * a.ldc + col;
    const float c_in = a.beta != 0.0f ? load_elem(a.C, a.out_dtype, ci) : 0.0f;
    const float bj = a.bias ? load_elem(a.bias, a.bias_dtype, col) : 0.0f;
    store_elem(a.C, a.out_dtype, ci, epilogue_value(x, a.alpha, a.beta, c_in, bj, a.act));
}

}  // namespace
}  // namespace gemm

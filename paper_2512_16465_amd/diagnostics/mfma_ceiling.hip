// What the matrix cores of a gfx950 part sustain when nothing but they works: loops of MFMA
// instructions on operands that sit in registers, no memory traffic inside the timed part.
// A measuring aid for bench.py, not part of the GEMM library and not linked into it: the bench
// quotes the rate of this loop on data drawn like the benchmark's operands beside the rate on
// zeros, so that a reader sees how much of the nominal 2.5 PFLOP/s (2.4 GHz, all pipes full)
// the part's power limit leaves to *any* kernel on such data.
//
// Both loops issue back-to-back independent MFMAs on 256 accumulator registers per lane, the
// same register blocking as the 256x256 macro tile (128x128 per wave): 64 instructions of
// 16x16x32 or 32 instructions of 32x32x16 per pass, one wave per SIMD, one workgroup per CU.
#include <hip/hip_runtime.h>
#include <cstdint>

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

namespace {

constexpr int kThreads = 256;            // 4 waves, one per SIMD
constexpr int kFragments = 16;           // 8 of A and 8 of B, 16 bytes per lane each
constexpr size_t kBytesPerWorkgroup = size_t(kThreads) * kFragments * 16;

// SHAPE 0: v_mfma_f32_32x32x16_bf16, 1: v_mfma_f32_16x16x32_bf16.  Every pass is 2^20 flop per wave.
template <int SHAPE>
__global__ __launch_bounds__(kThreads) void mfma_ceiling_kernel(const u32x4* __restrict__ data, int data_workgroups,
                                                                 int passes, float* sink, long long* stamps) {
  const int tid = threadIdx.x;
  const u32x4* mine = data + size_t(blockIdx.x % data_workgroups) * kThreads * kFragments;
  u32x4 fa[8], fb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    fa[i] = mine[i * kThreads + tid];
    fb[i] = mine[(8 + i) * kThreads + tid];
  }
  float t = 0.f;
  if constexpr (SHAPE == 0) {
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < passes; ++it) {
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int m = 0; m < 16; ++m)
          acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[(m / 4) + 4 * half]),
                                                           __builtin_bit_cast(bf16x8, fb[(m % 4) + 4 * half]), acc[m], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (tid == 0) { stamps[2 * blockIdx.x] = c1 - c0; stamps[2 * blockIdx.x + 1] = w1 - w0; }
#pragma unroll
    for (int i = 0; i < 16; ++i) t += acc[i][0] + acc[i][15];
  } else {
    f32x4 acc[64];
#pragma unroll
    for (int i = 0; i < 64; ++i)
#pragma unroll
      for (int v = 0; v < 4; ++v) acc[i][v] = 0.f;
    const long long c0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < passes; ++it) {
#pragma unroll
      for (int m = 0; m < 64; ++m)
        acc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fa[m / 8]),
                                                         __builtin_bit_cast(bf16x8, fb[m % 8]), acc[m], 0, 0, 0);
    }
    const long long c1 = clock64(), w1 = wall_clock64();
    if (tid == 0) { stamps[2 * blockIdx.x] = c1 - c0; stamps[2 * blockIdx.x + 1] = w1 - w0; }
#pragma unroll
    for (int i = 0; i < 64; ++i) t += acc[i][0] + acc[i][3];
  }
  // keeps the accumulators alive; the comparison is false for every finite sum but -0.0f's bit pattern
  if (__float_as_uint(t) == 0x80000000u) sink[0] = t;
}

}  // namespace

extern "C" {

// Bytes of operand data one workgroup reads before its loop (16 fragments of 16 bytes per lane).
__attribute__((visibility("default"))) size_t mfma_ceiling_bytes_per_workgroup() { return kBytesPerWorkgroup; }

// Flop of one launch: every pass is 2^20 flop per wave in both shapes.
__attribute__((visibility("default"))) double mfma_ceiling_flop(int workgroups, int passes) {
  return double(workgroups) * 4.0 * double(passes) * 1048576.0;
}

// Enqueues one launch on `stream` and returns without waiting.
//   shape           0: 32x32x16 bf16, 1: 16x16x32 bf16
//   workgroups      grid size (one workgroup of 256 lanes fills a compute unit's four SIMDs)
//   passes          loop trips; a pass is 1024 matrix-pipe cycles
//   data            device pointer, data_workgroups * mfma_ceiling_bytes_per_workgroup() bytes of bf16 operand values
//                   (workgroup w reads block w mod data_workgroups); caller owns it
//   sink            device pointer, 4 bytes, never written in practice
//   stamps          device pointer, 2 * workgroups int64: per workgroup the shader-clock cycles and the
//                   100 MHz constant-clock ticks of its loop (clock = cycles / ticks * 0.1 GHz)
// Returns 0, or -1 for an argument out of range, or the hipError_t of the launch.
__attribute__((visibility("default"))) int mfma_ceiling_launch(int shape, int workgroups, int passes, const void* data,
                                                               int data_workgroups, float* sink, long long* stamps, void* stream) {
  if ((shape != 0 && shape != 1) || workgroups < 1 || workgroups > 65536 || passes < 1 || passes > (1 << 20) || !data ||
      data_workgroups < 1 || !sink || !stamps || (reinterpret_cast<uintptr_t>(data) & 15))
    return -1;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (shape == 0)
    hipLaunchKernelGGL(mfma_ceiling_kernel<0>, dim3(workgroups), dim3(kThreads), 0, s, static_cast<const u32x4*>(data),
                       data_workgroups, passes, sink, stamps);
  else
    hipLaunchKernelGGL(mfma_ceiling_kernel<1>, dim3(workgroups), dim3(kThreads), 0, s, static_cast<const u32x4*>(data),
                       data_workgroups, passes, sink, stamps);
  return static_cast<int>(hipGetLastError());
}

}  // extern "C"

// What a kernel that does nothing but read reaches on this part: a grid-stride loop of 16-byte loads
// over a buffer, eight per lane in flight, the words folded into one value that is never stored.
// A measuring aid for bench.py beside the register-only MFMA loops of mfma_ceiling.hip: the
// bandwidth-bound rows of the bench are priced against the nominal 8 TB/s, and this is the share of
// it that plain coalesced reads get.  Not part of the GEMM library.
#include <hip/hip_runtime.h>
#include <cstdint>

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;      // 16-byte loads per lane and trip: 32 KiB per workgroup and trip

__global__ __launch_bounds__(kThreads) void hbm_read_kernel(const u32x4* __restrict__ p, size_t n16, unsigned* sink) {
  size_t i = size_t(blockIdx.x) * kThreads * kUnroll + threadIdx.x;
  const size_t stride = size_t(gridDim.x) * kThreads * kUnroll;
  unsigned acc = 0;
  // n16 is a multiple of kThreads * kUnroll (the launcher checks), so a trip is inside the buffer as a whole
  for (; i < n16; i += stride) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = p[i + size_t(u) * kThreads];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  // keeps the loads alive: the caller's fill makes the folded value of any lane differ from this pattern
  if (acc == 0x9e3779b9u) sink[0] = acc;
}

}  // namespace

extern "C" {

// Enqueues one read of `bytes` bytes at `data` (device pointer, 16-byte aligned, caller owns it) on
// `stream` and returns without waiting.  bytes must be a positive multiple of 32768; workgroups 1 ... 65536.
// sink: device pointer, 4 bytes.  Returns 0, -1 for an argument out of range, or the hipError_t of the launch.
__attribute__((visibility("default"))) int hbm_read_launch(const void* data, size_t bytes, int workgroups, unsigned* sink, void* stream) {
  if (!data || !sink || (reinterpret_cast<uintptr_t>(data) & 15) || bytes == 0 || bytes % (size_t(kThreads) * kUnroll * 16) != 0 ||
      workgroups < 1 || workgroups > 65536)
    return -1;
  hipLaunchKernelGGL(hbm_read_kernel, dim3(workgroups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(data), bytes / 16, sink);
  return static_cast<int>(hipGetLastError());
}

}  // extern "C"

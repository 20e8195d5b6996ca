// Streaming kernel for bf16 / fp16 operands, a weight stored N x K ([out, in]) and very few rows of C
// (M <= 8): the matrix-vector product of a decoding step, the paper's memory-bound kernel
// (Section 5.3).  At one to eight flop per byte of B the call sits left of the lower ridge of the
// roofline (Section 4.3); the vector ALUs are enough, and what the matrix cores would add is padding
// to 16 rows and, in the skinny kernel built on them, a split of k with a second launch.  Here a
// stored row of B is one dot product per row of A and needs no split once there are enough rows:
//
//   a wave owns CB stored rows of B (columns of C) and its lanes lie along k, 8 elements (16 bytes)
//   per lane and 512 per trip, a kilobyte of contiguous memory per wave instruction; A is read the
//   same way (it stays in the caches); both are widened to fp32 in registers and multiplied on the
//   vector ALUs into CB x R fp32 sums per lane, which are folded across the wave after the last trip.
//
// One launch for the whole product; a split of k over workgroups (partial sums added in a fixed order
// by the reduction kernel of the skinny family) only where N alone gives too few workgroups.
// 1 x 8192 x 8192: 21.3 us (6.3 TB/s) against 26.0 for the MFMA kernel with its second launch;
// 1 x 4096 x 4096 (cache resident): 6.4 against 12.0 on split macro tiles.
#include "common.hpp"
#include "gemv_common.hpp"

namespace gemm {

namespace {

constexpr int G16_WAVES = 4;
constexpr int G16_TRIP = 512;            // k per trip of a wave: 64 lanes x 8 elements
constexpr int G16_MAX_ROWS = 8;

// the two 16-bit values of a word as fp32 (exact for both types)
template <bool IS_BF16>
__device__ __forceinline__ void g16_widen(uint32_t w, float& lo, float& hi) {
    if constexpr (IS_BF16) {
        lo = __uint_as_float(w << 16);
        hi = __uint_as_float(w & 0xffff0000u);
    } else {
        typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
        const half2_t v = __builtin_bit_cast(half2_t, w);
        lo = (float)v[0];
        hi = (float)v[1];
    }
}

template <int R, int CB, bool IS_BF16>
__global__ __launch_bounds__(G16_WAVES * 64) void gemv16_nt_kernel(Args a, int split_k, float* ws) {
    static_assert(CB * R <= 64, "one lane per sum stores the result");
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int M = (int)a.M, K = (int)a.K;
    const int64_t N = a.N;

    const int total_trips = (K + G16_TRIP - 1) / G16_TRIP;
    const int per_split = (total_trips + split_k - 1) / split_k;
    const int beg = (int)blockIdx.y * per_split;
    const int end = (beg + per_split) < total_trips ? (beg + per_split) : total_trips;

    const int64_t n0 = (int64_t)blockIdx.x * (G16_WAVES * CB) + wave * CB;
    const __amdgpu_buffer_rsrc_t rb = gv_rsrc(a.B, ((int64_t)(N - 1) * a.ldb + K) * 2);
    const __amdgpu_buffer_rsrc_t ra = gv_rsrc(a.A, ((int64_t)(M - 1) * a.lda + K) * 2);
    uint32_t b_row[CB], a_row[R];          // wave-uniform byte offsets of the rows
#pragma unroll
    for (int c = 0; c < CB; ++c) b_row[c] = (uint32_t)((n0 + c < N ? n0 + c : N - 1) * a.ldb * 2);     // columns >= N repeat a valid one
#pragma unroll
    for (int r = 0; r < R; ++r) a_row[r] = (uint32_t)((int64_t)(r < M ? r : M - 1) * a.lda * 2);      // rows >= M too; neither is stored

    float acc[CB][R];
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[c][r] = 0.0f;

    // K % 8 == 0: a lane's eight elements lie inside or outside K as a whole; outside, both operands are
    // fetched at an offset past the end of either and read as zero
    auto load = [&](u32x4 (&b)[CB], u32x4 (&av)[R], int trip) {
        const int k = trip * G16_TRIP + 8 * lane;
        const uint32_t k_off = k < K ? (uint32_t)k * 2 : GV_MASKED;      // one address register per trip; the rows are scalars
#pragma unroll
        for (int c = 0; c < CB; ++c) b[c] = gv_load16(rb, k_off, b_row[c]);
#pragma unroll
        for (int r = 0; r < R; ++r) av[r] = gv_load16(ra, k_off, a_row[r]);
    };
    auto multiply = [&](const u32x4 (&b)[CB], const u32x4 (&av)[R]) {
        float af[R][8];
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int w = 0; w < 4; ++w) g16_widen<IS_BF16>(av[r][w], af[r][2 * w], af[r][2 * w + 1]);
#pragma unroll
        for (int c = 0; c < CB; ++c) {
            float bf[8];
#pragma unroll
            for (int w = 0; w < 4; ++w) g16_widen<IS_BF16>(b[c][w], bf[2 * w], bf[2 * w + 1]);
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[c][r] = fmaf(af[r][e], bf[e], acc[c][r]);
        }
    };
    // two sets of landing registers; the fences keep the compiler from moving a trip's loads above the
    // multiplications that still read their registers (it would need a third set)
    u32x4 b0[CB], b1[CB], a0[R], a1[R];
    // A fixed position along k is a fixed memory channel whatever the stored row when the rows are a power of two
    // apart, and waves that walked k in step would queue on a few channels: every wave starts at a trip of its
    // own and wraps around (1 x 8192 x 8192: 27.7 -> 21.3 us).  The start must not be the wave's index itself:
    // with rows of 32 KiB, start = index mod 32 puts the same five bits into the address twice, 7 bits apart,
    // and the part's channel choice, which folds higher address bits onto lower ones, cancels them
    // (1 x 16384 x 16384: 106 us; with the index multiplied by 11 and its upper bits added: 86).  The order
    // of a column's sum is a fixed function of its wave.
    const int n_trips = end - beg;
    const unsigned group = (unsigned)blockIdx.x * G16_WAVES + (unsigned)wave;
    const int rot = n_trips > 0 ? (int)((group * 11u + (group >> 5) * 3u) % (unsigned)n_trips) : 0;
    auto trip_at = [&](int i) { const int j = i + rot; return beg + (j >= n_trips ? j - n_trips : j); };
    if (n_trips > 0) {
        int t = 0;
        load(b0, a0, trip_at(0));
        for (; t + 2 < n_trips; t += 2) {
            load(b1, a1, trip_at(t + 1));
            __builtin_amdgcn_sched_barrier(0);
            multiply(b0, a0);
            __builtin_amdgcn_sched_barrier(0);
            load(b0, a0, trip_at(t + 2));
            __builtin_amdgcn_sched_barrier(0);
            multiply(b1, a1);
            __builtin_amdgcn_sched_barrier(0);
        }
        // one or two trips are left, the first of them requested already
        if (t + 1 < n_trips) {
            load(b1, a1, trip_at(t + 1));
            __builtin_amdgcn_sched_barrier(0);
            multiply(b0, a0);
            multiply(b1, a1);
        } else {
            multiply(b0, a0);
        }
    }

    // fold the lanes' partial dot products: after the six exchanges every lane holds every sum
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float v = acc[c][r];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
            acc[c][r] = v;
        }
    // lane c * R + r stores element (row r, column n0 + c)
    float mine = 0.0f;
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
        for (int r = 0; r < R; ++r)
            if (lane == c * R + r) mine = acc[c][r];
    if (lane < CB * R) {
        const int c = lane / R, r = lane % R;
        if (r < M && n0 + c < N) gv_store(a, split_k, (int)blockIdx.y, ws, r, n0 + c, mine);
    }
}

// Stored rows of B per wave.  Four: 16 columns per workgroup keep every compute unit busy from N = 4096 on and
// several workgroups resident per unit beyond (eight rows per wave: 1 x 11008 x 4096 23.1 against 16.6 us,
// 1 x 32000 x 4096 57 against 46).
constexpr int G16_COLS = 4;
int64_t g16_groups(const Args& a) {
    const int64_t cols = G16_WAVES * G16_COLS;
    return (a.N + cols - 1) / cols;
}
int64_t g16_trips(const Args& a) { return (a.K + G16_TRIP - 1) / G16_TRIP; }

}  // namespace

bool gemv16_supports(const Args& a) {
    if ((a.dtype != DT_BF16 && a.dtype != DT_F16) || a.transA || !a.transB) return false;
    if (a.M < 1 || a.M > G16_MAX_ROWS || a.N < 8 || a.K < 8) return false;
    if ((a.N & 7) || (a.K & 7) || (a.lda & 7) || (a.ldb & 7)) return false;          // (the reduction kernel takes 8 columns per thread)
    if (((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return false;
    if (a.N * a.ldb * 2 >= (int64_t)GV_MASKED || a.M * a.lda * 2 >= (int64_t)GV_MASKED) return false;
    if (g16_groups(a) > 65535 * 16) return false;
    return true;
}

int gemv16_max_split(const Args& a) {
    const int64_t s = g16_trips(a) / 4;      // at least four trips per slice
    return (int)(s < 1 ? 1 : (s > 64 ? 64 : s));
}

// A workgroup streams whole stored rows and needs no help from a split once there are enough groups of
// columns; only between a quarter and one group per compute unit do two slices pay for the second kernel.
int gemv16_default_split(const Args& a, int num_cus) {
    const int64_t cus = num_cus > 0 ? num_cus : 256, groups = g16_groups(a), max_s = gemv16_max_split(a);
    int64_t s = (groups * 4 > cus && groups * 2 <= cus) ? 2 : 1;
    if (s > max_s) s = max_s;
    return (int)(s < 1 ? 1 : s);
}

hipError_t launch_gemv16(const Args& a, int split_k, float* workspace, hipStream_t stream) {
    if (!gemv16_supports(a)) return hipErrorInvalidValue;
    if (split_k < 1) split_k = 1;
    const int64_t trips = g16_trips(a);
    if (split_k > trips) split_k = (int)trips;
    if (split_k > 1 && workspace == nullptr) return hipErrorInvalidValue;
    const dim3 grid((unsigned)g16_groups(a), (unsigned)split_k), block(G16_WAVES * 64);
#define GEMM_G16_LAUNCH(R)                                                                                                    \
    do {                                                                                                                      \
        if (a.dtype == DT_BF16) hipLaunchKernelGGL((gemv16_nt_kernel<R, G16_COLS, true>), grid, block, 0, stream, a, split_k, workspace);  \
        else hipLaunchKernelGGL((gemv16_nt_kernel<R, G16_COLS, false>), grid, block, 0, stream, a, split_k, workspace);      \
    } while (0)
    if (a.M == 1) GEMM_G16_LAUNCH(1);
    else if (a.M == 2) GEMM_G16_LAUNCH(2);
    else if (a.M <= 4) GEMM_G16_LAUNCH(4);
    else GEMM_G16_LAUNCH(8);
#undef GEMM_G16_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split_k == 1) return e;
    return launch_splitk_reduce(a, split_k, workspace, stream);
}

}  // namespace gemm

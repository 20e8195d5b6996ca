// Streaming kernels for fp32 operands and very few rows of C (M <= 8): the matrix-vector product
// that the paper uses as its memory-bound kernel (Section 5.3), and its neighbours.  At M/2 flop
// per byte of B the call sits far left of every ridge of the roofline (Section 4.3): the vector
// ALUs are more than enough and the matrix cores have nothing to add, so the kernels are built for
// bytes per second alone -- 16-byte loads, a kilobyte of contiguous memory per wave instruction,
// B read exactly once, and a split of the k range over workgroups whose partial sums are added in
// a fixed order by the reduction kernel of the skinny family.
//
//   B row-major (K x N): a lane owns four consecutive columns, a wave 256; the four waves of a
//     workgroup take a quarter of the workgroup's k range each and add their sums through LDS.
//     The elements of A are wave-uniform and travel through the scalar path.
//   B stored N x K: a wave owns eight stored rows (columns of C) at a time and its lanes lie along
//     k, 256 elements per trip; A is read the same way (it stays in the caches), and the 64 partial
//     dot products of a lane are folded across the wave at the end of the k range.
#include "common.hpp"
#include "gemv_common.hpp"

namespace gemm {

namespace {

constexpr int GV_WAVES = 4;
constexpr int GV_NN_COLS = 256;          // columns per workgroup, row-major B
constexpr int GV_NN_UNROLL = 8;          // k-rows per step
constexpr int GV_NT_COLS_PER_WAVE = 8;   // stored rows of B per wave
constexpr int GV_NT_COLS = GV_WAVES * GV_NT_COLS_PER_WAVE;
constexpr int GV_NT_TRIP = 256;          // k per trip of a wave

template <int R>
__global__ __launch_bounds__(GV_WAVES * 64) void gemv_f32_nn_kernel(Args a, int split_k, float* ws) {
    __shared__ f32x4 red[(GV_WAVES - 1) * R * 64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int M = (int)a.M, K = (int)a.K;
    const int64_t N = a.N;

    // k range of this workgroup and of this wave, in steps of GV_NN_UNROLL rows
    const int total_steps = (K + GV_NN_UNROLL - 1) / GV_NN_UNROLL;
    const int per_split = (total_steps + split_k - 1) / split_k;
    const int wg_beg = (int)blockIdx.y * per_split;
    const int wg_end = (wg_beg + per_split) < total_steps ? (wg_beg + per_split) : total_steps;
    const int wg_steps = wg_end > wg_beg ? wg_end - wg_beg : 0;
    const int per_wave = (wg_steps + GV_WAVES - 1) / GV_WAVES;
    const int my_beg = wg_beg + wave * per_wave;
    const int my_end = (my_beg + per_wave) < wg_end ? (my_beg + per_wave) : wg_end;

    const int64_t col0 = (int64_t)blockIdx.x * GV_NN_COLS + 4 * lane;
    const bool col_ok = col0 < N;                                         // N % 4 == 0: all four or none
    const uint32_t col_off = (uint32_t)((col_ok ? col0 : N - 4) * 4);     // loads stay inside the matrix
    const __amdgpu_buffer_rsrc_t rb = gv_rsrc(a.B, ((int64_t)(K - 1) * a.ldb + N) * 4);     // rows >= K read as zero
    const uint32_t ldb_b = (uint32_t)a.ldb * 4;
    const float* A = (const float*)a.A;

    f32x4 acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto load = [&](f32x4 (&b)[GV_NN_UNROLL], int step) {
        uint32_t off = (uint32_t)(step * GV_NN_UNROLL) * ldb_b + col_off;
#pragma unroll
        for (int u = 0; u < GV_NN_UNROLL; ++u) {
            b[u] = gv_load4(rb, off);
            off += ldb_b;
        }
    };
    auto multiply = [&](const f32x4 (&b)[GV_NN_UNROLL], int step) {
        const int k0 = step * GV_NN_UNROLL;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const float* ar = A + (int64_t)(r < M ? r : M - 1) * a.lda;      // rows >= M repeat a valid one and are never stored
#pragma unroll
            for (int u = 0; u < GV_NN_UNROLL; ++u) {
                const float av = k0 + u < K ? ar[k0 + u] : 0.0f;            // wave-uniform
                acc[r] += av * b[u];
            }
        }
    };
    f32x4 b0[GV_NN_UNROLL], b1[GV_NN_UNROLL];
    if (my_beg < my_end) load(b0, my_beg);
    for (int s = my_beg; s < my_end; s += 2) {
        if (s + 1 < my_end) load(b1, s + 1);
        multiply(b0, s);
        if (s + 2 < my_end) load(b0, s + 2);
        if (s + 1 < my_end) multiply(b1, s + 1);
    }

    // waves 1 .. 3 park their sums; wave 0 adds them in the order of the waves
    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) red[((wave - 1) * R + r) * 64 + lane] = acc[r];
    }
    __syncthreads();
    if (wave == 0 && col_ok) {
#pragma unroll
        for (int w = 0; w < GV_WAVES - 1; ++w)
#pragma unroll
            for (int r = 0; r < R; ++r) acc[r] += red[(w * R + r) * 64 + lane];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r >= M) break;
#pragma unroll
            for (int e = 0; e < 4; ++e) gv_store(a, split_k, (int)blockIdx.y, ws, r, col0 + e, acc[r][e]);
        }
    }
}

template <int R>
__global__ __launch_bounds__(GV_WAVES * 64) void gemv_f32_nt_kernel(Args a, int split_k, float* ws) {
    constexpr int CB = GV_NT_COLS_PER_WAVE;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int M = (int)a.M, K = (int)a.K;
    const int64_t N = a.N;

    const int total_trips = (K + GV_NT_TRIP - 1) / GV_NT_TRIP;
    const int per_split = (total_trips + split_k - 1) / split_k;
    const int beg = (int)blockIdx.y * per_split;
    const int end = (beg + per_split) < total_trips ? (beg + per_split) : total_trips;

    const int64_t n0 = (int64_t)blockIdx.x * GV_NT_COLS + wave * CB;
    const __amdgpu_buffer_rsrc_t rb = gv_rsrc(a.B, ((int64_t)(N - 1) * a.ldb + K) * 4);
    const __amdgpu_buffer_rsrc_t ra = gv_rsrc(a.A, ((int64_t)(M - 1) * a.lda + K) * 4);
    uint32_t b_row[CB], a_row[R];
#pragma unroll
    for (int c = 0; c < CB; ++c) b_row[c] = (uint32_t)((n0 + c < N ? n0 + c : N - 1) * a.ldb * 4);     // columns >= N repeat a valid one
#pragma unroll
    for (int r = 0; r < R; ++r) a_row[r] = (uint32_t)((int64_t)(r < M ? r : M - 1) * a.lda * 4);

    float acc[CB][R];
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
        for (int r = 0; r < R; ++r) acc[c][r] = 0.0f;

    // K % 4 == 0: a lane's four elements lie inside or outside K as a whole; outside, both operands
    // are fetched at an offset past the end of either and read as zero
    auto load = [&](f32x4 (&b)[CB], f32x4 (&av)[R], int trip) {
        const int k = trip * GV_NT_TRIP + 4 * lane;
        const uint32_t k_off = k < K ? (uint32_t)k * 4 : GV_MASKED;      // one address register per trip; the rows are scalars
#pragma unroll
        for (int c = 0; c < CB; ++c) b[c] = __builtin_bit_cast(f32x4, gv_load16(rb, k_off, b_row[c]));
#pragma unroll
        for (int r = 0; r < R; ++r) av[r] = __builtin_bit_cast(f32x4, gv_load16(ra, k_off, a_row[r]));
    };
    auto multiply = [&](const f32x4 (&b)[CB], const f32x4 (&av)[R]) {
#pragma unroll
        for (int c = 0; c < CB; ++c)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[c][r] = fmaf(av[r][e], b[c][e], acc[c][r]);
    };
    // A fixed position along k is a fixed memory channel whatever the stored row when the rows are a power of two
    // apart, and waves that walked k in step would queue on a few channels: every wave starts at a trip of its
    // own and wraps around.  The start is not the wave's index itself (with rows of 32 KiB that puts the same
    // bits into the address twice, and the part's channel choice folds them onto each other: 8 x 8192 x 8192
    // 58 -> 65 us) but the index multiplied by 11 with its upper bits added.  The order of a column's sum is a
    // fixed function of its wave.
    const int n_trips = end - beg;
    const unsigned walker = (unsigned)blockIdx.x * GV_WAVES + (unsigned)wave;
    const int rot = n_trips > 0 ? (int)((walker * 11u + (walker >> 5) * 3u) % (unsigned)n_trips) : 0;
    auto trip_at = [&](int i) { const int j = i + rot; return beg + (j >= n_trips ? j - n_trips : j); };
    // two sets of landing registers; the fences keep the compiler from moving a trip's loads above the
    // multiplications that still read their registers (it would need a third set)
    f32x4 b0[CB], b1[CB], a0[R], a1[R];
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

}  // namespace

bool gemv_f32_supports(const Args& a) {
    if (a.dtype != DT_F32 || a.transA) return false;
    if (a.M < 1 || a.M > 8 || a.N < 8 || a.K < 4) return false;
    if ((a.N & 7) || (a.K & 3) || (a.lda & 3) || (a.ldb & 3)) return false;          // (the reduction kernel takes 8 columns per thread)
    if (((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return false;
    const int64_t b_bytes = a.transB ? a.N * a.ldb * 4 : (a.K + GV_NN_UNROLL) * a.ldb * 4;
    if (b_bytes >= (int64_t)GV_MASKED || a.M * a.lda * 4 >= (int64_t)GV_MASKED) return false;
    return true;
}

// units the k range is cut in
static int64_t gemv_f32_k_units(const Args& a) { return a.transB ? (a.K + GV_NT_TRIP - 1) / GV_NT_TRIP : (a.K + GV_NN_UNROLL - 1) / GV_NN_UNROLL; }
static int64_t gemv_f32_groups(const Args& a) { return a.transB ? (a.N + GV_NT_COLS - 1) / GV_NT_COLS : (a.N + GV_NN_COLS - 1) / GV_NN_COLS; }

int gemv_f32_max_split(const Args& a) {
    // at least four trips (B stored N x K) or 16 steps per wave (row-major B) per slice
    const int64_t s = a.transB ? gemv_f32_k_units(a) / 4 : gemv_f32_k_units(a) / (GV_WAVES * 16);
    return (int)(s < 1 ? 1 : (s > 64 ? 64 : s));
}

// Measured on 2048^2 ... 16384^2 weights with 1, 4 and 8 rows.  Row-major B: one workgroup per compute
// unit (two with more than four rows, whose steps are long) - 1 x 8192 x 8192: 49 us in 8 slices, 56 in
// 16, 84 in 2.  B stored N x K: a workgroup streams whole stored rows and needs no help from a split
// once there are enough column groups; with at most half a group per unit the slices that fill the units
// pay for the second kernel from 32 MiB on (8 x 4096 x 4096: 20 us in 2 slices, 22 whole; 1 x 2048 x 2048,
// 16 MiB: 7 whole, 10 in 2).
int gemv_f32_default_split(const Args& a, int num_cus) {
    const int64_t cus = num_cus > 0 ? num_cus : 256, groups = gemv_f32_groups(a), max_s = gemv_f32_max_split(a);
    int64_t s;
    // (with at most half a group per unit and 32 MiB or more to stream, as many slices as fill the units:
    // 8 x 2048 x 8192 36 us whole, 21 in 4 slices)
    if (a.transB) s = (groups * 2 <= cus && a.N * a.K * 4 >= ((int64_t)32 << 20)) ? cus / groups : 1;
    else s = ((a.M > 4 ? 2 : 1) * cus + groups - 1) / groups;
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    return (int)s;
}

hipError_t launch_gemv_f32(const Args& a, int split_k, float* workspace, hipStream_t stream) {
    if (split_k < 1) split_k = 1;
    const int64_t units = gemv_f32_k_units(a);
    if (split_k > units) split_k = (int)units;
    if (split_k > 1 && workspace == nullptr) return hipErrorInvalidValue;
    const dim3 grid((unsigned)gemv_f32_groups(a), (unsigned)split_k), block(GV_WAVES * 64);
#define GEMM_GEMV_LAUNCH(KERNEL)                                                                      \
    do {                                                                                              \
        if (a.M == 1) hipLaunchKernelGGL((KERNEL<1>), grid, block, 0, stream, a, split_k, workspace); \
        else if (a.M <= 4) hipLaunchKernelGGL((KERNEL<4>), grid, block, 0, stream, a, split_k, workspace); \
        else hipLaunchKernelGGL((KERNEL<8>), grid, block, 0, stream, a, split_k, workspace);          \
    } while (0)
    if (a.transB) GEMM_GEMV_LAUNCH(gemv_f32_nt_kernel);
    else GEMM_GEMV_LAUNCH(gemv_f32_nn_kernel);
#undef GEMM_GEMV_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split_k == 1) return e;
    return launch_splitk_reduce(a, split_k, workspace, stream);
}

}  // namespace gemm

// The skinny kernels: M <= 64 rows of C, bf16 / fp16 operands, A row-major (k contiguous) and
// B row-major K x N (n contiguous) -- the decode-shaped product whose cost is reading B once.
// By the paper's roofline rule (Section 4.3) such a call sits left of the matrix-core ridge, so
// the objective is memory throughput, not matrix-core occupancy: B streams HBM -> registers
// with no LDS staging, many 16-byte loads in flight per wave, and the K range is split over
// waves (reduced through LDS) and over workgroups (reduced through an fp32 workspace in a
// fixed order, so results are reproducible bit for bit).
//
// Data path of one wave for one step of 16 along k and 256 columns:
//   lane (c = lane%32, h = lane/32) loads rows k0+8h .. k0+8h+7 of B, columns 8c .. 8c+7
//   (eight 16-byte loads), transposes the 8x8 block of 16-bit values in registers with
//   v_perm_b32, and so holds, for each j < 8, the B operand of a 32x32x16 MFMA for column
//   8c+j.  MFMA j accumulates C[0:32, {8c+j : c}]; a lane ends up owning 8 consecutive columns
//   of 16 rows, which it stores as full 16- or 32-byte vectors.
#include <type_traits>
#include "common.hpp"

namespace gemm {

namespace {

constexpr int SK_COLS = 256;     // columns per workgroup
constexpr int SK_WAVES = 4;      // waves per workgroup (one per SIMD), each a slice of the workgroup's k range
constexpr int SK_DEPTH = 3;      // steps of 16 k-rows in flight per wave (8 KiB each)
constexpr int SK_MAX_ROWS = 64;  // rows of C the skinny kernels take
// Up to here a 16-bit weight stored N x K goes to the vector-ALU kernel (variant 4): with 1, 2 and 4 rows it is ahead of
// the MFMA kernel on every weight measured (1 x 8192 x 8192 21.3 against 26.0 us, 4 x 28672 x 8192 78 against 79.5) or
// level (4 x 16384 x 16384 90.4 against 89.5); with 8 rows its multiplications show (8 x 8192 x 8192 29 against 27.5,
// 8 x 28672 x 8192 102 against 79).
constexpr int SK_GEMV16_ROWS = 4;
// The kernel with 16 columns per workgroup (variant 5) takes up to 16 rows and is preferred where N / 16 workgroups
// are one round of the chip at most, each with a k range long enough to fill its ring, on a weight below 128 MiB:
// 8 x 4096 x 4096 8.7 us against 12.3 on split tiles and 16.3 in the wide kernel, 16 x 4096 x 4096 10.0 against 12.2,
// 8 x 1024 x 8192 10.6 against 14.2, 8 x 4096 x 14336 21.8 against 24.2.  Beyond N = 4096 the short-lived
// workgroups lose (8 x 11008 x 4096 25.8 against 20.4 wide, 8 x 16384 x 2048 29.6 against 17.3), and with 32 rows
// (two row blocks, three visits in flight) it lost everywhere: that instance is not built.
constexpr int SK_NARROW_ROWS = 16;
// (a short k does not hurt it: 8 x 4096 x 256 7.2 us against 8.1, 8 x 1024 x 1024 7.7 against 10.4, 16 x 4096 x 512 7.4 against 9.3)
constexpr int64_t SK_NARROW_BYTES = (int64_t)128 << 20, SK_NARROW_MAX_N = 4096, SK_NARROW_MIN_K = 256;
// Up to three rounds of workgroups it still pays with two visits in flight per wave, so that two workgroups share a
// compute unit and fill each other's gaps, where k is long enough: 8 x 8192 x 8192 25.0 us against 27.5 wide,
// 8 x 8192 x 4096 14.6 against 17.4 on split tiles, 8 x 11008 x 4096 19.9 against 20.4 wide and 23.3 on tiles; not
// beyond (8 x 32000 x 4096 56 against 52.5, 16 x 28672 x 8192 96 against 79).
// With 9 to 16 rows the partly filled last round shows: 16 x 5120 x 5120 18.2 against 15.4 on split tiles (320 workgroups
// on 512 places), 16 x 9216 x 4608 22.7 against 20.1 (576 on 1024), but 16 x 11008 x 4096 22.0 against 23.3 (688 on 1024):
// then the places must be 65 % full.  The places are those of a 256-unit part.
constexpr int64_t SK_NARROW_FAR_N = 12288, SK_NARROW_FAR_K = 1024, SK_NARROW_PLACES = 512;
constexpr uint32_t SK_MASKED = 0x7ffffff0u;   // an offset past the end of any operand: the load returns zero

__device__ __forceinline__ __amdgpu_buffer_rsrc_t sk_rsrc(const void* base, int64_t bytes) {
    const int64_t cap = 0xffffffffll;
    const uint32_t n = (uint32_t)(bytes < 0 ? 0 : (bytes > cap ? cap : bytes));
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)n, 0x00020000);
}

template <bool IS_BF16>
__device__ __forceinline__ f32x16 sk_mfma(u32x4 a, u32x4 b, f32x16 c) {
    if constexpr (IS_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

template <int MB>
struct SkStage {
    u32x4 a[MB];
    u32x4 b[8];
};

// C_in and bias of 8 consecutive outputs of one row, widened to fp32 (zeros where the epilogue
// does not use them).  Separate from the store so that a caller can have these loads in flight
// together with the loads of its partial sums.
struct SkRowInputs { float c_in[8]; float bias[8]; };

__device__ __forceinline__ void sk_unpack16(u32x4 u, int dtype, float (&out)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const uint16_t b = (uint16_t)(u[e >> 1] >> (16 * (e & 1)));
        out[e] = dtype == DT_BF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
    }
}

__device__ __forceinline__ void sk_load_row_inputs(const Args& a, int64_t row, int64_t col, bool vec_ok, SkRowInputs& in) {
    const int64_t idx = row * a.ldc + col;
    if (a.beta != 0.0f) {
        if (vec_ok && a.out_dtype != DT_F32) {
            sk_unpack16(*(const u32x4*)((const uint16_t*)a.C + idx), a.out_dtype, in.c_in);
        } else if (vec_ok) {
            const f32x4 lo = *(const f32x4*)((const float*)a.C + idx), hi = *(const f32x4*)((const float*)a.C + idx + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { in.c_in[e] = lo[e]; in.c_in[4 + e] = hi[e]; }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) in.c_in[e] = load_elem(a.C, a.out_dtype, idx + e);
        }
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) in.c_in[e] = 0.0f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) in.bias[e] = a.bias ? load_elem(a.bias, a.bias_dtype, col + e) : 0.0f;
}

// Stores 8 consecutive outputs of one row, after the epilogue, in the type of C.
__device__ __forceinline__ void sk_store_row(const Args& a, int64_t row, int64_t col, const float (&x)[8], const SkRowInputs& in, bool vec_ok) {
    float o[8];
    const int64_t idx = row * a.ldc + col;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = epilogue_value(x[e], a.alpha, a.beta, in.c_in[e], in.bias[e], a.act);
    if (a.out_dtype == DT_F32) {
        float* p = (float*)a.C + idx;
        if (vec_ok) {
            *(f32x4*)p = f32x4{o[0], o[1], o[2], o[3]};
            *(f32x4*)(p + 4) = f32x4{o[4], o[5], o[6], o[7]};
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = o[e];
        }
    } else {
        uint16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = a.out_dtype == DT_BF16 ? f32_to_bf16_bits(o[e]) : f32_to_f16_bits(o[e]);
        uint16_t* p = (uint16_t*)a.C + idx;
        if (vec_ok) {
            u32x4 u;
#pragma unroll
            for (int e = 0; e < 4; ++e) u[e] = (uint32_t)h[2 * e] | ((uint32_t)h[2 * e + 1] << 16);
            *(u32x4*)p = u;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) p[e] = h[e];
        }
    }
}

// MB = number of 32-row blocks of C: 1 serves M <= 32, 2 serves M <= 64 (every piece of B that a
// wave has transposed then feeds two MFMAs instead of one; B is still read once).
template <bool IS_BF16, int MB>
__global__ __launch_bounds__(SK_WAVES * 64) void skinny_nn_kernel(Args a, int split_k, float* ws, int c_vec_ok) {
    // partial accumulators of the upper half of the waves, [wave][row block][register quad][lane]
    __shared__ f32x4 red[(SK_WAVES / 2) * MB * 32 * 64];

    constexpr int DEPTH = MB == 1 ? SK_DEPTH : 2;        // steps in flight per wave; two row blocks leave registers for two
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int M = (int)a.M, K = (int)a.K;
    const int64_t N = a.N;

    // k range of this workgroup and of this wave, in steps of 16
    const int total_steps = (K + 15) / 16;
    const int per_split = (total_steps + split_k - 1) / split_k;
    const int wg_beg = blockIdx.y * per_split;
    const int wg_end = (wg_beg + per_split) < total_steps ? (wg_beg + per_split) : total_steps;
    const int wg_steps = wg_end > wg_beg ? wg_end - wg_beg : 0;
    const int per_wave = (wg_steps + SK_WAVES - 1) / SK_WAVES;
    const int my_beg = wg_beg + wave * per_wave;
    const int my_end = (my_beg + per_wave) < wg_end ? (my_beg + per_wave) : wg_end;

    const int64_t col0 = (int64_t)blockIdx.x * SK_COLS + 8 * l32;       // first of this lane's 8 columns
    const bool col_ok = col0 < N;                                        // N % 8 == 0: all 8 or none
    const int64_t col_ld = col_ok ? col0 : N - 8;                        // loads stay inside the matrix

    const __amdgpu_buffer_rsrc_t rb = sk_rsrc(a.B, ((int64_t)(K - 1) * a.ldb + N) * 2);   // rows >= K read as zero
    const __amdgpu_buffer_rsrc_t ra = sk_rsrc(a.A, ((int64_t)(M - 1) * a.lda + K) * 2);
    const uint32_t ldb_b = (uint32_t)a.ldb * 2;
    uint32_t a_row_off[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int r = 32 * mb + l32;
        a_row_off[mb] = (uint32_t)((r < M ? r : M - 1) * a.lda * 2);     // rows >= M are computed from a valid row, never stored
    }

    f32x16 acc[MB][8];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][j][v] = 0.0f;

    auto load = [&](SkStage<MB>& st, int step) {
        const int k = step * 16 + 8 * lhi;
        // A: 8 consecutive k of row a_row; K % 8 == 0, so the chunk is inside or outside as a whole.
        // Outside, the lane asks for an offset past the end of A and gets zeros (clearing the
        // register after the load would be a write behind a load in flight, which waits for it).
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
            st.a[mb] = __builtin_amdgcn_raw_buffer_load_b128(ra, k < K ? a_row_off[mb] + (uint32_t)k * 2 : SK_MASKED, 0, 0);
        uint32_t off = (uint32_t)k * ldb_b + (uint32_t)col_ld * 2;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            st.b[j] = __builtin_amdgcn_raw_buffer_load_b128(rb, off, 0, 0);
            off += ldb_b;
        }
    };
    // One step: transpose the stage's 8x8 blocks, then at once refill the stage with the step two
    // ahead (so that the loads are not held up behind the MFMAs, which issue slowly while the
    // other wave of the SIMD owns the matrix pipe), then the eight MFMAs.
    auto process = [&](SkStage<MB>& st, int refill_step, bool refill) {
        u32x4 o[8];
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const uint32_t sel = (n & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
            for (int kp = 0; kp < 4; ++kp)
                o[n][kp] = __builtin_amdgcn_perm(st.b[2 * kp + 1][n >> 1], st.b[2 * kp][n >> 1], sel);
        }
        u32x4 a_cur[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) a_cur[mb] = st.a[mb];
        if (refill) load(st, refill_step);
#pragma unroll
        for (int n = 0; n < 8; ++n)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) acc[mb][n] = sk_mfma<IS_BF16>(a_cur[mb], o[n], acc[mb][n]);
    };

    SkStage<MB> st[DEPTH];
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
        if (my_beg + d < my_end) load(st[d], my_beg + d);
    for (int s = my_beg; s < my_end; s += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (s + d < my_end) process(st[d], s + d + DEPTH, s + d + DEPTH < my_end);
    }

    // fold the waves' partial sums pairwise through LDS: (0..3)+=(4..7), (0,1)+=(2,3), 0+=1
#pragma unroll
    for (int half = SK_WAVES / 2; half >= 1; half >>= 1) {
        if (wave >= half && wave < 2 * half) {
            f32x4* dst = red + (wave - half) * MB * 32 * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
#pragma unroll
                    for (int c = 0; c < 4; ++c)
                        dst[((mb * 8 + j) * 4 + c) * 64] =
                            f32x4{acc[mb][j][4 * c], acc[mb][j][4 * c + 1], acc[mb][j][4 * c + 2], acc[mb][j][4 * c + 3]};
                    asm volatile("" ::: "memory");      // one accumulator at a time: no need to hold them all in vector registers
                }
        }
        __syncthreads();
        if (wave < half) {
            const f32x4* src = red + wave * MB * 32 * 64 + lane;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const f32x4 t = src[((mb * 8 + j) * 4 + c) * 64];
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[mb][j][4 * c + e] += t[e];
                    }
                    asm volatile("" ::: "memory");
                }
        }
        __syncthreads();
    }

    if (wave == 0 && col_ok) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * mb + 8 * (v >> 2) + 4 * lhi + (v & 3);
            if (row < M) {
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = acc[mb][j][v];
                if (split_k > 1) {
                    float* p = ws + ((int64_t)blockIdx.y * M + row) * N + col0;
                    *(f32x4*)p = f32x4{x[0], x[1], x[2], x[3]};
                    *(f32x4*)(p + 4) = f32x4{x[4], x[5], x[6], x[7]};
                } else {
                    SkRowInputs in;
                    sk_load_row_inputs(a, row, col0, c_vec_ok != 0, in);
                    sk_store_row(a, row, col0, x, in, c_vec_ok != 0);
                }
            }
        }
    }
}

// ---- B stored N x K ("column-major B", the layout of a weight matrix kept as [out, in]) ----
//
// Every row of the stored B is one column of the product and is contiguous along k, so 16 bytes
// of it are an MFMA operand as they come (16x16x32 MFMA: lane (c = lane%16, g = lane/16) holds
// B[n + c][k + 8g .. +7]).  Loading them in that lane order would make neighbouring lanes fetch
// from stored rows tens of kilobytes apart, one cache line per lane, and the address path of the
// memory pipeline, not HBM, would set the pace.  So B goes through LDS instead, with loads whose
// 64 lanes cover two stored rows x 512 contiguous bytes (eight whole cache lines) and write
// straight to LDS (no registers): a "visit" is eight such instructions = 16 stored rows x 512 B
// = 8 KiB, each wave keeps a private ring of ST_DEPTH visits, and the MFMA operands are read back
// with ds_read_b128.  Layout of a visit in LDS: row r (of 16), 16-byte slot s (of 32) at
// r*512 + s*16 holds piece s xor r of the row, so that the 16 lanes of an operand read (16 rows,
// same piece) hit 16 different bank groups; the swizzle is applied on the global side, where a
// lane simply fetches the piece that belongs in its slot.
//
// A wave owns 64 columns of C (four blocks of 16, visited in turn for every chunk of 256 along
// k) over the workgroup's whole k range, so waves never add their sums to each other.  The
// pieces of A for a chunk go to registers with the chunk's first visit and serve all four
// blocks (the four waves of a workgroup read the same pieces: one trip to L2, three hits in L1).
// The k range is cut over workgroups exactly as in the row-major kernel.
//   accumulator register v of MFMA (h, jb) is C[16h + 4g + v][n0 + 16jb + c].
constexpr int ST_COLS = 256;
constexpr int ST_WAVES = 4;
constexpr int ST_RUN = 8;                        // MFMA steps (32 along k) per visit: 512 contiguous bytes per stored row
constexpr int ST_DEPTH = 4;                      // visits in flight per wave
constexpr int ST_CHUNK = ST_RUN * 32;            // k per chunk
constexpr int ST_VISIT_BYTES = 16 * ST_RUN * 64; // 8 KiB
constexpr uint32_t ST_MASKED = SK_MASKED;

template <bool IS_BF16>
__device__ __forceinline__ f32x4 st_mfma(u32x4 a, u32x4 b, f32x4 c) {
    if constexpr (IS_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Lane l fetches 16 bytes at byte offset `off` of the buffer; the wave's 64 pieces land at LDS
// address dst + 16*l.  (Only the device pass of the compiler knows the builtin.)
__device__ __forceinline__ void st_load_to_lds(__amdgpu_buffer_rsrc_t rsrc, char* dst, uint32_t off) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)dst, 16, off, 0, 0, 0);
#else
    (void)rsrc; (void)dst; (void)off;
#endif
}

// Waits until at most N vector-memory loads issued by this wave are still in flight (they finish
// in the order of issue).
template <int N>
__device__ __forceinline__ void st_wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// H = number of 16-row blocks of C: 1 serves M <= 16, 2 serves M <= 32, 4 serves M <= 64.
template <bool IS_BF16, int H>
__global__ __launch_bounds__(ST_WAVES * 64) void skinny_nt_kernel(Args a, int split_k, float* ws) {
    static_assert(ST_DEPTH == 4 && ST_RUN == 8, "the visit loop and the load counts below are written for a ring of four visits of eight steps");
    __shared__ __attribute__((aligned(1024))) char ring[ST_WAVES * ST_DEPTH * ST_VISIT_BYTES];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c16 = lane & 15, g = lane >> 4;
    const int M = (int)a.M, K = (int)a.K;
    const int64_t N = a.N;

    const int total_chunks = (K + ST_CHUNK - 1) / ST_CHUNK;
    const int per_split = (total_chunks + split_k - 1) / split_k;
    const int cbeg = blockIdx.y * per_split;
    const int cend = (cbeg + per_split) < total_chunks ? (cbeg + per_split) : total_chunks;
    const int nch = cend > cbeg ? cend - cbeg : 0;
    const int nvis = nch * 4;                                  // visit v: chunk number v/4 of this workgroup, column block v%4
    // The stored rows of B are a large power of two apart, so one position along k means one
    // memory channel whatever the row: workgroups that walked k in step would all queue on the
    // same few channels.  Every column group therefore starts at a chunk of its own and wraps
    // around (the order of summation is a fixed function of the column group).
    const int rot = nch > 0 ? (int)(((unsigned)blockIdx.x * 11u + ((unsigned)blockIdx.x >> 5) * 3u) % (unsigned)nch) : 0;
    auto chunk_of = [&](int v) {      // for v < nvis
        const int c = (v >> 2) + rot;
        return cbeg + (c >= nch ? c - nch : c);
    };

    const int64_t n0 = (int64_t)blockIdx.x * ST_COLS + wave * 64;
    const __amdgpu_buffer_rsrc_t rb = sk_rsrc(a.B, ((int64_t)(N - 1) * a.ldb + K) * 2);
    const __amdgpu_buffer_rsrc_t ra = sk_rsrc(a.A, ((int64_t)(M - 1) * a.lda + K) * 2);

    // global side of a visit: instruction i fetches stored rows 2i and 2i+1 of the block; this
    // lane serves row 2i + lr, slot ls, i.e. piece ls xor (2i + lr) of that row
    const int lr = lane >> 5, ls = lane & 31;
    const int n_first = (int)n0, n_last = (int)N - 1;
    const uint32_t ldb_b = (uint32_t)a.ldb * 2;
    char* const my_ring = ring + wave * (ST_DEPTH * ST_VISIT_BYTES);
    // LDS side: operand of step t for this lane = row c16, piece 4t + g, kept in slot (4t + g) xor c16
    uint32_t frag_addr[ST_RUN];
#pragma unroll
    for (int t = 0; t < ST_RUN; ++t)
        frag_addr[t] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)my_ring + (uint32_t)(c16 * 512 + (((4 * t + g) ^ c16) << 4));

    uint32_t a_row_off[H];
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const int r = 16 * h + c16;
        a_row_off[h] = (uint32_t)((r < M ? r : M - 1) * a.lda * 2);     // rows >= M repeat a valid one and are never stored
    }

    f32x4 acc[H][4];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int jb = 0; jb < 4; ++jb) acc[h][jb] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 aq[2][H][ST_RUN];              // pieces of A of the chunk in work and of the next one

    // K % 8 == 0: a piece of 8 lies inside or outside as a whole; outside, both operands read as
    // zero (what follows a row in memory is the next row or padding, not zeros)
    // Every visit slot of the loop below issues its loads whether the visit exists or not (a
    // visit past the end fetches nothing: all its offsets are masked and read as zero), so the
    // number of loads in flight behind any given one is the same on every path and the waits,
    // the compiler's for A and the explicit ones for B, can be exact.
    auto load_visit = [&](auto slot_c, auto jb_c, auto par_c, int v) {
        constexpr int slot = decltype(slot_c)::value, jb = decltype(jb_c)::value, par = decltype(par_c)::value;
        const bool live = v < nvis;
        const int chunk = chunk_of(v);
        if constexpr (jb == 0) {
            const int kbase = chunk * ST_CHUNK + 8 * g;
#pragma unroll
            for (int t = 0; t < ST_RUN; ++t) {
                const int k = kbase + 32 * t;
#pragma unroll
                for (int h = 0; h < H; ++h)
                    aq[par][h][t] = __builtin_amdgcn_raw_buffer_load_b128(ra, (live && k < K) ? a_row_off[h] + (uint32_t)k * 2 : ST_MASKED, 0, 0);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rl = 2 * i + lr;                                   // row of the block
            const int n = n_first + 16 * jb + rl;
            const int k = chunk * ST_CHUNK + ((ls ^ rl) << 3);
            const uint32_t off = (uint32_t)(n < n_last ? n : n_last) * ldb_b + (uint32_t)k * 2;   // columns >= N repeat a valid one and are never stored
            const uint32_t masked_off = (live && k < K) ? off : ST_MASKED;
            st_load_to_lds(rb, my_ring + slot * ST_VISIT_BYTES + i * 1024, masked_off);
        }
    };
    // visit d of a group of eight (two chunks): ring slot d%4, column block d%4, A buffer (d/4)%2.
    // Loads issued after this visit's own: those of the three visits behind it in the ring, 8 each,
    // plus the 8*H pieces of A that travel with a chunk's first visit (one of the three unless
    // this visit is a first one itself).
    auto process = [&](auto d_c, int v) {
        constexpr int d = decltype(d_c)::value, slot = d % 4, jb = d % 4, par = (d / 4) % 2;
        st_wait_loads<24 + (jb != 0 ? 8 * H : 0)>();
        u32x4 cur[ST_RUN];
#pragma unroll
        for (int t = 0; t < ST_RUN; ++t)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(cur[t]) : "v"(frag_addr[t]), "n"(slot * ST_VISIT_BYTES) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(cur[0]), "+v"(cur[1]), "+v"(cur[2]), "+v"(cur[3]), "+v"(cur[4]), "+v"(cur[5]), "+v"(cur[6]), "+v"(cur[7])
                     :: "memory");
        // the slot has been read out: refill it with visit v + 4 (same column block, the other A buffer)
        load_visit(std::integral_constant<int, slot>{}, std::integral_constant<int, jb>{}, std::integral_constant<int, 1 - par>{}, v + 4);
#pragma unroll
        for (int t = 0; t < ST_RUN; ++t)
#pragma unroll
            for (int h = 0; h < H; ++h) acc[h][jb] = st_mfma<IS_BF16>(aq[par][h][t], cur[t], acc[h][jb]);
    };

    load_visit(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, 0);
    load_visit(std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{}, std::integral_constant<int, 0>{}, 1);
    load_visit(std::integral_constant<int, 2>{}, std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{}, 2);
    load_visit(std::integral_constant<int, 3>{}, std::integral_constant<int, 3>{}, std::integral_constant<int, 0>{}, 3);
    for (int v0 = 0; v0 < nvis; v0 += 8) {      // a trailing half group works on zeros
        process(std::integral_constant<int, 0>{}, v0 + 0);
        process(std::integral_constant<int, 1>{}, v0 + 1);
        process(std::integral_constant<int, 2>{}, v0 + 2);
        process(std::integral_constant<int, 3>{}, v0 + 3);
        process(std::integral_constant<int, 4>{}, v0 + 4);
        process(std::integral_constant<int, 5>{}, v0 + 5);
        process(std::integral_constant<int, 6>{}, v0 + 6);
        process(std::integral_constant<int, 7>{}, v0 + 7);
    }
    st_wait_loads<0>();      // the masked loads of the last visits still write (zeros) to LDS

#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 16 * h + 4 * g + v;
            if (row >= M) continue;
#pragma unroll
            for (int jb = 0; jb < 4; ++jb) {
                const int64_t col = n0 + 16 * jb + c16;
                if (col >= N) continue;
                const float x = acc[h][jb][v];
                if (split_k > 1) {
                    ws[((int64_t)blockIdx.y * M + row) * N + col] = x;
                } else {
                    const int64_t ci = row * a.ldc + col;
                    const float c_in = a.beta != 0.0f ? load_elem(a.C, a.out_dtype, ci) : 0.0f;
                    const float bj = a.bias ? load_elem(a.bias, a.bias_dtype, col) : 0.0f;
                    store_elem(a.C, a.out_dtype, ci, epilogue_value(x, a.alpha, a.beta, c_in, bj, a.act));
                }
            }
        }
}

// The same kernel cut for weights that are short of workgroups: a workgroup owns one block of 16 columns
// and its four waves take every fourth chunk of the k range each, adding their sums through LDS at the end
// (wave 0 adds waves 1, 2, 3 in that order).  N / 16 workgroups fill the chip from N = 4096 on, so a weight
// below 128 MiB needs no split of k and no second launch, which is what the wide kernel costs there
// (8 x 4096 x 4096: 16 us in 4 slices).  The price is A: every visit brings its own pieces of A (the wide
// kernel shares them over four column blocks) into the registers of its ring slot, as many bytes through the
// caches as B brings from memory.  Four visits in flight per wave (the waits count the wave's younger loads,
// 16 per visit, and the counter ends at 63).
template <bool IS_BF16, int H, int D>
__global__ __launch_bounds__(ST_WAVES * 64) void skinny_nt_narrow_kernel(Args a, int split_k, float* ws) {
    static_assert(H == 1, "16 rows of C (a second row block needs the registers of a visit in flight)");
    static_assert(D == 2 || D == 4, "visits in flight per wave: four, or two with two workgroups per compute unit");
    constexpr int PER_VISIT = 8 + 8 * H;              // loads a visit issues: 8 H for A, 8 for B
    static_assert((D - 1) * PER_VISIT <= 63, "the wait counter has six bits");
    __shared__ __attribute__((aligned(1024))) char ring[ST_WAVES * D * ST_VISIT_BYTES];
    __shared__ f32x4 red[(ST_WAVES - 1) * H * 64];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c16 = lane & 15, g = lane >> 4;
    const int M = (int)a.M, K = (int)a.K;
    const int64_t N = a.N;

    const int total_chunks = (K + ST_CHUNK - 1) / ST_CHUNK;
    const int per_split = (total_chunks + split_k - 1) / split_k;
    const int cbeg = blockIdx.y * per_split;
    const int cend = (cbeg + per_split) < total_chunks ? (cbeg + per_split) : total_chunks;
    const int nch = cend > cbeg ? cend - cbeg : 0;
    // wave w takes the chunks at positions w, w + 4, ... of the workgroup's walk, which starts at a chunk of
    // the column block's own and wraps around (the starts decorrelated from the block's index as in
    // gemv16_kernel.hip); the order of summation is a fixed function of the column block
    const int nvis = nch > wave ? (nch - wave + ST_WAVES - 1) / ST_WAVES : 0;
    const int rot = nch > 0 ? (int)(((unsigned)blockIdx.x * 11u + ((unsigned)blockIdx.x >> 5) * 3u) % (unsigned)nch) : 0;
    auto chunk_of = [&](int v) {      // for v < nvis
        const int c = v * ST_WAVES + wave + rot;
        return cbeg + (c >= nch ? c - nch : c);
    };

    const int64_t n0 = (int64_t)blockIdx.x * 16;
    const __amdgpu_buffer_rsrc_t rb = sk_rsrc(a.B, ((int64_t)(N - 1) * a.ldb + K) * 2);
    const __amdgpu_buffer_rsrc_t ra = sk_rsrc(a.A, ((int64_t)(M - 1) * a.lda + K) * 2);

    // global side of a visit: instruction i fetches stored rows 2i and 2i+1 of the block; this
    // lane serves row 2i + lr, slot ls, i.e. piece ls xor (2i + lr) of that row
    const int lr = lane >> 5, ls = lane & 31;
    const int n_first = (int)n0, n_last = (int)N - 1;
    const uint32_t ldb_b = (uint32_t)a.ldb * 2;
    char* const my_ring = ring + wave * (D * ST_VISIT_BYTES);
    // LDS side: operand of step t for this lane = row c16, piece 4t + g, kept in slot (4t + g) xor c16
    uint32_t frag_addr[ST_RUN];
#pragma unroll
    for (int t = 0; t < ST_RUN; ++t)
        frag_addr[t] = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)my_ring + (uint32_t)(c16 * 512 + (((4 * t + g) ^ c16) << 4));

    uint32_t a_row_off[H];
#pragma unroll
    for (int h = 0; h < H; ++h) {
        const int r = 16 * h + c16;
        a_row_off[h] = (uint32_t)((r < M ? r : M - 1) * a.lda * 2);     // rows >= M repeat a valid one and are never stored
    }

    f32x4 acc[H];
#pragma unroll
    for (int h = 0; h < H; ++h) acc[h] = f32x4{0.f, 0.f, 0.f, 0.f};

    u32x4 aq[D][H][ST_RUN];              // the pieces of A of the visit in each ring slot

    // Every visit slot of the loop below issues its loads whether the visit exists or not (a visit past
    // the end fetches nothing: all its offsets are masked and read as zero), so the number of loads in
    // flight behind any given one is the same on every path and the waits can be exact.
    auto load_visit = [&](auto slot_c, int v) {
        constexpr int slot = decltype(slot_c)::value;
        const bool live = v < nvis;
        const int chunk = live ? chunk_of(v) : cbeg;
        const int kbase = chunk * ST_CHUNK + 8 * g;
#pragma unroll
        for (int t = 0; t < ST_RUN; ++t) {
            const int k = kbase + 32 * t;
#pragma unroll
            for (int h = 0; h < H; ++h)
                aq[slot][h][t] = __builtin_amdgcn_raw_buffer_load_b128(ra, (live && k < K) ? a_row_off[h] + (uint32_t)k * 2 : ST_MASKED, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int rl = 2 * i + lr;                                   // row of the block
            const int n = n_first + rl;
            const int k = chunk * ST_CHUNK + ((ls ^ rl) << 3);
            const uint32_t off = (uint32_t)(n < n_last ? n : n_last) * ldb_b + (uint32_t)k * 2;   // columns >= N repeat a valid one and are never stored
            const uint32_t masked_off = (live && k < K) ? off : ST_MASKED;
            st_load_to_lds(rb, my_ring + slot * ST_VISIT_BYTES + i * 1024, masked_off);
        }
    };
    // Loads issued after this visit's own: those of the D - 1 visits behind it in the ring.  The slot is
    // refilled (visit v + D, LDS and registers of A alike) once the multiplications that read it are issued.
    auto process = [&](auto slot_c, int v) {
        constexpr int slot = decltype(slot_c)::value;
        st_wait_loads<(D - 1) * PER_VISIT>();
        u32x4 cur[ST_RUN];
#pragma unroll
        for (int t = 0; t < ST_RUN; ++t)
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(cur[t]) : "v"(frag_addr[t]), "n"(slot * ST_VISIT_BYTES) : "memory");
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(cur[0]), "+v"(cur[1]), "+v"(cur[2]), "+v"(cur[3]), "+v"(cur[4]), "+v"(cur[5]), "+v"(cur[6]), "+v"(cur[7])
                     :: "memory");
#pragma unroll
        for (int t = 0; t < ST_RUN; ++t)
#pragma unroll
            for (int h = 0; h < H; ++h) acc[h] = st_mfma<IS_BF16>(aq[slot][h][t], cur[t], acc[h]);
        __builtin_amdgcn_sched_barrier(0);
        load_visit(slot_c, v + D);
        __builtin_amdgcn_sched_barrier(0);
    };

    load_visit(std::integral_constant<int, 0>{}, 0);
    load_visit(std::integral_constant<int, 1>{}, 1);
    if constexpr (D == 4) {
        load_visit(std::integral_constant<int, 2>{}, 2);
        load_visit(std::integral_constant<int, 3>{}, 3);
    }
    for (int v0 = 0; v0 < nvis; v0 += D) {      // a trailing part of a group works on zeros
        process(std::integral_constant<int, 0>{}, v0 + 0);
        process(std::integral_constant<int, 1>{}, v0 + 1);
        if constexpr (D == 4) {
            process(std::integral_constant<int, 2>{}, v0 + 2);
            process(std::integral_constant<int, 3>{}, v0 + 3);
        }
    }
    st_wait_loads<0>();      // the masked loads of the last visits still write (zeros) to LDS

    // waves 1 .. 3 park their sums; wave 0 adds them in the order of the waves
    if (wave > 0) {
#pragma unroll
        for (int h = 0; h < H; ++h) red[((wave - 1) * H + h) * 64 + lane] = acc[h];
    }
    __syncthreads();
    if (wave > 0) return;
#pragma unroll
    for (int w = 0; w < ST_WAVES - 1; ++w)
#pragma unroll
        for (int h = 0; h < H; ++h) acc[h] += red[(w * H + h) * 64 + lane];
#pragma unroll
    for (int h = 0; h < H; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int row = 16 * h + 4 * g + v;
            if (row >= M) continue;
            const int64_t col = n0 + c16;
            if (col >= N) continue;
            const float x = acc[h][v];
            if (split_k > 1) {
                ws[((int64_t)blockIdx.y * M + row) * N + col] = x;
            } else {
                const int64_t ci = row * a.ldc + col;
                const float c_in = a.beta != 0.0f ? load_elem(a.C, a.out_dtype, ci) : 0.0f;
                const float bj = a.bias ? load_elem(a.bias, a.bias_dtype, col) : 0.0f;
                store_elem(a.C, a.out_dtype, ci, epilogue_value(x, a.alpha, a.beta, c_in, bj, a.act));
            }
        }
}

// Sums the split-K slices in the order 0, 1, ..., S-1 and applies the epilogue; 8 columns per thread.
// The kernel is one round trip to memory long, so everything it reads is requested before
// anything is used: S > 0 fixes the number of slices at compile time (all their loads are issued
// back to back, together with those of C_in and bias); S == 0 takes any number.
template <int S>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(Args a, int split_k, const float* ws, int c_vec_ok) {
    const int64_t groups_per_row = a.N / 8;
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= a.M * groups_per_row) return;
    const int64_t row = g / groups_per_row, col = (g % groups_per_row) * 8;
    const int64_t slice = a.M * a.N;
    const float* p = ws + row * a.N + col;
    SkRowInputs in;
    float x[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if constexpr (S > 0) {
        f32x4 lo[S], hi[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            lo[s] = *(const f32x4*)(p + s * slice);
            hi[s] = *(const f32x4*)(p + s * slice + 4);
        }
        sk_load_row_inputs(a, row, col, c_vec_ok != 0, in);
#pragma unroll
        for (int s = 0; s < S; ++s)
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[e] += lo[s][e]; x[4 + e] += hi[s][e]; }
    } else {
        sk_load_row_inputs(a, row, col, c_vec_ok != 0, in);
        for (int s = 0; s < split_k; ++s) {
            const f32x4 lo = *(const f32x4*)(p + s * slice), hi = *(const f32x4*)(p + s * slice + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { x[e] += lo[e]; x[4 + e] += hi[e]; }
        }
    }
    sk_store_row(a, row, col, x, in, c_vec_ok != 0);
}

// A stored K x M (transA): the few rows of op(A) are gathered once into a row-major M x K copy in the
// workspace (2 MiB at most), and the streaming kernels then run on the copy.  One thread moves eight
// consecutive k of one row: neighbouring lanes read neighbouring elements of a stored row and each
// writes 16 bytes of the copy.
__global__ __launch_bounds__(256) void skinny_transpose_a_kernel(const uint16_t* A, int64_t lda, int M, int K, uint16_t* At) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t blocks = K / 8;
    if (idx >= blocks * M) return;
    const int m = (int)(idx % M);
    const int64_t k0 = (idx / M) * 8;
    u32x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        o[j] = (uint32_t)A[(k0 + 2 * j) * lda + m] | ((uint32_t)A[(k0 + 2 * j + 1) * lda + m] << 16);
    *(u32x4*)(At + (int64_t)m * K + k0) = o;
}

}  // namespace

bool skinny_supports(const Args& a) {
    if (a.dtype == DT_F32) return gemv_f32_supports(a);
    if (a.dtype != DT_BF16 && a.dtype != DT_F16) return false;
    if (a.M < 1 || a.M > SK_MAX_ROWS || a.N < 8 || a.K < 8) return false;
    if ((a.N & 7) || (a.K & 7) || (a.ldb & 7)) return false;
    if ((uintptr_t)a.B & 15) return false;
    // a row-major A is read in 16-byte pieces; an A stored K x M element by element, into an aligned copy
    if (!a.transA && ((a.lda & 7) || ((uintptr_t)a.A & 15))) return false;
    if (a.transA && a.K * a.lda * 2 >= (int64_t)1 << 40) return false;
    // 32-bit byte offsets into A and B (row-major B: with room for the rows past K that read as
    // zero; B stored N x K: below the offset that masks a lane)
    const int64_t b_bytes = a.transB ? a.N * a.ldb * 2 : (a.K + 16) * a.ldb * 2;
    if (b_bytes >= (int64_t)ST_MASKED) return false;
    if ((a.M * (a.transA ? a.K : a.lda)) * 2 >= (int64_t)ST_MASKED) return false;
    if ((a.N + SK_COLS - 1) / SK_COLS > 65535 * 16) return false;
    return true;
}

// variant 0: row-major B (K x N); variant 1: B stored N x K.  The layout of the call decides.
// Variants 2 and 3: the same two layouts for fp32 operands and at most 8 rows (gemv_f32_kernel.hip).
// Variant 4: 16-bit operands, B stored N x K, at most 8 rows, on the vector ALUs (gemv16_kernel.hip);
// preferred to variant 1 up to SK_GEMV16_ROWS rows.
// Variant 5: variant 1 with 16 columns per workgroup (skinny_nt_narrow_kernel), at most 16 rows; preferred
// to variant 1 for small weights (see SK_NARROW_ROWS).
const char* skinny_variant_name(int variant) {
    switch (variant) {
        case 0: return "skinny_nn_32x256_w4";
        case 1: return "skinny_nt_32x256_w4";
        case 2: return "gemv_f32_nn_8x256_w4";
        case 3: return "gemv_f32_nt_8x32_w4";
        case 4: return "gemv16_nt_8x32_w4";
        case 5: return "skinny_nt_16x16_w4";
        default: return nullptr;
    }
}

static bool skinny_narrow_serves(const Args& a) { return a.dtype != DT_F32 && a.transB && a.M <= SK_NARROW_ROWS; }

int skinny_variant_of(const Args& a) {
    if (a.dtype != DT_F32 && a.M <= SK_GEMV16_ROWS && gemv16_supports(a)) return 4;
    if (skinny_narrow_serves(a) && !a.transA && a.K >= SK_NARROW_MIN_K && a.N * a.K * 2 <= SK_NARROW_BYTES) {
        const int64_t groups = (a.N + 15) / 16, rounds = (groups + SK_NARROW_PLACES - 1) / SK_NARROW_PLACES;
        const bool full_enough = a.M <= 8 || groups * 100 >= rounds * SK_NARROW_PLACES * 65;
        if (a.N <= SK_NARROW_MAX_N || (a.N <= SK_NARROW_FAR_N && a.K >= SK_NARROW_FAR_K && full_enough)) return 5;
    }
    return (a.dtype == DT_F32 ? 2 : 0) + (a.transB ? 1 : 0);
}

bool skinny_variant_serves(const Args& a, int variant) {
    if (variant < 0 || variant == skinny_variant_of(a)) return true;
    if (variant == 4) return gemv16_supports(a);
    if (variant == 5) return skinny_narrow_serves(a);
    // the wide MFMA kernel for a weight stored N x K also takes the calls that variants 4 and 5 are preferred for
    return variant == 1 && a.dtype != DT_F32 && a.transB;
}

// units the k range is cut in: steps of 16 (row-major B) or chunks of ST_CHUNK (B stored N x K)
static int64_t skinny_k_units(const Args& a) { return a.transB ? (a.K + ST_CHUNK - 1) / ST_CHUNK : (a.K + 15) / 16; }

int skinny_max_split(const Args& a, int variant) {
    if (a.dtype == DT_F32) return gemv_f32_max_split(a);
    const int v = variant < 0 ? skinny_variant_of(a) : variant;
    if (v == 4) return gemv16_max_split(a);
    if (v == 5) {      // four visits per wave and slice at least
        const int64_t s = skinny_k_units(a) / (ST_WAVES * 4);
        return (int)(s < 1 ? 1 : (s > 64 ? 64 : s));
    }
    const int64_t units = skinny_k_units(a);
    return (int)(units < 1 ? 1 : (units > 64 ? 64 : units));
}

int skinny_default_split(const Args& a, int num_cus, int variant) {
    if (a.dtype == DT_F32) return gemv_f32_default_split(a, num_cus);
    const int v = variant < 0 ? skinny_variant_of(a) : variant;
    if (v == 4) return gemv16_default_split(a, num_cus);
    if (v == 5) {      // one launch wherever N gives half a workgroup per compute unit or more; else the slices that fill the units
        const int64_t g16 = (a.N + 15) / 16, units = num_cus > 0 ? num_cus : 256, max16 = skinny_max_split(a, 5);
        int64_t s16 = g16 * 2 <= units ? units / g16 : 1;
        if (s16 > max16) s16 = max16;
        return (int)(s16 < 1 ? 1 : s16);
    }
    const int64_t groups = (a.N + SK_COLS - 1) / SK_COLS, cus = num_cus > 0 ? num_cus : 256;
    // keep the pipeline of every wave filled a few times over (row-major B: the waves of a
    // workgroup share its k range; B stored N x K: every wave walks all of it, four visits per chunk)
    int64_t max_s = a.transB ? skinny_k_units(a) / 4 : skinny_k_units(a) / (SK_WAVES * 2 * SK_DEPTH);
    if (max_s > 64) max_s = 64;
    if (max_s < 1) max_s = 1;
    // One workgroup per compute unit is resident; groups x slices workgroups run in whole rounds
    // of them, and a partly filled round streams at a fraction of the memory rate.  Time in us:
    // B at 6.1 TB/s stretched by the unfilled part of the rounds, 5 us per round for filling and
    // draining a workgroup's pipelines, plus the second kernel (launch + the partial sums written
    // and read once at 4.5 TB/s).  28672 columns = 112 groups: 2 slices fill 224 of 256 units in
    // one round (32x28672x8192: 91 to 93 us); "one workgroup per unit" rounded up gave 3 slices =
    // two rounds at 66 % (113 to 117 us), and 9 slices fill four rounds but pay for them (101 to 104).
    const double stream = (double)a.N * (double)a.K * 2.0 / 6.1e6, part = (double)a.M * (double)a.N * 8.0 / 4.5e6;
    int64_t best = 1;
    double best_t = 0.0;
    for (int64_t s = 1; s <= max_s; ++s) {
        const int64_t wgs = groups * s, rounds = (wgs + cus - 1) / cus;
        const double t = stream * (double)(rounds * cus) / (double)wgs + 5.0 * (double)rounds + (s > 1 ? 3.0 + part * (double)s : 0.0);
        if (s == 1 || t < best_t) { best_t = t; best = s; }
    }
    return (int)best;
}

// fp32 partial results [split][M][N] (none without a split), then the row-major copy of an A stored K x M
static size_t skinny_partial_bytes(const Args& a, int split_k) {
    const size_t n = split_k > 1 ? (size_t)split_k * (size_t)a.M * (size_t)a.N * sizeof(float) : 0;
    return (n + 255) & ~(size_t)255;
}
size_t skinny_workspace_bytes(const Args& a, int split_k) {
    return skinny_partial_bytes(a, split_k) + (a.transA && a.dtype != DT_F32 ? (size_t)a.M * (size_t)a.K * 2 : 0);
}

namespace {
template <bool IS_BF16>
void launch_nt(const Args& a, dim3 grid, int split_k, float* ws, hipStream_t stream) {
    if (a.M <= 16)
        hipLaunchKernelGGL((skinny_nt_kernel<IS_BF16, 1>), grid, dim3(ST_WAVES * 64), 0, stream, a, split_k, ws);
    else if (a.M <= 32)
        hipLaunchKernelGGL((skinny_nt_kernel<IS_BF16, 2>), grid, dim3(ST_WAVES * 64), 0, stream, a, split_k, ws);
    else
        hipLaunchKernelGGL((skinny_nt_kernel<IS_BF16, 4>), grid, dim3(ST_WAVES * 64), 0, stream, a, split_k, ws);
}
}  // namespace

hipError_t launch_skinny(const Args& call, int split_k, float* workspace, hipStream_t stream, int variant) {
    if (call.dtype == DT_F32) return launch_gemv_f32(call, split_k, workspace, stream);
    const int v = variant < 0 ? skinny_variant_of(call) : variant;
    if (v == 4) return launch_gemv16(call, split_k, workspace, stream);
    Args a = call;
    if (call.transA) {
        if (workspace == nullptr) return hipErrorInvalidValue;
        const int64_t units = skinny_k_units(call);
        const int s = split_k < 1 ? 1 : (split_k > units ? (int)units : split_k);
        uint16_t* copy = (uint16_t*)((char*)workspace + skinny_partial_bytes(call, s));
        const int64_t threads = call.M * (call.K / 8);
        hipLaunchKernelGGL(skinny_transpose_a_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, stream,
                           (const uint16_t*)call.A, call.lda, (int)call.M, (int)call.K, copy);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        a.A = copy; a.lda = call.K; a.transA = 0;
    }
    const int64_t groups = (a.N + SK_COLS - 1) / SK_COLS;
    const int64_t units = skinny_k_units(a);
    if (split_k < 1) split_k = 1;
    if (split_k > units) split_k = (int)units;
    if (split_k > 1 && workspace == nullptr) return hipErrorInvalidValue;
    // 8 outputs per vector store: 32 bytes of fp32 or 16 bytes of a 16-bit type
    const int c_vec_ok = (a.ldc % 8 == 0) && ((uintptr_t)a.C % 16 == 0);
    const dim3 grid((unsigned)groups, (unsigned)split_k), block(SK_WAVES * 64);
    if (a.transB && v == 5) {
        if (a.M > SK_NARROW_ROWS) return hipErrorInvalidValue;
        const dim3 ngrid((unsigned)((a.N + 15) / 16), (unsigned)split_k), nblock(ST_WAVES * 64);
        // one round of workgroups at most: four visits in flight per wave; more: two, and two workgroups per compute unit
        if (a.N <= SK_NARROW_MAX_N) {
            if (a.dtype == DT_BF16) hipLaunchKernelGGL((skinny_nt_narrow_kernel<true, 1, 4>), ngrid, nblock, 0, stream, a, split_k, workspace);
            else hipLaunchKernelGGL((skinny_nt_narrow_kernel<false, 1, 4>), ngrid, nblock, 0, stream, a, split_k, workspace);
        } else {
            if (a.dtype == DT_BF16) hipLaunchKernelGGL((skinny_nt_narrow_kernel<true, 1, 2>), ngrid, nblock, 0, stream, a, split_k, workspace);
            else hipLaunchKernelGGL((skinny_nt_narrow_kernel<false, 1, 2>), ngrid, nblock, 0, stream, a, split_k, workspace);
        }
    } else if (a.transB) {
        if (a.dtype == DT_BF16) launch_nt<true>(a, grid, split_k, workspace, stream);
        else launch_nt<false>(a, grid, split_k, workspace, stream);
    } else if (a.dtype == DT_BF16) {
        if (a.M <= 32) hipLaunchKernelGGL((skinny_nn_kernel<true, 1>), grid, block, 0, stream, a, split_k, workspace, c_vec_ok);
        else hipLaunchKernelGGL((skinny_nn_kernel<true, 2>), grid, block, 0, stream, a, split_k, workspace, c_vec_ok);
    } else {
        if (a.M <= 32) hipLaunchKernelGGL((skinny_nn_kernel<false, 1>), grid, block, 0, stream, a, split_k, workspace, c_vec_ok);
        else hipLaunchKernelGGL((skinny_nn_kernel<false, 2>), grid, block, 0, stream, a, split_k, workspace, c_vec_ok);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split_k == 1) return e;
    return launch_splitk_reduce(a, split_k, workspace, stream);
}

hipError_t launch_splitk_reduce(const Args& a, int split_k, const float* partials, hipStream_t stream) {
    if (split_k < 1 || partials == nullptr || (a.N & 7)) return hipErrorInvalidValue;
    const int c_vec_ok = (a.ldc % 8 == 0) && ((uintptr_t)a.C % 16 == 0);
    const int64_t threads = a.M * (a.N / 8);
    const dim3 rgrid((unsigned)((threads + 255) / 256)), rblock(256);
    switch (split_k) {
        case 2: hipLaunchKernelGGL(splitk_reduce_kernel<2>, rgrid, rblock, 0, stream, a, split_k, partials, c_vec_ok); break;
        case 4: hipLaunchKernelGGL(splitk_reduce_kernel<4>, rgrid, rblock, 0, stream, a, split_k, partials, c_vec_ok); break;
        case 8: hipLaunchKernelGGL(splitk_reduce_kernel<8>, rgrid, rblock, 0, stream, a, split_k, partials, c_vec_ok); break;
        case 16: hipLaunchKernelGGL(splitk_reduce_kernel<16>, rgrid, rblock, 0, stream, a, split_k, partials, c_vec_ok); break;
        default: hipLaunchKernelGGL(splitk_reduce_kernel<0>, rgrid, rblock, 0, stream, a, split_k, partials, c_vec_ok); break;
    }
    return hipGetLastError();
}

}  // namespace gemm

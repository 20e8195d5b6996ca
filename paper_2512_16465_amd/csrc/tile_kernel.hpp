// The macro-tile GEMM kernel for bf16 / fp16 operands on the gfx950 matrix cores.
//
// One workgroup computes a BM x BN block of C.  Per step of BK along k it stages a BM x BK slab
// of op(A) and a BN x BK slab of op(B) in LDS, both stored k-contiguous per row whatever the
// layout in memory, in two stages so that the global loads of step t+1 overlap the MFMAs of
// step t.  Each wave owns a (BM/WM) x (BN/WN) sub-block as a grid of 32x32 accumulators fed by
// v_mfma_f32_32x32x16_{bf16,f16}.  This is the paper's list of GEMM strategies (Section 5.4,
// Table 1) recast for CDNA4: matrix cores, block/wave/register tiling, 16-byte vector access,
// a swizzled (conflict-free) shared-memory layout, workgroup-id swizzle for L2 locality and
// double buffering.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace gemm {
namespace tile {

template <int BM_, int BN_, int BK_, int WM_, int WN_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_;
    static constexpr int NT = WM * WN * 64;           // threads per workgroup
    static constexpr int WTM = BM / WM, WTN = BN / WN; // wave sub-block
    static constexpr int TM = WTM / 32, TN = WTN / 32; // 32x32 accumulators per wave
    static constexpr int CPR = BK / 8;                 // 16-byte chunks per LDS row
    static constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static_assert(BK == 32 || BK == 64, "the swizzle below is written for 64- or 128-byte rows");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave sub-block must be whole 32x32 tiles");
};

// LDS byte offset of 16-byte chunk c of row `row`.  Chunks are numbered row-major, grouped in
// 128-byte lines of 8, and the position inside a line is XOR-ed with a hash of the line number.
// With it, 8 (and 16) consecutive lanes that read the same logical chunk of consecutive rows,
// write the 8 chunks of one row, or write one chunk of rows 8 apart, all touch distinct banks.
template <int CPR>
__device__ __forceinline__ uint32_t swz(uint32_t row, uint32_t c) {
    const uint32_t chunk = row * CPR + c;
    const uint32_t line = chunk >> 3;
    const uint32_t pos = (chunk & 7u) ^ ((line ^ (line >> 3)) & 7u);
    return (line << 7) | (pos << 4);
}

// ---- global -> register -> LDS movers, one flavour per memory layout of the operand ----

// Buffer descriptor over [base, base + avail): loads take a 32-bit byte offset per lane (no
// 64-bit address arithmetic in vector registers) and anything past the end reads as zero instead
// of faulting.  The descriptor is rebuilt with scalar instructions at every k step.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const char* base, int64_t avail) {
    const int64_t cap = 0xffffffffll;
    const uint32_t n = (uint32_t)(avail < 0 ? 0 : (avail > cap ? cap : avail));
    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)n, 0x00020000);
}

// Operand whose k index is contiguous in memory: tile row r, k-chunk c is 16 bytes at
// base + r*ld + 8c.  Each thread moves L chunks.
template <int ROWS, int BK, int NT>
struct LoaderKC {
    static constexpr int CPR = BK / 8, CHUNKS = ROWS * CPR, L = CHUNKS / NT;
    static_assert(CHUNKS % NT == 0, "chunks must divide evenly over the threads");
    u32x4 r[L];
    uint32_t goff[L];

    __device__ __forceinline__ void init(int tid, int valid_rows, int64_t ld) {
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int id = i * NT + tid, row = id / CPR, c = id % CPR;
            const int rc = row < valid_rows ? row : valid_rows - 1;   // rows past the edge re-read a valid row
            goff[i] = (uint32_t)((rc * ld + c * 8) * 2);
        }
    }
    // base = first byte of the tile at this k step, avail = bytes from there to the end of the matrix
    template <bool MASKED>
    __device__ __forceinline__ void gload(const char* base, int64_t avail, int tid, int k0, int K, int32_t /*ld_bytes*/) {
        const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(base, avail);
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int c = (i * NT + tid) % CPR;
            if (!MASKED || k0 + c * 8 < K) r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[i], 0, 0);
            else r[i] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    __device__ __forceinline__ void lstore(char* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < L; ++i) store_piece(i, lds, tid);
    }
    // One piece = one 16-byte chunk: a single global load, a single LDS store.
    static constexpr int PIECES = L;
    __device__ __forceinline__ void load_piece(int i, __amdgpu_buffer_rsrc_t rsrc, int /*tid*/, int32_t /*ld_bytes*/) {
        r[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[i], 0, 0);
    }
    __device__ __forceinline__ void store_piece(int i, char* lds, int tid) const {
        const int id = i * NT + tid;
        *(u32x4*)(lds + swz<CPR>(id / CPR, id % CPR)) = r[i];
    }
    static __device__ __forceinline__ const char* tile_base(const void* p, int64_t first_row, int64_t ld) {
        return (const char*)p + first_row * ld * 2;
    }
    static __device__ __forceinline__ int64_t k_step_bytes(int64_t /*ld*/) { return BK * 2; }
};

// Operand whose m (or n) index is contiguous in memory: element (k, r) is at base + k*ld + r.
// A thread unit is 8 k-rows x 8 r: eight 16-byte loads, an 8x8 transposition of 16-bit values
// in registers (one v_perm_b32 per output dword), eight 16-byte LDS stores.
template <int ROWS, int BK, int NT>
struct LoaderMC {
    static constexpr int CPR = BK / 8, RC = ROWS / 8, UNITS = RC * CPR, U = (UNITS + NT - 1) / NT;
    static_assert(UNITS % 64 == 0, "whole waves must be active or idle");
    u32x4 r[U][8];
    uint32_t goff[U];

    __device__ __forceinline__ void init(int tid, int valid_rows, int64_t ld) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int unit = u * NT + tid, c = unit % RC, g = unit / RC;
            const int c8 = (c * 8 + 8 <= valid_rows) ? c * 8 : valid_rows - 8;   // stay inside the matrix
            goff[u] = (uint32_t)((g * 8 * ld + c8) * 2);
        }
    }
    template <bool MASKED>
    __device__ __forceinline__ void gload(const char* base, int64_t avail, int tid, int k0, int K, int32_t ld_bytes) {
        const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(base, avail);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int unit = u * NT + tid, g = unit / RC;
            if (UNITS % NT != 0 && unit >= UNITS) continue;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (!MASKED || k0 + g * 8 + j < K) r[u][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[u], j * ld_bytes, 0);
                else r[u][j] = u32x4{0u, 0u, 0u, 0u};
            }
        }
    }
    __device__ __forceinline__ void lstore(char* lds, int tid) const {
#pragma unroll
        for (int q = 0; q < PIECES; ++q) store_piece(q, lds, tid);
    }
    // One load piece = one of the eight k-rows of a unit; one store piece = one of its eight
    // output rows: four v_perm_b32 gather that row's 8 k-values, one 16-byte LDS store writes them.
    static constexpr int PIECES = 8 * U;
    __device__ __forceinline__ void load_piece(int q, __amdgpu_buffer_rsrc_t rsrc, int tid, int32_t ld_bytes) {
        const int u = q / 8, j = q % 8;
        if (UNITS % NT != 0 && u * NT + tid >= UNITS) return;
        r[u][j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[u], j * ld_bytes, 0);
    }
    __device__ __forceinline__ void store_piece(int q, char* lds, int tid) const {
        const int u = q / 8, n = q % 8;
        const int unit = u * NT + tid, c = unit % RC, g = unit / RC;
        if (UNITS % NT != 0 && unit >= UNITS) return;
        u32x4 o;
        const uint32_t sel = (n & 1) ? 0x07060302u : 0x05040100u;   // high or low halves of both sources
#pragma unroll
        for (int kp = 0; kp < 4; ++kp)
            o[kp] = __builtin_amdgcn_perm(r[u][2 * kp + 1][n >> 1], r[u][2 * kp][n >> 1], sel);
        *(u32x4*)(lds + swz<CPR>(c * 8 + n, g)) = o;
    }
    static __device__ __forceinline__ const char* tile_base(const void* p, int64_t first_row, int64_t /*ld*/) {
        return (const char*)p + first_row * 2;
    }
    static __device__ __forceinline__ int64_t k_step_bytes(int64_t ld) { return (int64_t)BK * ld * 2; }
};

template <bool IS_BF16>
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
    if constexpr (IS_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Workgroup id -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs, each
// with its own L2, so the ids that land on one XCD are first made contiguous, and contiguous ids
// then walk C in bands of group_m tile rows, column by column: the ~32 workgroups resident on
// an XCD cover a compact block of C and share their A and B slabs in that XCD's L2.
__device__ __forceinline__ void tile_of_workgroup(int pid, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
    const int T = tiles_m * tiles_n;
    const int xcd = pid & 7, local = pid >> 3;
    const int q = T >> 3, rem = T & 7;
    const int id = xcd * q + (xcd < rem ? xcd : rem) + local;
    const int band = group_m * tiles_n;
    const int first_m = (id / band) * group_m;
    const int rows = (tiles_m - first_m) < group_m ? (tiles_m - first_m) : group_m;
    const int in = id % band;
    tm = first_m + in % rows;
    tn = in / rows;
}

// ---- epilogue helpers: four consecutive outputs of one row, in the type of C ----

template <int OUT> struct OutVec;
template <> struct OutVec<DT_F32> {
    typedef float elem;
    static __device__ __forceinline__ f32x4 load4(const elem* p) { return *(const f32x4*)p; }
    static __device__ __forceinline__ float load1(const elem* p) { return *p; }
    static __device__ __forceinline__ void store4(elem* p, f32x4 v) { __builtin_nontemporal_store(v, (f32x4*)p); }
    static __device__ __forceinline__ void store1(elem* p, float v) { *p = v; }
};
template <> struct OutVec<DT_BF16> {
    typedef uint16_t elem;
    static __device__ __forceinline__ f32x4 load4(const elem* p) {
        const uint2 u = *(const uint2*)p;
        return f32x4{__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                     __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
    }
    static __device__ __forceinline__ float load1(const elem* p) { return bf16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store4(elem* p, f32x4 v) {
        typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
        __builtin_nontemporal_store(__builtin_bit_cast(u32x2, __builtin_convertvector(v, bf16x4)), (u32x2*)p);   // v_cvt_pk_bf16_f32, nearest even
    }
    static __device__ __forceinline__ void store1(elem* p, float v) { *p = __builtin_bit_cast(uint16_t, (__bf16)v); }
};
template <> struct OutVec<DT_F16> {
    typedef uint16_t elem;
    static __device__ __forceinline__ f32x4 load4(const elem* p) {
        return f32x4{f16_bits_to_f32(p[0]), f16_bits_to_f32(p[1]), f16_bits_to_f32(p[2]), f16_bits_to_f32(p[3])};
    }
    static __device__ __forceinline__ float load1(const elem* p) { return f16_bits_to_f32(*p); }
    static __device__ __forceinline__ void store4(elem* p, f32x4 v) {
        typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
        __builtin_nontemporal_store(__builtin_bit_cast(u32x2, __builtin_convertvector(v, f16x4)), (u32x2*)p);    // v_cvt_f16_f32, nearest even
    }
    static __device__ __forceinline__ void store1(elem* p, float v) { *p = f32_to_f16_bits(v); }
};

template <class C>
struct EpiLayout {
    // Each wave parks one 32-row band of its sub-block in a private LDS region, row-major with a
    // padded row, and reads it back as 16-byte vectors along the row.
    static constexpr int RS = C::WTN + 8;               // floats per staged row (pad keeps the two lane halves on different banks)
    static constexpr int REGION = 32 * RS * 4;          // bytes per wave
    static constexpr int BYTES = REGION * C::WM * C::WN;
    static constexpr int LPR = C::WTN / 4;              // lanes that cover one row
    static constexpr int RPI = 64 / LPR;                // rows per read instruction
    static_assert(LPR <= 64 && 64 % LPR == 0, "a row must be covered by a whole fraction of a wave");
};

// The epilogue of one workgroup tile.  In a 32x32 accumulator lane (l32, lhi) owns column l32 and
// rows 8*(v/4) + 4*lhi + v%4.  Band by band (32 rows) each wave transposes that through its
// private LDS region so that a lane ends up with four consecutive columns of one row, and C is
// read and written with full-width vector accesses.  Every wave of the workgroup must be done
// with the operand stages in LDS before this is called.
//
// `dump(band, region)` writes rows 32*band .. 32*band+31 of the wave's sub-block, as held in
// that wave's accumulators, to region[(row * EL::RS + column) * 4]; `band` is an
// std::integral_constant, so the accumulator registers it names are static.
template <class C, class Dump>
__device__ __forceinline__ void tile_epilogue_bands(Dump dump, char* lds, const Args& a, int64_t m0, int64_t n0, int c_vec_ok,
                                                    int64_t live_rows = INT64_MAX) {
    constexpr int TM = C::TM;
    using EL = EpiLayout<C>;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % C::WM, wn = wave / C::WM;
    char* region = lds + wave * EL::REGION;
    const float alpha = a.alpha, beta = a.beta;
    const int act = a.act;
    const int cl = (lane % EL::LPR) * 4;                 // first of this lane's four columns inside the wave sub-block
    const int64_t col = n0 + wn * C::WTN + cl;
    f32x4 bias4 = {0.0f, 0.0f, 0.0f, 0.0f};
    if (a.bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < a.N) bias4[e] = load_elem(a.bias, a.bias_dtype, col + e);
    }

    // The code below runs once per tile, so its size matters more than its instruction count: a
    // kernel that streams tens of kilobytes of straight-line epilogue through the instruction
    // cache spends longer fetching it than executing it.  Only the register -> LDS dump of a band
    // needs static register numbers; the bands are walked by a real loop that picks the dump with
    // a compare chain, and the read-back/store part exists once.
    static_assert(TM <= 4, "the band switch below lists four cases");
    const bool interior = c_vec_ok && (m0 + C::BM <= a.M) && (n0 + C::BN <= a.N);
    auto run_epilogue = [&](auto tag) {
        using OV = OutVec<decltype(tag)::value>;
        typename OV::elem* Cp = (typename OV::elem*)a.C;
#pragma unroll 1
        for (int i = 0; i < TM; ++i) {
            // this band and the ones below it lie under the last row of C (`live_rows`: the same for a caller that
            // stores a whole tile somewhere else)
            if (m0 + wm * C::WTM + i * 32 >= a.M || wm * C::WTM + i * 32 >= live_rows) break;
            // one case per band; the distinct marker at the end of each case keeps the optimiser from
            // merging the cases into an indexed (scratch-memory) access to the accumulators
            switch (i) {
                case 0: dump(std::integral_constant<int, 0>{}, region); asm volatile("; band 0" ::: "memory"); break;
                case 1: if constexpr (TM > 1) dump(std::integral_constant<int, 1 % TM>{}, region); asm volatile("; band 1" ::: "memory"); break;
                case 2: if constexpr (TM > 2) dump(std::integral_constant<int, 2 % TM>{}, region); asm volatile("; band 2" ::: "memory"); break;
                default: if constexpr (TM > 3) dump(std::integral_constant<int, 3 % TM>{}, region); asm volatile("; band 3" ::: "memory"); break;
            }
            __builtin_amdgcn_wave_barrier();
            constexpr int TRIPS = 32 / EL::RPI;
            constexpr int GROUP = TRIPS % 4 == 0 ? 4 : 1;
            if (interior) {
                // Whole tile inside C and rows aligned for vector access: no per-lane conditions at
                // all, only wave-uniform branches on beta and the activation; four rows in flight
                // per trip so that the LDS and C_in latencies overlap.
                typename OV::elem* p0 = Cp + (m0 + wm * C::WTM + i * 32 + lane / EL::LPR) * a.ldc + col;
                const int64_t step = (int64_t)EL::RPI * a.ldc;
                const char* rd = region + ((lane / EL::LPR) * EL::RS + cl) * 4;
#pragma unroll 1
                for (int it0 = 0; it0 < TRIPS; it0 += GROUP) {
                    f32x4 s[GROUP];
#pragma unroll
                    for (int g = 0; g < GROUP; ++g) s[g] = *(const f32x4*)(rd + (it0 + g) * EL::RPI * EL::RS * 4);
                    if (beta != 0.0f) {
                        f32x4 cin[GROUP];
#pragma unroll
                        for (int g = 0; g < GROUP; ++g) cin[g] = OV::load4(p0 + (it0 + g) * step);
#pragma unroll
                        for (int g = 0; g < GROUP; ++g) s[g] = alpha * s[g] + beta * cin[g] + bias4;
                    } else {
#pragma unroll
                        for (int g = 0; g < GROUP; ++g) s[g] = alpha * s[g] + bias4;
                    }
                    apply_act4(s, act);
#pragma unroll
                    for (int g = 0; g < GROUP; ++g) OV::store4(p0 + (it0 + g) * step, s[g]);
                }
            } else {
#pragma unroll 1
                for (int it = 0; it < TRIPS; ++it) {
                    const int rl = it * EL::RPI + lane / EL::LPR;
                    const f32x4 s = *(const f32x4*)(region + (rl * EL::RS + cl) * 4);
                    const int64_t row = m0 + wm * C::WTM + i * 32 + rl;
                    if (row < a.M && col < a.N) {
                        typename OV::elem* p = Cp + row * a.ldc + col;
                        if (c_vec_ok && col + 3 < a.N) {
                            f32x4 cin = {0.0f, 0.0f, 0.0f, 0.0f};
                            if (beta != 0.0f) cin = OV::load4(p);
                            f32x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) o[e] = epilogue_value(s[e], alpha, beta, cin[e], bias4[e], act);
                            OV::store4(p, o);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < a.N) {
                                    const float c1 = (beta != 0.0f) ? OV::load1(p + e) : 0.0f;
                                    OV::store1(p + e, epilogue_value(s[e], alpha, beta, c1, bias4[e], act));
                                }
                        }
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    };
    if (a.out_dtype == DT_F32) run_epilogue(std::integral_constant<int, DT_F32>{});
    else if (a.out_dtype == DT_BF16) run_epilogue(std::integral_constant<int, DT_BF16>{});
    else run_epilogue(std::integral_constant<int, DT_F16>{});
}

// The staged epilogue for accumulators of the 32x32x16 MFMA.
template <class C>
__device__ __forceinline__ void tile_epilogue(f32x16 (&acc)[C::TM][C::TN], char* lds, const Args& a,
                                              int64_t m0, int64_t n0, int c_vec_ok) {
    using EL = EpiLayout<C>;
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, lhi = lane >> 5;
    tile_epilogue_bands<C>(
        [&](auto band, char* region) {
            constexpr int b = decltype(band)::value;
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    *(float*)(region + ((8 * (v >> 2) + 4 * lhi + (v & 3)) * EL::RS + j * 32 + l32) * 4) = acc[b][j][v];
        },
        lds, a, m0, n0, c_vec_ok);
}

// The plainest epilogue, C = alpha*A*B on a problem made of whole tiles (beta == 0, no bias, no
// activation): no LDS, every accumulator register is scaled, rounded and stored straight from
// the MFMA layout.  A store instruction covers two rows x 32 columns (128-byte segments in
// fp32); the row base is wave-uniform, the lane part is one 32-bit offset.  It lives in kernel
// instances of its own: a kernel that contains both epilogues copies all 256 accumulators into
// vector registers ahead of the branch between them, and spills.
template <class C>
__device__ __forceinline__ void tile_epilogue_plain(f32x16 (&acc)[C::TM][C::TN], const Args& a, int64_t m0, int64_t n0) {
    constexpr int TM = C::TM, TN = C::TN;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wm = wave % C::WM, wn = wave / C::WM;
    const float alpha = a.alpha;
    auto run_direct = [&](auto tag) {
        using OV = OutVec<decltype(tag)::value>;
        typename OV::elem* base = (typename OV::elem*)a.C + (m0 + wm * C::WTM) * a.ldc + n0 + wn * C::WTN;
        const uint32_t lane_off = (uint32_t)(4 * lhi * a.ldc + l32);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                typename OV::elem* rowp = base + (int64_t)(i * 32 + 8 * (v >> 2) + (v & 3)) * a.ldc;
#pragma unroll
                for (int j = 0; j < TN; ++j) OV::store1(rowp + lane_off + j * 32, alpha * acc[i][j][v]);
            }
    };
    if (a.out_dtype == DT_F32) run_direct(std::integral_constant<int, DT_F32>{});
    else if (a.out_dtype == DT_BF16) run_direct(std::integral_constant<int, DT_BF16>{});
    else run_direct(std::integral_constant<int, DT_F16>{});
}

// true if the call can use the kernels built around tile_epilogue_plain
template <class C>
inline bool plain_epilogue_applies(const Args& a) {
    return a.beta == 0.0f && a.bias == nullptr && a.act == ACT_NONE && a.M % C::BM == 0 && a.N % C::BN == 0 &&
           a.ldc < (1 << 26);
}

template <class C, bool IS_BF16, bool A_KC, bool B_KC>
__global__ __launch_bounds__(C::NT) void tile_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok) {
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::NT, TM = C::TM, TN = C::TN, CPR = C::CPR;
    using EL = EpiLayout<C>;
    constexpr int LDS_BYTES = 2 * C::STAGE > EL::BYTES ? 2 * C::STAGE : EL::BYTES;
    __shared__ __attribute__((aligned(128))) char lds[LDS_BYTES];
    select_batch(a);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wm = wave % C::WM, wn = wave / C::WM;

    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, group_m, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    const int valid_m = (a.M - m0) < BM ? (int)(a.M - m0) : BM;
    const int valid_n = (a.N - n0) < BN ? (int)(a.N - n0) : BN;
    const int K = (int)a.K;

    using LA = typename std::conditional<A_KC, LoaderKC<BM, BK, NT>, LoaderMC<BM, BK, NT>>::type;
    using LB = typename std::conditional<B_KC, LoaderKC<BN, BK, NT>, LoaderMC<BN, BK, NT>>::type;
    LA la;
    LB lb;
    la.init(tid, valid_m, a.lda);
    lb.init(tid, valid_n, a.ldb);
    const char* pa = LA::tile_base(a.A, m0, a.lda);
    const char* pb = LB::tile_base(a.B, n0, a.ldb);
    const int64_t a_step = LA::k_step_bytes(a.lda), b_step = LB::k_step_bytes(a.ldb);
    const int32_t lda_b = (int32_t)a.lda * 2, ldb_b = (int32_t)a.ldb * 2;
    // bytes from the tile's first element to the end of each operand's storage
    const int64_t a_bytes = ((A_KC ? (a.M - 1) * a.lda + a.K : (a.K - 1) * a.lda + a.M) * 2) - (pa - (const char*)a.A);
    const int64_t b_bytes = ((B_KC ? (a.N - 1) * a.ldb + a.K : (a.K - 1) * a.ldb + a.N) * 2) - (pb - (const char*)a.B);

    // LDS byte offsets of this lane's fragment rows at k-chunk 0; chunk 2*ks + lhi is reached by
    // XOR-ing (ks << 5), because the chunk index only occupies the swizzled position bits.
    uint32_t fa[TM], fb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = swz<CPR>(wm * C::WTM + i * 32 + l32, lhi);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = C::A_BYTES + swz<CPR>(wn * C::WTN + j * 32 + l32, lhi);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int k_tiles = (K + BK - 1) / BK;
    const int full_tiles = K / BK;      // k tiles that need no mask; at most one masked tile follows
    constexpr int NKS = BK / 16;        // MFMA k-steps per staged slab

    u32x4 af[2][TM], bf[2][TN];         // operand fragments, double-buffered in registers

    auto read_frags = [&](int buf, int stage, int ks) {
        const char* st = lds + stage * C::STAGE;
#pragma unroll
        for (int i = 0; i < TM; ++i) af[buf][i] = *(const u32x4*)(st + (fa[i] ^ (uint32_t)(ks << 5)));
#pragma unroll
        for (int j = 0; j < TN; ++j) bf[buf][j] = *(const u32x4*)(st + (fb[j] ^ (uint32_t)(ks << 5)));
    };
    auto mfmas = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = mfma32<IS_BF16>(af[buf][i], bf[buf][j], acc[i][j]);
    };
    auto lstore = [&](int stage) {
        la.lstore(lds + stage * C::STAGE, tid);
        lb.lstore(lds + stage * C::STAGE + C::A_BYTES, tid);
    };
    auto gload = [&](int kt, auto masked) {
        la.template gload<decltype(masked)::value>(pa + kt * a_step, a_bytes - kt * a_step, tid, kt * BK, K, lda_b);
        lb.template gload<decltype(masked)::value>(pb + kt * b_step, b_bytes - kt * b_step, tid, kt * BK, K, ldb_b);
    };
    const std::true_type masked_t{};
    const std::false_type full_t{};

    // One k step of the software pipeline, for the slab staged in LDS stage kt&1:
    //   k-steps 0 .. NKS-3 : MFMAs of k-step ks  ||  LDS reads of the fragments of ks+1
    //   k-step  NKS-2      : ... || registers holding slab kt+1 are written to the other stage
    //   barrier (the only one per step)
    //   k-step  NKS-1      : MFMAs || LDS reads of k-step 0 of slab kt+1 || global loads of slab kt+2
    // The fragments of the first k-step are already in registers on entry.  In the steady state
    // (HOT: slabs kt+1 and kt+2 exist and need no mask) the other instructions are dealt out one
    // slot after each MFMA and fenced there, so that they issue in the shadow of the matrix pipe
    // instead of in bursts; the remaining steps take the flags and a plain order.
    constexpr int NM = TM * TN, NR = TM + TN;
    constexpr int PW = LA::PIECES + LB::PIECES;          // store (and load) pieces per slab and thread
    constexpr int SLOTS_W = NM - NM / 4 > 0 ? NM - NM / 4 : 1;   // leave the last MFMAs free so the stores drain before the barrier
    auto read_one = [&](int buf, int stage, int ks, int q) {
        const char* st = lds + stage * C::STAGE;
        if (q < TM) af[buf][q] = *(const u32x4*)(st + (fa[q] ^ (uint32_t)(ks << 5)));
        else bf[buf][q - TM] = *(const u32x4*)(st + (fb[q - TM] ^ (uint32_t)(ks << 5)));
    };
    auto step_hot = [&](int kt) {
        const int stage = kt & 1;
        char* wr = lds + (stage ^ 1) * C::STAGE;
        const __amdgpu_buffer_rsrc_t ra = make_rsrc(pa + (kt + 2) * a_step, a_bytes - (kt + 2) * a_step);
        const __amdgpu_buffer_rsrc_t rb = make_rsrc(pb + (kt + 2) * b_step, b_bytes - (kt + 2) * b_step);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            const bool last = ks == NKS - 1;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                acc[m / TN][m % TN] = mfma32<IS_BF16>(af[cur][m / TN], bf[cur][m % TN], acc[m / TN][m % TN]);
#pragma unroll
                for (int q = (m * NR) / NM; q < ((m + 1) * NR) / NM; ++q)
                    read_one(nxt, last ? stage ^ 1 : stage, last ? 0 : ks + 1, q);
                if (ks == NKS - 2 && m < SLOTS_W) {
#pragma unroll
                    for (int q = (m * PW) / SLOTS_W; q < ((m + 1) * PW) / SLOTS_W; ++q) {
                        if (q < LA::PIECES) la.store_piece(q, wr, tid);
                        else lb.store_piece(q - LA::PIECES, wr + C::A_BYTES, tid);
                    }
                }
                if (last) {
#pragma unroll
                    for (int q = (m * PW) / NM; q < ((m + 1) * PW) / NM; ++q) {
                        if (q < LA::PIECES) la.load_piece(q, ra, tid, lda_b);
                        else lb.load_piece(q - LA::PIECES, rb, tid, ldb_b);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (ks == NKS - 2) __syncthreads();
        }
    };
    auto step = [&](int kt, bool have_next, int load_mode /*0 none, 1 full, 2 masked*/) {
        const int stage = kt & 1;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks < NKS - 1) {
                read_frags(nxt, stage, ks + 1);
                if (ks == NKS - 2 && have_next) lstore(stage ^ 1);
                mfmas(cur);
                if (ks == NKS - 2) __syncthreads();
            } else {
                if (have_next) read_frags(nxt, stage ^ 1, 0);
                if (load_mode == 1) gload(kt + 2, full_t);
                else if (load_mode == 2) gload(kt + 2, masked_t);
                mfmas(cur);
            }
        }
    };

    if (k_tiles > 0) {
        if (full_tiles > 0) gload(0, full_t); else gload(0, masked_t);
        lstore(0);
        if (k_tiles > 1) { if (full_tiles > 1) gload(1, full_t); else gload(1, masked_t); }
        __syncthreads();
        read_frags(0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        for (; kt + 2 < full_tiles; ++kt) step_hot(kt);
        for (; kt < k_tiles; ++kt) {
            const int nn = kt + 2;
            step(kt, kt + 1 < k_tiles, nn < full_tiles ? 1 : (nn < k_tiles ? 2 : 0));
        }
        __syncthreads();                 // every wave is done with the operand stages: LDS is reused below
    }

    tile_epilogue<C>(acc, lds, a, m0, n0, c_vec_ok);
}

// One translation unit per variant instantiates this with its Cfg.
template <class C>
hipError_t launch_variant(const Args& a, int group_m, hipStream_t stream) {
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)a.batch), block(C::NT);
    const bool bf = a.dtype == DT_BF16;
    const bool akc = !a.transA, bkc = a.transB != 0;
    // vector access to C needs 16-byte (fp32) or 8-byte (16-bit types) aligned rows
    const int c_vec_ok = c_rows_take_vec4(a);
#define GEMM_TILE_LAUNCH(BF, AKC, BKC)                                                                       \
    hipLaunchKernelGGL((tile_kernel<C, BF, AKC, BKC>), grid, block, 0, stream, a, tiles_m, tiles_n, group_m, \
                       c_vec_ok)
    if (bf) {
        if (akc && bkc) GEMM_TILE_LAUNCH(true, true, true);
        else if (akc && !bkc) GEMM_TILE_LAUNCH(true, true, false);
        else if (!akc && bkc) GEMM_TILE_LAUNCH(true, false, true);
        else GEMM_TILE_LAUNCH(true, false, false);
    } else {
        if (akc && bkc) GEMM_TILE_LAUNCH(false, true, true);
        else if (akc && !bkc) GEMM_TILE_LAUNCH(false, true, false);
        else if (!akc && bkc) GEMM_TILE_LAUNCH(false, false, true);
        else GEMM_TILE_LAUNCH(false, false, false);
    }
#undef GEMM_TILE_LAUNCH
    return hipGetLastError();
}

}  // namespace tile
}  // namespace gemm

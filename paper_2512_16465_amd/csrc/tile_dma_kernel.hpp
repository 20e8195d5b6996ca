// The macro-tile GEMM kernel with direct-to-LDS operand loads (bf16 / fp16, gfx950).
//
// Same tiling as tile_kernel.hpp (BM x BN x BK workgroup tile, 32x32x16 MFMA accumulators per
// wave, LDS-staged epilogue), but the operand slabs travel global memory -> LDS without passing
// through registers (buffer_load ... lds, 16 bytes per lane), into a ring of NS stages, and are
// issued a few at a time between the MFMAs of the whole k step.  That removes the bursts of
// global loads and of LDS stores that the register-staged kernel suffers from (the texture path
// of a compute unit moves 64 bytes per clock, the LDS write port 128), frees 64 registers, and
// gives every load two full k steps to arrive.  It is the CDNA4 counterpart of the paper's
// "asynchronous copy" and "multi-stage pipeline" strategies (Section 5.4, Table 1).
//
// A direct-to-LDS load writes lane l of a wave to LDS byte M0 + 16*l: the destination of one
// instruction is a contiguous kilobyte.  The swizzled layouts are therefore produced on the
// global side: each lane fetches the chunk that belongs in its LDS slot.
//   k-contiguous operand (A in NN/NT, B in NT): LDS rows are k-contiguous, chunk (row, c) lives
//     in slot swz(row, c); fragments are read with ds_read_b128 as in tile_kernel.hpp.
//   m/n-contiguous operand (B in NN, A in TN): LDS holds the slab as [k][row], 16-byte chunk c of
//     k-row k in slot k*(ROWS/8) + (c xor mc_swizzle(k)); the MFMA operand (8 consecutive k of one
//     row per lane) is read with two transposing loads ds_read_b64_tr_b16, in which lane j of a
//     16-lane group supplies the address of row k0 + j/4, columns 4*(j%4).., and lane i receives
//     column i of rows k0 .. k0+3.
// Rows of a k-contiguous operand past its end return zero through the buffer descriptor's range
// check; the chunks of an m/n-contiguous operand past the tile's last valid column are clamped to
// the last valid chunk (the range check does not see the scalar k advance of the steady state); a
// partial last k slab masks the lanes whose chunk lies beyond K (k-contiguous operands) by giving
// them an out-of-range offset.
#pragma once
#include "tile_kernel.hpp"

namespace gemm {
namespace tile {

template <int BM_, int BN_, int BK_, int WM_, int WN_, int NS_>
struct DmaCfg : Cfg<BM_, BN_, BK_, WM_, WN_> {
    static constexpr int NS = NS_;     // LDS stages in the ring
    static_assert(NS_ >= 2, "one stage is multiplied while the others are filled");
};

#define GEMM_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

// One direct-to-LDS load: lane l fetches 16 bytes at byte offset `off` + `soff` of the buffer and
// the wave's 64 chunks land at LDS address `dst` + 16*l.  `soff` is wave-uniform and is NOT part
// of the descriptor's range check (only `off` is): callers add it only where every lane whose
// `off` is in range stays inside the operand.  Only the device pass of the compiler sees the
// builtin: the host pass does not accept it inside templates and would silently drop the launch
// stub of every kernel that reaches it.
__device__ __forceinline__ void load_to_lds_b128(__amdgpu_buffer_rsrc_t rsrc, char* dst, uint32_t off, uint32_t soff) {
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, GEMM_LDS_PTR(dst), 16, off, soff, 0, 0);
#else
    (void)rsrc; (void)dst; (void)off; (void)soff;
#endif
}

typedef __attribute__((ext_vector_type(4))) short s16x4;

// ---- operand movers ----

// Hash of the 128-byte line number that is XOR-ed into the chunk position of a k-contiguous slab.
// FOLD = true is the layout of tile_kernel.hpp's swz (fragments that span 32 rows: 16 lines);
// FOLD = false uses the low three bits only, which is enough for fragments that span 16 rows and
// makes the slab periodic in 1024 bytes (16 rows), so that the fragments of successive 16-row
// tiles lie at a fixed distance from each other.
template <bool FOLD>
__device__ __forceinline__ uint32_t kc_line_hash(uint32_t line) { return FOLD ? ((line ^ (line >> 3)) & 7u) : (line & 7u); }

// k-contiguous operand: ROWS x BK slab, element (row, k) at base + row*ld + k.
template <int ROWS, int BK, int NT, bool FOLD = true>
struct DmaKC {
    static constexpr int CPR = BK / 8, SLOTS = ROWS * CPR, L = SLOTS / NT;
    static constexpr int BYTES = ROWS * BK * 2;
    static constexpr bool TRANSPOSED = false;
    static_assert(SLOTS % NT == 0, "slots must divide evenly over the threads");
    uint32_t voff[L];      // byte offset of this lane's chunk from the slab's first byte

    __device__ __forceinline__ void init(int tid, int64_t ld, int /*valid_rows*/) {
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const uint32_t S = i * NT + tid;                      // LDS slot this lane fills with load i
            const uint32_t line = S >> 3;
            const uint32_t pos = (S & 7u) ^ kc_line_hash<FOLD>(line);
            const uint32_t chunk = (line << 3) | pos;             // logical chunk: row*CPR + c
            const uint32_t row = chunk / CPR, c = chunk % CPR;
            voff[i] = (uint32_t)((row * ld + c * 8) * 2);
        }
    }
    // k offset (in elements) of the chunk of load i inside the slab
    __device__ __forceinline__ int chunk_k(int i, int tid) const {
        const uint32_t S = i * NT + tid, line = S >> 3;
        const uint32_t pos = (S & 7u) ^ kc_line_hash<FOLD>(line);
        return (int)((((line << 3) | pos) % CPR) * 8);
    }
    __device__ __forceinline__ void issue(bool MASKED, int i, __amdgpu_buffer_rsrc_t rsrc, char* stage, int wave, int tid, int k0,
                                          int K, uint32_t soff = 0) const {
        uint32_t off = voff[i];
        if (MASKED && k0 + chunk_k(i, tid) >= K) off = 0x7ffffff0u;       // past the end of any supported operand: the slot is filled with zeros
        load_to_lds_b128(rsrc, stage + (i * NT + wave * 64) * 16, off, soff);
    }
    // unmasked load i whose destination is given for this wave: `wave_dst` = stage + wave * 1024
    __device__ __forceinline__ void issue_at(int i, __amdgpu_buffer_rsrc_t rsrc, char* wave_dst, uint32_t soff) const {
        load_to_lds_b128(rsrc, wave_dst + i * NT * 16, voff[i], soff);
    }
    static __device__ __forceinline__ const char* tile_base(const void* p, int64_t first_row, int64_t ld) {
        return (const char*)p + first_row * ld * 2;
    }
    static __device__ __forceinline__ int64_t k_step_bytes(int64_t /*ld*/) { return BK * 2; }
    static __device__ __forceinline__ int64_t total_bytes(int64_t rows, int64_t K, int64_t ld) { return ((rows - 1) * ld + K) * 2; }

    // fragment addressing: byte offset inside the slab of this lane's row for 32-row block t, k-chunk lhi
    static __device__ __forceinline__ uint32_t frag_base(int row0, int l32, int lhi) { return swz<CPR>(row0 + l32, lhi); }
    // fragments are ordinary LDS loads: the compiler tracks their completion itself
    typedef u32x4 Raw;
    static constexpr bool MANUAL_WAIT = false;
    static __device__ __forceinline__ void read_frag(const char* slab, uint32_t base, int ks, Raw& r) {
        r = *(const u32x4*)(slab + (base ^ (uint32_t)(ks << 5)));
    }
    static __device__ __forceinline__ u32x4 finish(const Raw& r) { return r; }
};

// Position swizzle of the [k][row] slabs: 16-byte chunk c of k-row k is stored at chunk position
// c xor mc_swizzle(k).  A transposing read takes 32 bytes from each of four consecutive k-rows
// per 16 lanes, and 32 lanes are served together: bits 2-3 spread the four k-rows over the 64-byte
// blocks of a 256-byte bank line, bit 1 separates the two 16-lane groups when they read the same
// columns of k-rows 8 apart (16x16x32 fragments).  Only bits 1-3 move, so four consecutive
// lanes of a direct-to-LDS load still fetch one aligned 64-byte piece.
__device__ __forceinline__ uint32_t mc_swizzle(uint32_t k) { return ((k & 3u) << 2) ^ (((k >> 3) & 1u) << 1); }

// m- or n-contiguous operand: element (k, row) at base + k*ld + row; LDS keeps [k][row].
template <int ROWS, int BK, int NT>
struct DmaMC {
    static constexpr int CPK = ROWS / 8, SLOTS = BK * CPK, L = SLOTS / NT;   // chunks per k-row
    static constexpr int BYTES = ROWS * BK * 2;
    static constexpr bool TRANSPOSED = true;
    static_assert(SLOTS % NT == 0 && CPK % 16 == 0, "a k-row must be whole 256-byte windows");
    uint32_t voff[L];

    // `valid_rows`: rows (columns of the stored matrix) of this tile inside the operand, a multiple
    // of 8.  Chunks beyond them would lie in the next stored row or, in the operand's last k-row,
    // past its end, and the steady state's scalar k advance escapes the range check: such lanes fetch
    // the tile's last valid chunk instead (their rows of the tile are never stored).
    __device__ __forceinline__ void init(int tid, int64_t ld, int valid_rows) {
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const uint32_t S = i * NT + tid;
            const uint32_t k = S / CPK, cs = S % CPK;
            const uint32_t c = cs ^ mc_swizzle(k);
            const uint32_t c8 = (int)(c * 8 + 8) <= valid_rows ? c * 8 : (uint32_t)(valid_rows - 8);
            voff[i] = (uint32_t)((k * ld + c8) * 2);
        }
    }
    __device__ __forceinline__ void issue(bool /*masked*/, int i, __amdgpu_buffer_rsrc_t rsrc, char* stage, int wave, int /*tid*/,
                                          int /*k0*/, int /*K*/, uint32_t soff = 0) const {
        // k-rows past K lie past the end of the operand and read as zero by themselves (as long
        // as the descriptor starts at the slab, i.e. soff == 0)
        load_to_lds_b128(rsrc, stage + (i * NT + wave * 64) * 16, voff[i], soff);
    }
    __device__ __forceinline__ void issue_at(int i, __amdgpu_buffer_rsrc_t rsrc, char* wave_dst, uint32_t soff) const {
        load_to_lds_b128(rsrc, wave_dst + i * NT * 16, voff[i], soff);
    }
    static __device__ __forceinline__ const char* tile_base(const void* p, int64_t first_row, int64_t /*ld*/) {
        return (const char*)p + first_row * 2;
    }
    static __device__ __forceinline__ int64_t k_step_bytes(int64_t ld) { return (int64_t)BK * ld * 2; }
    static __device__ __forceinline__ int64_t total_bytes(int64_t rows, int64_t K, int64_t ld) { return ((K - 1) * ld + rows) * 2; }

    // address this lane supplies to the transposing read for 32-row block starting at row0:
    // k-row (8*lhi + j/4), columns row0 + 16*((lane%32)/16) + 4*(j%4), j = lane%16
    static __device__ __forceinline__ uint32_t frag_base(int row0, int l32, int lhi) {
        const uint32_t j = l32 & 15, grp = l32 >> 4;
        const uint32_t k = 8 * lhi + (j >> 2);
        const uint32_t col = row0 + 16 * grp + 4 * (j & 3);
        const uint32_t cs = (col >> 3) ^ mc_swizzle(k);
        return (k * CPK + cs) * 16 + (col & 7) * 2;
    }
    // The transposing reads are issued as assembly: the compiler would otherwise make each of
    // them wait for every direct-to-LDS load in flight.  It therefore does not know when their
    // results arrive; the kernel waits (lgkmcnt) before the first use, see wait_raw.
    struct Raw { uint2 lo, hi; };
    static constexpr bool MANUAL_WAIT = true;
    static constexpr int KS_BYTES = 16 * CPK * 16, HALF_BYTES = 4 * CPK * 16;   // 16 and 4 k-rows further
    static_assert(KS_BYTES * (BK / 16 - 1) + HALF_BYTES < 65536, "offsets must fit the instruction's immediate");
    static __device__ __forceinline__ void read_frag(const char* slab, uint32_t base, int ks, Raw& r) {
        const uint32_t addr = (uint32_t)(uintptr_t)GEMM_LDS_PTR(slab) + base;
        static_assert(BK <= 64, "at most four k-steps per slab");
        if (ks == 0) {
            asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.lo) : "v"(addr));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(HALF_BYTES));
        } else if (ks == 1) {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.lo) : "v"(addr), "n"(KS_BYTES));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(KS_BYTES + HALF_BYTES));
        } else if (ks == 2) {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.lo) : "v"(addr), "n"(2 * KS_BYTES));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(2 * KS_BYTES + HALF_BYTES));
        } else {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.lo) : "v"(addr), "n"(3 * KS_BYTES));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(3 * KS_BYTES + HALF_BYTES));
        }
    }
    static __device__ __forceinline__ u32x4 finish(const Raw& r) { return u32x4{r.lo.x, r.lo.y, r.hi.x, r.hi.y}; }
};

// Waits until every LDS read issued so far has returned.  The raw fragments are passed through
// the statement so that nothing that consumes them can be moved ahead of the wait.
template <class Raw>
__device__ __forceinline__ void wait_raw(Raw (&r)[2]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi));
}
template <class Raw>
__device__ __forceinline__ void wait_raw(Raw (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi), "+v"(r[2].lo), "+v"(r[2].hi), "+v"(r[3].lo), "+v"(r[3].hi));
}
__device__ __forceinline__ void wait_raw(u32x4 (&)[2]) {}
__device__ __forceinline__ void wait_raw(u32x4 (&)[4]) {}

template <class C, bool IS_BF16, bool A_KC, bool B_KC, bool PLAIN>
__global__ __launch_bounds__(C::NT) void tile_dma_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok, int rotate) {
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::NT, TM = C::TM, TN = C::TN, NS = C::NS;
    using EL = EpiLayout<C>;
    constexpr int RING = NS * C::STAGE;
    constexpr int LDS_BYTES = RING > EL::BYTES ? RING : EL::BYTES;
    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
    select_batch(a);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    const int wm = wave % C::WM, wn = wave / C::WM;

    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, group_m, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    const int K = (int)a.K;

    using LA = typename std::conditional<A_KC, DmaKC<BM, BK, NT>, DmaMC<BM, BK, NT>>::type;
    using LB = typename std::conditional<B_KC, DmaKC<BN, BK, NT>, DmaMC<BN, BK, NT>>::type;
    LA la;
    LB lb;
    la.init(tid, a.lda, (int)(a.M - m0 < BM ? a.M - m0 : BM));
    lb.init(tid, a.ldb, (int)(a.N - n0 < BN ? a.N - n0 : BN));
    const char* pa = LA::tile_base(a.A, m0, a.lda);
    const char* pb = LB::tile_base(a.B, n0, a.ldb);
    const int64_t a_step = LA::k_step_bytes(a.lda), b_step = LB::k_step_bytes(a.ldb);
    const int64_t a_bytes = LA::total_bytes(a.M, a.K, a.lda) - (pa - (const char*)a.A);
    const int64_t b_bytes = LB::total_bytes(a.N, a.K, a.ldb) - (pb - (const char*)a.B);

    uint32_t fa[TM], fb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = LA::frag_base(wm * C::WTM + i * 32, l32, lhi);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = C::A_BYTES + LB::frag_base(wn * C::WTN + j * 32, l32, lhi);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int k_tiles = (K + BK - 1) / BK;
    const int full_tiles = K / BK;
    // Rotation of the k walk (`rotate`, set by the host for calls that stream from HBM an operand
    // whose rows lie a multiple of 4 KiB apart: at a given k all its rows sit on one memory channel,
    // and workgroups walking k in step would queue there).  Step t takes the slab (t + rot) mod
    // k_tiles; rot depends on the tile's index along the longer side of C, so that the tiles
    // sharing a panel of the larger operand still walk it together.  Whole slabs only.
    const int rot = (rotate && k_tiles == full_tiles && k_tiles >= 2 * NS)
                        ? (int)((unsigned)((a.N >= a.M ? tn : tm) * 10) % (unsigned)k_tiles) : 0;
    auto physical = [&](int t) { const int p = t + rot; return p >= k_tiles ? p - k_tiles : p; };
    constexpr int NKS = BK / 16;
    constexpr int NM = TM * TN, NR = TM + TN;
    constexpr int LPT = LA::L + LB::L;            // direct-to-LDS loads per thread and slab
    constexpr int D = NS - 1;                     // slab kt + D is requested while slab kt is multiplied

    typename LA::Raw af[2][TM];      // operand fragments as read from LDS, double-buffered in registers
    typename LB::Raw bf[2][TN];

    auto read_one = [&](int buf, int stage, int ks, int q) {
        const char* st = lds + stage * C::STAGE;
        if (q < TM) LA::read_frag(st, fa[q], ks, af[buf][q]);
        else LB::read_frag(st, fb[q - TM], ks, bf[buf][q - TM]);
    };
    // all MFMAs of one k-sub-step; `slot` runs after MFMA m
    auto run_mfmas = [&](int cur, auto slot) {
        if (LA::MANUAL_WAIT) wait_raw(af[cur]);
        if (LB::MANUAL_WAIT) wait_raw(bf[cur]);
        u32x4 ua[TM], ub[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) ua[i] = LA::finish(af[cur][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) ub[j] = LB::finish(bf[cur][j]);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            slot(m, 0);
            // boustrophedon order over the wave's accumulators: consecutive MFMAs share one operand
            const int i = m / TN, j = (i & 1) ? TN - 1 - m % TN : m % TN;
            acc[i][j] = mfma32<IS_BF16>(ua[i], ub[j], acc[i][j]);
            slot(m, 1);
        }
    };
    auto issue_one = [&](int q, __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, char* stage, int k0, auto masked,
                         uint32_t soff_a = 0, uint32_t soff_b = 0) {
        constexpr bool M = decltype(masked)::value;
        if (q < LA::L) la.issue(M, q, ra, stage, wave, tid, k0, K, soff_a);
        else lb.issue(M, q - LA::L, rb, stage + C::A_BYTES, wave, tid, k0, K, soff_b);
    };
    auto issue_tile = [&](int t, auto masked) {
        const int p = physical(t);
        const __amdgpu_buffer_rsrc_t ra = make_rsrc(pa + p * a_step, a_bytes - p * a_step);
        const __amdgpu_buffer_rsrc_t rb = make_rsrc(pb + p * b_step, b_bytes - p * b_step);
        char* stage = lds + (t % NS) * C::STAGE;
#pragma unroll
        for (int q = 0; q < LPT; ++q) issue_one(q, ra, rb, stage, p * BK, masked);
    };

    // The barrier of a k step: this wave's share of slab kt+1 has landed once at most `pending`
    // younger loads are outstanding (loads complete in order); after the barrier every wave's
    // share has, and every wave is done reading slab kt-... whose stage the next loads overwrite.
#define GEMM_WAIT_VM_BARRIER(N)                                                                                   \
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory")

    constexpr int BAR_SLOT = NM / 4;              // MFMAs of the last k-sub-step issued before the barrier
    // All loads of a slab are issued before its step's barrier.  With a single slab of lookahead the
    // barrier of the same step waits for them, so they go out first, one per MFMA.
    constexpr int BEFORE_BAR = (NKS - 1) * NM + BAR_SLOT;
    constexpr int LOAD_SLOTS = (D == 1 && LPT < BEFORE_BAR) ? LPT : BEFORE_BAR;

    // Steady state: slabs kt+1 .. kt+D exist and need no mask.  The descriptors stay at the tile's
    // first slab and the k advance travels as the loads' scalar offset (one scalar add per operand
    // and step): a wave has room for only a handful of instructions next to each MFMA, and
    // rebuilding two descriptors costs two dozen.  The scalar offset escapes the range check, which
    // is safe here because every lane whose own offset is in range addresses a row of the operand,
    // and slab t lies wholly inside K.
    const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa, a_bytes), rb0 = make_rsrc(pb, b_bytes);
    auto step_hot = [&](int kt) {
        const int stage = kt % NS, next = (kt + 1) % NS;
        const int t = kt + D, p = physical(t);
        const uint32_t soff_a = (uint32_t)(p * a_step), soff_b = (uint32_t)(p * b_step);
        char* dst = lds + (t % NS) * C::STAGE;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            const bool last = ks == NKS - 1;
            run_mfmas(cur, [&](int m, int after) {
                if (!after) {
                    if (last && m == BAR_SLOT) GEMM_WAIT_VM_BARRIER((D - 1) * LPT);
                    return;
                }
                if (!last) {
#pragma unroll
                    for (int q = (m * NR) / NM; q < ((m + 1) * NR) / NM; ++q) read_one(nxt, stage, ks + 1, q);
                } else if (m >= BAR_SLOT) {
                    constexpr int RS = NM - BAR_SLOT - NM / 4 > 0 ? NM - BAR_SLOT - NM / 4 : 1;   // slots used for the reads
                    const int mm = m - BAR_SLOT;
                    if (mm < RS) {
#pragma unroll
                        for (int q = (mm * NR) / RS; q < ((mm + 1) * NR) / RS; ++q) read_one(nxt, next, 0, q);
                    }
                }
                const int slot = ks * NM + m;
                if (slot < LOAD_SLOTS) {
#pragma unroll
                    for (int q = (slot * LPT) / LOAD_SLOTS; q < ((slot + 1) * LPT) / LOAD_SLOTS; ++q)
                        issue_one(q, ra0, rb0, dst, p * BK, std::false_type{}, soff_a, soff_b);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };
    // the first and last steps: flags instead of assumptions, everything outstanding is awaited
    auto step_edge = [&](int kt) {
        const int stage = kt % NS, next = (kt + 1) % NS;
        const int t = kt + D;
        if (t < full_tiles) issue_tile(t, std::false_type{});
        else if (t < k_tiles) issue_tile(t, std::true_type{});
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks < NKS - 1) {
#pragma unroll
                for (int q = 0; q < NR; ++q) read_one(nxt, stage, ks + 1, q);
            } else if (kt + 1 < k_tiles) {
                GEMM_WAIT_VM_BARRIER(0);
#pragma unroll
                for (int q = 0; q < NR; ++q) read_one(nxt, next, 0, q);
            }
            run_mfmas(cur, [](int, int) {});
        }
    };

    if (k_tiles > 0) {
#pragma unroll
        for (int t = 0; t < D; ++t) {
            if (t < full_tiles) issue_tile(t, std::false_type{});
            else if (t < k_tiles) issue_tile(t, std::true_type{});
        }
        GEMM_WAIT_VM_BARRIER(0);
#pragma unroll
        for (int q = 0; q < NR; ++q) read_one(0, 0, 0, q);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        for (; kt + D < full_tiles; ++kt) step_hot(kt);
        // at least one step is left (kt + D >= full_tiles or kt == 0, and D >= 1): a loop that is entered
        // without a test, so that no path leads from the fragment reads above past every wait for them
        do { step_edge(kt); } while (++kt < k_tiles);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS is reused by the epilogue
#undef GEMM_WAIT_VM_BARRIER

    if constexpr (PLAIN) tile_epilogue_plain<C>(acc, a, m0, n0);
    else tile_epilogue<C>(acc, lds, a, m0, n0, c_vec_ok);
}

template <class C>
hipError_t launch_dma_variant(const Args& a, int group_m, hipStream_t stream) {
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)a.batch), block(C::NT);
    const bool bf = a.dtype == DT_BF16;
    const bool akc = !a.transA, bkc = a.transB != 0;
    const int c_vec_ok = c_rows_take_vec4(a);
    const bool plain = plain_epilogue_applies<C>(a);
    // a single row or column of tiles, operands beyond the last-level cache, one of them k-contiguous with
    // rows a multiple of 4 KiB apart (65536x128x4096: 125 -> 119 us, 128x28672x8192 with B stored N x K:
    // 123 -> 105; grids with several tiles in both directions did not gain)
    const bool a_aliases = akc && (a.lda * 2) % 4096 == 0, b_aliases = bkc && (a.ldb * 2) % 4096 == 0;
    const int rotate = (a_aliases || b_aliases) && a.k_total == 0 && (tiles_m == 1 || tiles_n == 1) &&
                       (a.M + a.N) * a.K * 2 > ((int64_t)256 << 20);
#define GEMM_TILE_LAUNCH(BF, AKC, BKC)                                                                         \
    do {                                                                                                       \
        if (plain)                                                                                             \
            hipLaunchKernelGGL((tile_dma_kernel<C, BF, AKC, BKC, true>), grid, block, 0, stream, a, tiles_m,   \
                               tiles_n, group_m, c_vec_ok, rotate);                                            \
        else                                                                                                   \
            hipLaunchKernelGGL((tile_dma_kernel<C, BF, AKC, BKC, false>), grid, block, 0, stream, a, tiles_m,  \
                               tiles_n, group_m, c_vec_ok, rotate);                                            \
    } while (0)
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

// Direct-to-LDS macro-tile kernel built on the 16x16x32 MFMA (bf16 / fp16, gfx950).
//
// Same operand movers and LDS layouts as tile_dma_kernel.hpp; what changes is the matrix
// instruction and, with it, the pipeline.  v_mfma_f32_16x16x32 does the same work per cycle as
// the 32x32x16 form but sums 32 products into each accumulator per instruction instead of 16, so
// the accumulator registers are read and written half as often per flop.  On this part the
// matrix pipeline is power-limited on real (non-constant) data, and that difference decides the
// sustained clock: a register-only loop on Gaussian bf16 data holds 2.06 GHz with 16x16x32
// against 1.81 GHz with 32x32x16 (2.07 vs 1.68 PFLOP/s).
//
// A wave's sub-block is a grid of 16x16 accumulators (4 registers each).  Per 32 of k a wave
// reads one 16-byte fragment per 16 rows of A and per 16 columns of B:
//   operand A of the MFMA: lane l holds row l%16, k = 8*(l/16) .. +7; operand B: column l%16,
//   same k; accumulator register v of lane l is row 4*(l/16)+v, column l%16.
//   k-contiguous operand: one ds_read_b128 of chunk (row, l/16) of the swizzled slab; the slab
//   is periodic in 16 rows (kc_line_hash<false>), so tile i is tile 0's address + 1024*i.
//   m/n-contiguous operand ([k][row] slab): two ds_read_b64_tr_b16; lane j of a 16-lane group
//   supplies k-row 8*(l/16) + j/4 (+4 for the second read), columns 4*(j%4)...
//
// One wave per SIMD issues one instruction every four cycles and an MFMA lasts sixteen: next to
// each MFMA there is room for three other instructions (two if they are vector ALU).  The steady
// state is therefore laid out slot by slot (slot m follows MFMA m), all fragment reads are
// assembly with fixed addresses + immediates, and the scalar bookkeeping of the next two steps is
// done in the otherwise empty slots at the end of a step.
#pragma once
#include <utility>
#include "tile_dma_kernel.hpp"

namespace gemm {
namespace tile {

// c += a * b, in place, accumulator in the accumulation registers.  Written as assembly: with 64
// small accumulators per wave the compiler's register allocation otherwise gives the result a
// register of its own and shuffles accumulators around every MFMA.  None of the accumulators is
// touched twice within 64 MFMAs and the fragments come from LDS reads (awaited by counter), so the
// loop needs no wait states; the code after the loop supplies those between the last MFMA and
// the first read of an accumulator.
template <bool IS_BF16>
__device__ __forceinline__ void mfma16(f32x4& c, u32x4 a, u32x4 b) {
    if constexpr (IS_BF16) asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
    else asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(a), "v"(b));
}

// ---- fragment readers for 16-row tiles ----
// Both take absolute LDS byte addresses and are assembly, so the compiler neither reorders them
// nor waits for them: the kernel waits (lgkmcnt) itself before the fragments are used.

// Registers of a fragment between its LDS read and the wait for it.  The value of a k-contiguous operand is
// the one 16-byte register group that the read defines, and it stays whole until the wait has named it: a
// value taken apart before the wait (two halves, say) may be put together again by register copies that the
// compiler is free to place ahead of the wait, where they would copy what the registers held before.
struct Frag16RawKC { u32x4 q; };
struct Frag16RawMC { u32x2 lo, hi; };
__device__ __forceinline__ u32x4 frag16_value(const Frag16RawKC& r) { return r.q; }
__device__ __forceinline__ u32x4 frag16_value(const Frag16RawMC& r) { return u32x4{r.lo.x, r.lo.y, r.hi.x, r.hi.y}; }

template <int ROWS, int BK>
struct Frag16KC {
    static constexpr int CPR = BK / 8;
    static_assert(BK == 32, "one 32-wide k block per slab");
    static constexpr bool PER_TILE_ADDRESS = false;            // tile i = tile 0 + 1024 * i
    // byte offset inside the operand's slab of this lane's chunk of the tile that starts at row0
    static __device__ __forceinline__ uint32_t base(int row0, int lane) {
        const uint32_t chunk = (uint32_t)(row0 + (lane & 15)) * CPR + (uint32_t)(lane >> 4);
        const uint32_t line = chunk >> 3;
        return (line << 7) | (((chunk & 7u) ^ kc_line_hash<false>(line)) << 4);
    }
    typedef Frag16RawKC Raw;
    template <int TILE>
    static __device__ __forceinline__ void read(uint32_t addr, Frag16RawKC& r) {
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r.q) : "v"(addr), "n"(TILE * 1024));
    }
};

template <int ROWS, int BK>
struct Frag16MC {
    static constexpr int CPK = ROWS / 8;
    static_assert(BK == 32, "one 32-wide k block per slab");
    static constexpr bool PER_TILE_ADDRESS = true;             // the swizzle is not additive in the tile index
    static __device__ __forceinline__ uint32_t base(int row0, int lane) {
        const uint32_t j = lane & 15, g = lane >> 4;
        const uint32_t k = 8 * g + (j >> 2);
        const uint32_t col = row0 + 4 * (j & 3);
        const uint32_t cs = (col >> 3) ^ mc_swizzle(k);
        return (k * CPK + cs) * 16 + (col & 7) * 2;
    }
    static constexpr int HALF_BYTES = 4 * CPK * 16;            // 4 k-rows further
    typedef Frag16RawMC Raw;
    template <int TILE>
    static __device__ __forceinline__ void read(uint32_t addr, Frag16RawMC& r) {
        asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.lo) : "v"(addr));
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(HALF_BYTES));
    }
};

__device__ __forceinline__ void wait_raw8(Frag16RawKC (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0].q), "+v"(r[1].q), "+v"(r[2].q), "+v"(r[3].q));
}
__device__ __forceinline__ void wait_raw8(Frag16RawKC (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0].q), "+v"(r[1].q), "+v"(r[2].q), "+v"(r[3].q), "+v"(r[4].q), "+v"(r[5].q), "+v"(r[6].q), "+v"(r[7].q));
}
__device__ __forceinline__ void wait_raw8(Frag16RawMC (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi), "+v"(r[2].lo), "+v"(r[2].hi), "+v"(r[3].lo), "+v"(r[3].hi));
}
__device__ __forceinline__ void wait_raw8(Frag16RawMC (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi), "+v"(r[2].lo), "+v"(r[2].hi), "+v"(r[3].lo), "+v"(r[3].hi),
                   "+v"(r[4].lo), "+v"(r[4].hi), "+v"(r[5].lo), "+v"(r[5].hi), "+v"(r[6].lo), "+v"(r[6].hi), "+v"(r[7].lo), "+v"(r[7].hi));
}

// Pipeline (BK = 32, one 64-MFMA step per slab).  During step kt a wave multiplies the
// fragments of slab kt, which it read from LDS during step kt-1, so LDS holds slabs kt+1 (being
// read) .. kt+NS-1 or kt+NS, and the stage of slab kt is free as soon as every wave has passed
// the barrier of step kt.  That barrier sits four MFMAs into the step; behind it the step reads
// the 16 fragments of slab kt+1 (one per two MFMAs, in the order the MFMAs will want them) and
// requests new slabs (one load per four MFMAs, in the slots between the reads):
//   ring of 4: slab kt+4 into the stage of slab kt;
//   ring of 5, "paired": a k-contiguous operand contributes 64 bytes per row and slab, half a
//     cache line, and the L2 serves a half-line request at the cost of a full one (16 TB/s
//     of half lines against 27 TB/s of full lines measured for this tile stream), so slabs are
//     requested in pairs (2j, 2j+1) with the two loads that fetch the two halves of the same rows
//     next to each other, which the L1 merges into one line request.  Even step kt: first half
//     of the rows of pair (kt+4, kt+5); odd step kt: second half of pair (kt+3, kt+4).  An
//     n-contiguous operand already fetches whole lines; its even slab goes in the even step.
// Loads complete in order, so the barrier's wait counts the younger ones that may stay in
// flight: two slabs in the ring of 4; in the ring of 5 the next pair (even step) or its first
// half (odd step).
//
// Tiles numbered >= split_first are computed by split_parts workgroups each (see TileSplit): such
// a workgroup runs the same pipeline over its share of the k slabs and stores its accumulators,
// unscaled, as an fp32 tile in `partials`.
template <class C, bool IS_BF16, bool A_KC, bool B_KC, bool DIRECT = false>
__global__ __launch_bounds__(C::NT) void tile_dma16_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok,
                                                           int split_first, int split_parts, float* partials, int rotate) {
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::NT, NS = C::NS;
    constexpr int TM = C::WTM / 16, TN = C::WTN / 16;        // 16x16 accumulators per wave
    static_assert((TM == 8 || TM == 4) && (TN == 8 || TN == 4),
                  "the slot plan below is written for a 128x128 wave sub-block, half or a quarter of one");
    static_assert(BK == 32, "one 32-wide k block per slab");
    static_assert(NS == 4 || NS == 5, "ring of 4, or ring of 5 with paired requests");
    constexpr bool PAIRED = NS == 5;
    using EL = EpiLayout<C>;
    constexpr int RING = NS * C::STAGE;
    constexpr int LDS_BYTES = RING > EL::BYTES ? RING : EL::BYTES;
    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];
    select_batch(a);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % C::WM, wn = wave / C::WM;

    int pid = (int)blockIdx.x, part = -1;
    if (pid >= split_first) {
        const int r = pid - split_first;
        part = r % split_parts;
        pid = split_first + r / split_parts;
    }
    int tm, tn;
    tile_of_workgroup(pid, tiles_m, tiles_n, group_m, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    // this workgroup's share of the k slabs: [slab0, slab0 + k_tiles), K counted from slab0
    const int all_tiles = (int)((a.K + BK - 1) / BK);
    // (shares start at even slabs, so that paired requests still cover whole cache lines)
    const int slab0 = part <= 0 ? 0 : (int)((int64_t)part * all_tiles / split_parts) & ~1;
    const int slab1 = (part < 0 || part == split_parts - 1) ? all_tiles : (int)((int64_t)(part + 1) * all_tiles / split_parts) & ~1;
    const int K = (int)a.K - slab0 * BK;

    using LA = typename std::conditional<A_KC, DmaKC<BM, BK, NT, false>, DmaMC<BM, BK, NT>>::type;
    using LB = typename std::conditional<B_KC, DmaKC<BN, BK, NT, false>, DmaMC<BN, BK, NT>>::type;
    using FA = typename std::conditional<A_KC, Frag16KC<BM, BK>, Frag16MC<BM, BK>>::type;
    using FB = typename std::conditional<B_KC, Frag16KC<BN, BK>, Frag16MC<BN, BK>>::type;
    static_assert(LA::L % 2 == 0 && LB::L % 2 == 0, "a slab is requested in two halves");
    LA la;
    LB lb;
    la.init(tid, a.lda, (int)(a.M - m0 < BM ? a.M - m0 : BM));
    lb.init(tid, a.ldb, (int)(a.N - n0 < BN ? a.N - n0 : BN));
    const int64_t a_step = LA::k_step_bytes(a.lda), b_step = LB::k_step_bytes(a.ldb);
    const char* pa = LA::tile_base(a.A, m0, a.lda) + slab0 * a_step;
    const char* pb = LB::tile_base(a.B, n0, a.ldb) + slab0 * b_step;
    const int64_t a_bytes = LA::total_bytes(a.M, a.K, a.lda) - (pa - (const char*)a.A);
    const int64_t b_bytes = LB::total_bytes(a.N, a.K, a.ldb) - (pb - (const char*)a.B);

    // LDS addresses of this lane's fragments in stage 0: one per operand, or one per tile
    constexpr int NFA = FA::PER_TILE_ADDRESS ? TM : 1, NFB = FB::PER_TILE_ADDRESS ? TN : 1;
    const uint32_t lds0 = (uint32_t)(uintptr_t)GEMM_LDS_PTR(lds);
    uint32_t fa[NFA], fb[NFB];
#pragma unroll
    for (int i = 0; i < NFA; ++i) fa[i] = lds0 + FA::base(wm * C::WTM + i * 16, lane);
#pragma unroll
    for (int j = 0; j < NFB; ++j) fb[j] = lds0 + C::A_BYTES + FB::base(wn * C::WTN + j * 16, lane);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int k_tiles = slab1 - slab0;
    const int full_tiles = K / BK < k_tiles ? K / BK : k_tiles;
    // Rotation of the k walk (`rotate`, set by the host for streaming calls whose k-contiguous
    // operand has rows a large power of two apart): at a given k every row of such an operand
    // lies on the same memory channel, so workgroups that walked k in step would queue on a few
    // channels.  This workgroup takes its slabs in the order rot, rot+1, ..., k_tiles-1, 0, ...,
    // rot-1 (rot even, so that pairs of slabs still cover whole cache lines); the sum over k is
    // taken in that order, a fixed function of the tile.  Needs whole slabs and an even count.
    // The start depends on the tile's index along the longer side of C only: tiles that share a
    // panel of the larger operand keep walking it in step, so one fetch still serves them all.
    const int rot_key = a.N >= a.M ? tn : tm;
    const int rot = (rotate && k_tiles == full_tiles && (k_tiles & 1) == 0 && k_tiles >= 2 * NS)
                        ? 2 * (int)((unsigned)(rot_key * 5 + (part > 0 ? part : 0) * 3) % (unsigned)(k_tiles / 2)) : 0;
    auto physical = [&](int t) { const int p = t + rot; return p >= k_tiles ? p - k_tiles : p; };   // slab in memory of step t
    constexpr int NM = TM * TN, NR = TM + TN;     // MFMAs and fragments per step
    constexpr int LPT = LA::L + LB::L;            // loads per thread and slab (= per half of a pair)

    typename FA::Raw af[2][TM];                   // fragments of two consecutive slabs
    typename FB::Raw bf[2][TN];

    // Fragment q of the slab in the stage at byte offset `off`, in the order the MFMAs first need
    // them: A0, B0..B7, A1..A7.  `ka`, `kb`: fragment addresses of tile 0 in that stage, for the
    // operands that need only one.
    auto read_a = [&](auto tile, int buf, uint32_t off, uint32_t ka) {
        constexpr int T = decltype(tile)::value;
        if constexpr (FA::PER_TILE_ADDRESS) FA::template read<T>(fa[T % NFA] + off, af[buf][T]);
        else FA::template read<T>(ka, af[buf][T]);
    };
    auto read_b = [&](auto tile, int buf, uint32_t off, uint32_t kb) {
        constexpr int T = decltype(tile)::value;
        if constexpr (FB::PER_TILE_ADDRESS) FB::template read<T>(fb[T % NFB] + off, bf[buf][T]);
        else FB::template read<T>(kb, bf[buf][T]);
    };
    auto read_one = [&](auto qc, int buf, uint32_t off, uint32_t ka, uint32_t kb) {
        constexpr int q = decltype(qc)::value;
        if constexpr (q == 0) read_a(std::integral_constant<int, 0>{}, buf, off, ka);
        else if constexpr (q <= TN) read_b(std::integral_constant<int, (q - 1) % TN>{}, buf, off, kb);
        else read_a(std::integral_constant<int, (q - TN) % TM>{}, buf, off, ka);
    };
    auto read_all = [&](int buf, uint32_t off) {
        const uint32_t ka = fa[0] + off, kb = fb[0] + off;
        [&]<int... Q>(std::integer_sequence<int, Q...>) { (read_one(std::integral_constant<int, Q>{}, buf, off, ka, kb), ...); }
        (std::make_integer_sequence<int, NR>{});
    };
    auto run_mfmas = [&](int cur, auto slot) {
        wait_raw8(af[cur]);
        wait_raw8(bf[cur]);
        u32x4 ua[TM], ub[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) ua[i] = frag16_value(af[cur][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) ub[j] = frag16_value(bf[cur][j]);
        [&]<int... M>(std::integer_sequence<int, M...>) {
            ([&] {
                slot(std::integral_constant<int, M>{}, std::false_type{});
                constexpr int i = M / TN, j = (i & 1) ? TN - 1 - M % TN : M % TN;     // boustrophedon: consecutive MFMAs share an operand
                mfma16<IS_BF16>(acc[i][j], ub[j], ua[i]);      // the block of C transposed: see the epilogue
                slot(std::integral_constant<int, M>{}, std::true_type{});
            }(), ...);
        }
        (std::make_integer_sequence<int, NM>{});
    };

    // ---- what a step requests ----
    // Load q (0 .. LPT-1) of a step: operand, which of the two slabs (kt_even+4, kt_even+5) of the
    // current pair of steps, instruction of that slab.  Ring of 4: all of slab kt+4.  Ring of 5:
    // see above; a k-contiguous operand alternates the two slabs, an n-contiguous one takes one
    // slab per step.
    struct Pick { bool is_a; int which, i; };
    auto pick = [](bool even, int q) -> Pick {
        const bool is_a = q < LA::L;
        const int r = is_a ? q : q - LA::L;
        const int L = is_a ? LA::L : LB::L;
        const bool transposed = is_a ? LA::TRANSPOSED : LB::TRANSPOSED;
        if (!PAIRED || transposed) return Pick{is_a, even ? 0 : 1, r};
        return Pick{is_a, r & 1, (even ? 0 : L / 2) + (r >> 1)};
    };
    // first and last steps: a descriptor per slab (its range check cuts off k-rows past K), a
    // mask for the chunks of a partial slab, nothing for slabs past the end
    auto issue_checked = [&](int kt_even, bool even, int q) {
        const Pick p = pick(even, q);
        const int t = kt_even + 4 + p.which;
        if (t >= k_tiles) return;
        char* stage = lds + (t % NS) * C::STAGE;
        const int pt = physical(t);
        if (p.is_a) {
            const __amdgpu_buffer_rsrc_t r = make_rsrc(pa + pt * a_step, a_bytes - pt * a_step);
            if (pt < full_tiles) la.issue(false, p.i, r, stage, wave, tid, pt * BK, K);
            else la.issue(true, p.i, r, stage, wave, tid, pt * BK, K);
        } else {
            const __amdgpu_buffer_rsrc_t r = make_rsrc(pb + pt * b_step, b_bytes - pt * b_step);
            if (pt < full_tiles) lb.issue(false, p.i, r, stage + C::A_BYTES, wave, tid, pt * BK, K);
            else lb.issue(true, p.i, r, stage + C::A_BYTES, wave, tid, pt * BK, K);
        }
    };

#define GEMM_WAIT_VM_BARRIER(N) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory")

    // Slot plan of a step: barrier before MFMA BAR_SLOT; fragment q of the next slab after MFMA
    // BAR_SLOT + 2q; load q after MFMA LOAD_FIRST + 4q (odd slots); the scalars of the next pair
    // of steps from slot TAIL_FIRST on.
    // The scalar updates change what the loads of the step use, so they come after the last load.
    // A half-size wave sub-block has 32 MFMAs per step: its updates go two to a slot, next to the
    // last fragment reads (which use a copy of their stage offset taken at the start of the step).
    // A quarter-size sub-block (64x64) has 16 MFMAs per step: a fragment read after every MFMA, a
    // load after every second one, the updates three to a slot.
#ifndef GEMM_DMA16_PIPELINED_TAIL
#define GEMM_DMA16_PIPELINED_TAIL 1
#endif
#ifndef GEMM_DMA16_SPREAD
#define GEMM_DMA16_SPREAD 1
#endif
    // Full sub-block (64 MFMAs per step): the 16 fragment reads are spread over the step, one after every
    // third MFMA, and the loads go one after every sixth: four waves reading a kilobyte after every second
    // MFMA would ask the LDS for all of its 128 bytes per clock for the first half of the step, on top of
    // the slabs arriving from memory, and a wave whose read finds the LDS queue full stops issuing MFMAs.
    constexpr bool SPREAD = GEMM_DMA16_SPREAD && NM == 64;
    constexpr int BAR_SLOT = 4, LOAD_FIRST = BAR_SLOT + 1, LOAD_EVERY = SPREAD ? 6 : (NM >= 32 ? 4 : 2),
                  READ_EVERY = SPREAD ? 3 : (NM >= 32 ? 2 : 1);
    constexpr int LAST_LOAD = LOAD_FIRST + (LPT - 1) * LOAD_EVERY;
    constexpr int TAIL_FIRST = NM == 64 ? (SPREAD ? 50 : 40) : LAST_LOAD + 1;
    constexpr int TAIL_PACK = NM == 32 ? 2 : 3;
    // slot of scalar update u (0 .. 9)
    auto tail_slot = [](int u) {
        constexpr int wide[10] = {0, 2, 4, 6, 8, 9, 10, 11, 12, 13};
        return TAIL_FIRST + (NM == 64 ? (SPREAD ? u : wide[u]) : u / TAIL_PACK);
    };
    static_assert(BAR_SLOT + READ_EVERY * (NR - 1) < NM && LAST_LOAD < TAIL_FIRST, "reads end inside the step, loads before the tail");
    static_assert(TAIL_FIRST + (NM == 64 ? 13 : 9 / TAIL_PACK) < NM, "the scalar updates fit the step");
    // loads that may still be in flight when slab kt+1 must have landed
    constexpr int PENDING_EVEN = PAIRED ? 2 * LPT : (NS - 2) * LPT, PENDING_ODD = PAIRED ? LPT : (NS - 2) * LPT;

    // Scalars of a pair of steps (kt even, kt+1): byte offsets of the stages read in the two steps
    // (slabs kt+1, kt+2) and written (slabs kt+4, kt+5), and the operands' byte offsets of the
    // written slabs.  Advanced by two slabs in the tail of the odd step.
    struct Sched { uint32_t r1, r2, w0, w1, sa0, sa1, sb0, sb1; };
    auto stage_off = [](int pos) { return (uint32_t)((pos % NS) * C::STAGE); };
    auto advance2 = [](uint32_t off) { const uint32_t n = off + 2 * C::STAGE; return n >= (uint32_t)RING ? n - RING : n; };
    const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa, a_bytes), rb0 = make_rsrc(pb, b_bytes);
    char* const wave_lds = lds + wave * 1024;
    const uint32_t span_a = (uint32_t)(k_tiles * a_step), span_b = (uint32_t)(k_tiles * b_step);   // bytes of the whole k walk

    // Steady state: every slab requested exists and lies wholly inside K; the k advance is the
    // loads' scalar offset, which the range check ignores (see load_to_lds_b128).
    // `da0`, `da1`, `db0`, `db1`: descriptors of A and B for the loads of the first and the second slab of
    // the pair (the operands' own in the steady state).
    auto step_hot = [&](Sched& s, auto parity, __amdgpu_buffer_rsrc_t da0, __amdgpu_buffer_rsrc_t da1, __amdgpu_buffer_rsrc_t db0,
                        __amdgpu_buffer_rsrc_t db1) {
        constexpr bool EVEN = decltype(parity)::value == 0;
        constexpr int cur = EVEN ? 0 : 1, nxt = cur ^ 1;
        const uint32_t roff = EVEN ? s.r1 : s.r2;
        uint32_t ka = 0, kb = 0;
        run_mfmas(cur, [&](auto mc, auto after) {
            constexpr int m = decltype(mc)::value;
            if constexpr (!decltype(after)::value) {
                if constexpr (m == BAR_SLOT) GEMM_WAIT_VM_BARRIER(EVEN ? PENDING_EVEN : PENDING_ODD);
            } else {
                if constexpr (m == 1) ka = fa[0] + roff;
                if constexpr (m == 2) kb = fb[0] + roff;
                if constexpr (m >= BAR_SLOT && (m - BAR_SLOT) % READ_EVERY == 0 && (m - BAR_SLOT) / READ_EVERY < NR)
                    read_one(std::integral_constant<int, (m - BAR_SLOT) / READ_EVERY % NR>{}, nxt, roff, ka, kb);
                if constexpr (m >= LOAD_FIRST && (m - LOAD_FIRST) % LOAD_EVERY == 0 && (m - LOAD_FIRST) / LOAD_EVERY < LPT) {
                    const Pick p = pick(EVEN, (m - LOAD_FIRST) / LOAD_EVERY);
                    char* dst = wave_lds + (p.which ? s.w1 : s.w0);
                    if (p.is_a) la.issue_at(p.i, p.which ? da1 : da0, dst, p.which ? s.sa1 : s.sa0);
                    else lb.issue_at(p.i, p.which ? db1 : db0, dst + C::A_BYTES, p.which ? s.sb1 : s.sb0);
                }
                if constexpr (!EVEN) {      // next pair of steps: everything moves on by two slabs
                    if constexpr (m == tail_slot(0)) s.r1 = advance2(s.r1);
                    if constexpr (m == tail_slot(1)) s.r2 = advance2(s.r2);
                    if constexpr (m == tail_slot(2)) s.w0 = advance2(s.w0);
                    if constexpr (m == tail_slot(3)) s.w1 = advance2(s.w1);
                    if constexpr (m == tail_slot(4)) { s.sa0 += (uint32_t)(2 * a_step); s.sa1 += (uint32_t)(2 * a_step); }
                    if constexpr (m == tail_slot(5)) { s.sb0 += (uint32_t)(2 * b_step); s.sb1 += (uint32_t)(2 * b_step); }
                    // a rotated walk wraps around the end of the k range (never reached without rotation)
                    if constexpr (m == tail_slot(6)) s.sa0 = s.sa0 >= span_a ? s.sa0 - span_a : s.sa0;
                    if constexpr (m == tail_slot(7)) s.sa1 = s.sa1 >= span_a ? s.sa1 - span_a : s.sa1;
                    if constexpr (m == tail_slot(8)) s.sb0 = s.sb0 >= span_b ? s.sb0 - span_b : s.sb0;
                    if constexpr (m == tail_slot(9)) s.sb1 = s.sb1 >= span_b ? s.sb1 - span_b : s.sb1;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        });
    };
    auto step_edge = [&](int kt, auto parity) {
        constexpr bool EVEN = decltype(parity)::value == 0;
        constexpr int cur = EVEN ? 0 : 1, nxt = cur ^ 1;
        if (kt + 1 < k_tiles) {
            GEMM_WAIT_VM_BARRIER(0);
#pragma unroll
            for (int q = 0; q < LPT; ++q) issue_checked(EVEN ? kt : kt - 1, EVEN, q);
            read_all(nxt, stage_off(kt + 1));
        }
        run_mfmas(cur, [](auto, auto) {});
    };
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;

    if (k_tiles > 0) {
        // slabs 0 .. 3: what the two pairs of steps "before the first" would have requested
#pragma unroll
        for (int kt_even = -4; kt_even < 0; kt_even += 2) {
#pragma unroll
            for (int q = 0; q < LPT; ++q) issue_checked(kt_even, true, q);
#pragma unroll
            for (int q = 0; q < LPT; ++q) issue_checked(kt_even, false, q);
        }
        GEMM_WAIT_VM_BARRIER(0);
        read_all(0, 0);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        Sched s{stage_off(1), stage_off(2), stage_off(4), stage_off(5), (uint32_t)(physical(4) * a_step), (uint32_t)(physical(5) * a_step),
                (uint32_t)(physical(4) * b_step), (uint32_t)(physical(5) * b_step)};
        for (; kt + 1 + NS < full_tiles; kt += 2) {      // the two steps request slabs up to kt + 5
            step_hot(s, Even{}, ra0, ra0, rb0, rb0);
            step_hot(s, Odd{}, ra0, ra0, rb0, rb0);
        }
        if (GEMM_DMA16_PIPELINED_TAIL && k_tiles == full_tiles) {
            // Whole slabs only: the last steps are steady-state steps too.  A slab past the end is
            // requested through a descriptor of length zero: the load fetches nothing, but it is issued
            // and completes in order like any other, so the wait counts of the steps (loads that may
            // stay in flight behind the slab needed next) remain exact, and what it writes, if
            // anything, goes to a stage that no later step reads.  The very last step also reads
            // fragments of a slab that does not exist; nothing multiplies them.
            const __amdgpu_buffer_rsrc_t ra_none = make_rsrc(pa, 0), rb_none = make_rsrc(pb, 0);
            for (; kt < k_tiles; kt += 2) {
                const bool has0 = kt + 4 < k_tiles, has1 = kt + 5 < k_tiles;
                const __amdgpu_buffer_rsrc_t da0 = has0 ? ra0 : ra_none, da1 = has1 ? ra0 : ra_none;
                const __amdgpu_buffer_rsrc_t db0 = has0 ? rb0 : rb_none, db1 = has1 ? rb0 : rb_none;
                step_hot(s, Even{}, da0, da1, db0, db1);
                if (kt + 1 < k_tiles) step_hot(s, Odd{}, da0, da1, db0, db1);
            }
        }
        for (; kt < k_tiles; kt += 2) {                 // a partial last slab: per-slab descriptors, masks, full waits
            step_edge(kt, Even{});
            if (kt + 1 < k_tiles) step_edge(kt + 1, Odd{});
        }
    }
    // LDS is reused by the epilogue; the wait states let the last MFMAs retire before their results are read
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#undef GEMM_WAIT_VM_BARRIER

    // a share of a split tile goes, as it is, to its fp32 tile among the partials
    Args e = a;
    int64_t em0 = m0, en0 = n0;
    const int64_t live_rows = a.M - m0;       // rows of the tile inside C: bands below them are not stored (nor read back)
    if (part >= 0) {
        e.C = partials + ((size_t)(pid - split_first) * split_parts + part) * (BM * BN);
        e.ldc = BN; e.M = BM; e.N = BN;
        e.out_dtype = DT_F32; e.alpha = 1.0f; e.beta = 0.0f; e.bias = nullptr; e.act = ACT_NONE;
        em0 = 0; en0 = 0; c_vec_ok = 1;
    }
    // The MFMAs took B's fragment as their first operand, so each 16x16 accumulator holds its block
    // of C transposed: register v of lane l is row l%16, column 4*(l/16) + v, and a lane's four
    // registers are four consecutive columns, parked with one 16-byte LDS write.
    const int c16 = lane & 15, g4 = lane >> 4;
    if constexpr (DIRECT) {
        // Whole tiles of a 16-bit C without C_in, bias or activation (the launcher checks) leave from the
        // registers: no pass through LDS and none of its waits.  A lane's four columns of a block are 8 bytes
        // once rounded; two neighbouring blocks trade halves (v_permlane16_swap: the odd 16-lane rows of its
        // first operand against the even rows of its second), which gives every lane 16 contiguous bytes and
        // every row of C 64; then the two halves of each 16-lane row trade pieces (a rotation by 8 under a
        // bank mask), which brings the two 64-byte halves of a 128-byte line into one instruction, eight rows
        // per store.  (Stores of 64-byte pieces make the L2 write lines twice.)
        // Nothing below moves above the wait that ends the k loop:
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) asm volatile("" : "+a"(acc[i][j]));
        const float alpha = a.alpha;
        const bool to_bf16 = a.out_dtype == DT_BF16;
        const int r8 = c16 & 7, up = c16 >> 3;
        const int64_t row0 = m0 + wm * C::WTM + r8;
        const int64_t col = n0 + wn * C::WTN + 32 * up + 16 * (g4 & 1) + 8 * (g4 >> 1);
        char* p = (char*)a.C + (row0 * a.ldc + col) * 2;
        const int64_t row_step = (int64_t)16 * a.ldc * 2, half_step = (int64_t)8 * a.ldc * 2;
        auto pack = [&](const f32x4& v) {
            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
            typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
            const f32x4 s = alpha * v;
            return to_bf16 ? __builtin_bit_cast(u32x2, __builtin_convertvector(s, bf16x4)) : __builtin_bit_cast(u32x2, __builtin_convertvector(s, f16x4));
        };
        auto piece = [&](const f32x4& left, const f32x4& right) {
            const u32x2 pl = pack(left), pr = pack(right);
            const auto lo = __builtin_amdgcn_permlane16_swap(pl.x, pr.x, false, false);
            const auto hi = __builtin_amdgcn_permlane16_swap(pl.y, pr.y, false, false);
            return u32x4{lo[0], hi[0], lo[1], hi[1]};
        };
        static_assert(TN % 4 == 0, "a line is four blocks wide");
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int q = 0; q < TN / 4; ++q) {
                const u32x4 lower = piece(acc[i][4 * q], acc[i][4 * q + 1]), upper = piece(acc[i][4 * q + 2], acc[i][4 * q + 3]);
                u32x4 d0, d1;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    d0[e] = (uint32_t)__builtin_amdgcn_update_dpp((int)lower[e], (int)upper[e], 0x128, 0xf, 0xc, false);     // row_ror:8
                    d1[e] = (uint32_t)__builtin_amdgcn_update_dpp((int)upper[e], (int)lower[e], 0x128, 0xf, 0x3, false);
                }
                __builtin_nontemporal_store(d0, (u32x4*)(p + i * row_step + q * 128));
                __builtin_nontemporal_store(d1, (u32x4*)(p + i * row_step + half_step + q * 128));
            }
        }
        return;
    }
    tile_epilogue_bands<C>(
        [&](auto band, char* region) {
            constexpr int b = decltype(band)::value;
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    *(f32x4*)(region + ((16 * i2 + c16) * EL::RS + j * 16 + 4 * g4) * 4) = acc[2 * b + i2][j];
        },
        lds, e, em0, en0, c_vec_ok, live_rows);
}

template <class C>
hipError_t launch_dma16_variant(const Args& a, int group_m, const TileSplit& split, hipStream_t stream) {
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const int tiles = tiles_m * tiles_n;
    const bool splits = split.parts > 1 && split.first_tile < tiles;
    const int split_first = splits ? split.first_tile : tiles, split_parts = splits ? split.parts : 1;
    const dim3 grid((unsigned)(split_first + (tiles - split_first) * split_parts), (unsigned)a.batch), block(C::NT);
    const bool bf = a.dtype == DT_BF16;
    const bool akc = !a.transA, bkc = a.transB != 0;
    const int c_vec_ok = c_rows_take_vec4(a);
    // A split call streams its operands (few tiles, long k), and so does a single row or column of
    // tiles whose operands exceed the last-level cache: rotate the k walk when a k-contiguous
    // operand has its rows a multiple of 4 KiB apart (see the kernel).  With more than four shares
    // per tile the shares themselves spread the workgroups over k, and a rotation would only stop
    // the tiles of one share from walking the smaller operand together (1024x512x65536 in 16 shares
    // on 128x256 tiles: 104 us rotated, 69 unrotated).
    const bool a_aliases = akc && (a.lda * 2) % 4096 == 0, b_aliases = bkc && (a.ldb * 2) % 4096 == 0;
    const bool one_panel_each = (tiles_m == 1 || tiles_n == 1) && (a.M + a.N) * a.K * 2 > ((int64_t)256 << 20);
    const int rotate = ((splits && split.parts <= 4) || one_panel_each) && (a_aliases || b_aliases);
    // whole tiles of a 16-bit C with nothing but alpha in the epilogue: the instances that store from the registers
    // (an fp32 C gains nothing from it: 713 against 715 us at 8192^3)
    constexpr bool HAS_DIRECT = C::NS == 5;
    const bool direct = HAS_DIRECT && !splits && a.out_dtype != DT_F32 && a.beta == 0.0f && a.bias == nullptr && a.act == ACT_NONE &&
                        a.M % C::BM == 0 && a.N % C::BN == 0 && a.ldc % 8 == 0 && ((uintptr_t)a.C & 15) == 0 &&
                        (a.batch == 1 || (a.strideC * 2) % 16 == 0);
#define GEMM_TILE_LAUNCH(BF, AKC, BKC)                                                                                          \
    do {                                                                                                                        \
        if constexpr (HAS_DIRECT) {                                                                                             \
            if (direct) {                                                                                                       \
                hipLaunchKernelGGL((tile_dma16_kernel<C, BF, AKC, BKC, true>), grid, block, 0, stream, a, tiles_m, tiles_n, group_m, \
                                   c_vec_ok, split_first, split_parts, split.partials, rotate);                                 \
                break;                                                                                                          \
            }                                                                                                                   \
        }                                                                                                                       \
        hipLaunchKernelGGL((tile_dma16_kernel<C, BF, AKC, BKC>), grid, block, 0, stream, a, tiles_m, tiles_n, group_m, c_vec_ok, \
                           split_first, split_parts, split.partials, rotate);                                                   \
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

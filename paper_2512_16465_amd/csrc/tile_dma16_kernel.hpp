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
//   k-contiguous operand: one ds_read_b128 of chunk (row, l/16) of the swizzled slab.
//   m/n-contiguous operand ([k][row] slab): two ds_read_b64_tr_b16; lane j of a 16-lane group
//   supplies k-row 8*(l/16) + j/4 (+4 for the second read), columns 4*(j%4)...
#pragma once
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

// ---- fragment readers for 16-row tiles; the slabs are those written by DmaKC / DmaMC ----

template <int ROWS, int BK>
struct Frag16KC {
    static constexpr int CPR = BK / 8;
    static_assert(BK == 32 || BK == 64, "one or two 32-wide k blocks per slab");
    static __device__ __forceinline__ uint32_t base(int row0, int lane) { return swz<CPR>(row0 + (lane & 15), lane >> 4); }
    typedef u32x4 Raw;
    static constexpr bool MANUAL_WAIT = false;
    // k block ks of the slab: chunk index + 4 flips bit 2 of the swizzled position
    static __device__ __forceinline__ void read(const char* slab, uint32_t b, int ks, Raw& r) {
        r = *(const u32x4*)(slab + (b ^ (uint32_t)(ks << 6)));
    }
    static __device__ __forceinline__ u32x4 finish(const Raw& r) { return r; }
};

template <int ROWS, int BK>
struct Frag16MC {
    static constexpr int CPK = ROWS / 8;
    static_assert(BK == 32 || BK == 64, "one or two 32-wide k blocks per slab");
    static __device__ __forceinline__ uint32_t base(int row0, int lane) {
        const uint32_t j = lane & 15, g = lane >> 4;
        const uint32_t k = 8 * g + (j >> 2);
        const uint32_t col = row0 + 4 * (j & 3);
        const uint32_t cs = (col >> 3) ^ mc_swizzle(k);
        return (k * CPK + cs) * 16 + (col & 7) * 2;
    }
    struct Raw { uint2 lo, hi; };
    static constexpr bool MANUAL_WAIT = true;
    static constexpr int KS_BYTES = 32 * CPK * 16, HALF_BYTES = 4 * CPK * 16;   // 32 and 4 k-rows further
    static_assert(KS_BYTES + HALF_BYTES < 65536, "offsets must fit the instruction's immediate");
    static __device__ __forceinline__ void read(const char* slab, uint32_t b, int ks, Raw& r) {
        const uint32_t addr = (uint32_t)(uintptr_t)GEMM_LDS_PTR(slab) + b;
        if (ks == 0) {
            asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.lo) : "v"(addr));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(HALF_BYTES));
        } else {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.lo) : "v"(addr), "n"(KS_BYTES));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(KS_BYTES + HALF_BYTES));
        }
    }
    static __device__ __forceinline__ u32x4 finish(const Raw& r) { return u32x4{r.lo.x, r.lo.y, r.hi.x, r.hi.y}; }
};

template <class Raw>
__device__ __forceinline__ void wait_raw8(Raw (&r)[8]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi), "+v"(r[2].lo), "+v"(r[2].hi), "+v"(r[3].lo), "+v"(r[3].hi),
                   "+v"(r[4].lo), "+v"(r[4].hi), "+v"(r[5].lo), "+v"(r[5].hi), "+v"(r[6].lo), "+v"(r[6].hi), "+v"(r[7].lo), "+v"(r[7].hi));
}
__device__ __forceinline__ void wait_raw8(u32x4 (&)[8]) {}

// Pipeline (BK = 32, one 64-MFMA sub-step per slab).  During step kt a wave multiplies the
// fragments of slab kt, which it read from LDS during step kt-1, so LDS holds slabs kt+1 (being
// read) .. kt+NS-1 or kt+NS, and the stage of slab kt is free as soon as every wave has passed
// the barrier of step kt.  That barrier sits four MFMAs into the step; behind it the step reads
// the 16 fragments of slab kt+1 (one per two MFMAs, in the order the MFMAs will want them) and
// requests new slabs (in the MFMA slots between the reads):
//   ring of 4: slab kt+4 into the stage of slab kt;
//   ring of 5, "paired": a k-contiguous operand contributes 64 bytes per row and slab, half a
//     cache line, and the L2 serves a half-line request at the cost of a full one (16 TB/s
//     of half lines against 27 TB/s of full lines measured for this tile stream), so slabs are
//     requested in pairs (2j, 2j+1) with the two loads that fetch the two halves of the same rows
//     back to back, which the L1 merges into one line request (24 TB/s).  Even step kt: first
//     half of the rows of pair (kt+4, kt+5); odd step kt: second half of pair (kt+3, kt+4).  An
//     n-contiguous operand already fetches whole lines; its even slab goes in the even step.
// Loads complete in order, so the barrier's wait counts the younger ones that may stay in
// flight: two slabs in the ring of 4; in the ring of 5 the next pair (even step) or its first
// half (odd step).
template <class C, bool IS_BF16, bool A_KC, bool B_KC>
__global__ __launch_bounds__(C::NT) void tile_dma16_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok) {
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::NT, NS = C::NS;
    constexpr int TM = C::WTM / 16, TN = C::WTN / 16;        // 16x16 accumulators per wave
    static_assert(TM == 8 && TN == 8, "the slot plan below is written for a 128x128 wave sub-block");
    static_assert(BK == 32, "one 32-wide k block per slab");
    static_assert(NS == 4 || NS == 5, "ring of 4, or ring of 5 with paired requests");
    constexpr bool PAIRED = NS == 5;
    using EL = EpiLayout<C>;
    constexpr int RING = NS * C::STAGE;
    constexpr int LDS_BYTES = RING > EL::BYTES ? RING : EL::BYTES;
    __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % C::WM, wn = wave / C::WM;

    int tm, tn;
    tile_of_workgroup(blockIdx.x, tiles_m, tiles_n, group_m, tm, tn);
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;
    const int K = (int)a.K;

    using LA = typename std::conditional<A_KC, DmaKC<BM, BK, NT>, DmaMC<BM, BK, NT>>::type;
    using LB = typename std::conditional<B_KC, DmaKC<BN, BK, NT>, DmaMC<BN, BK, NT>>::type;
    using FA = typename std::conditional<A_KC, Frag16KC<BM, BK>, Frag16MC<BM, BK>>::type;
    using FB = typename std::conditional<B_KC, Frag16KC<BN, BK>, Frag16MC<BN, BK>>::type;
    static_assert(LA::L % 2 == 0 && LB::L % 2 == 0, "a slab is requested in two halves");
    LA la;
    LB lb;
    la.init(tid, a.lda);
    lb.init(tid, a.ldb);
    const char* pa = LA::tile_base(a.A, m0, a.lda);
    const char* pb = LB::tile_base(a.B, n0, a.ldb);
    const int64_t a_step = LA::k_step_bytes(a.lda), b_step = LB::k_step_bytes(a.ldb);
    const int64_t a_bytes = LA::total_bytes(a.M, a.K, a.lda) - (pa - (const char*)a.A);
    const int64_t b_bytes = LB::total_bytes(a.N, a.K, a.ldb) - (pb - (const char*)a.B);

    uint32_t fa[TM], fb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = FA::base(wm * C::WTM + i * 16, lane);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = C::A_BYTES + FB::base(wn * C::WTN + j * 16, lane);

    f32x4 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    const int k_tiles = (K + BK - 1) / BK;
    const int full_tiles = K / BK;
    constexpr int NM = TM * TN, NR = TM + TN;     // MFMAs and fragments per step
    constexpr int LPT = LA::L + LB::L;            // loads per thread and slab (= per half of a pair)

    typename FA::Raw af[2][TM];                   // fragments of two consecutive slabs
    typename FB::Raw bf[2][TN];

    // Fragment q of a slab in the order the MFMAs first need them: A0, B0..B7, A1..A7.
    auto read_one = [&](int buf, int stage, int q) {
        const char* st = lds + stage * C::STAGE;
        if (q == 0) FA::read(st, fa[0], 0, af[buf][0]);
        else if (q <= TN) FB::read(st, fb[q - 1], 0, bf[buf][q - 1]);
        else FA::read(st, fa[q - TN], 0, af[buf][q - TN]);
    };
    auto run_mfmas = [&](int cur, auto slot) {
        if (FA::MANUAL_WAIT) wait_raw8(af[cur]);
        if (FB::MANUAL_WAIT) wait_raw8(bf[cur]);
        u32x4 ua[TM], ub[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) ua[i] = FA::finish(af[cur][i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) ub[j] = FB::finish(bf[cur][j]);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            slot(m, 0);
            const int i = m / TN, j = (i & 1) ? TN - 1 - m % TN : m % TN;     // boustrophedon: consecutive MFMAs share an operand
            mfma16<IS_BF16>(acc[i][j], ua[i], ub[j]);
            slot(m, 1);
        }
    };

    // ---- what a step requests ----
    // Load q (0 .. LPT-1) of a step: operand, slab, instruction of that slab.  `even` is the
    // parity of the step.  Ring of 4: all of slab kt+4.  Ring of 5: see above; a k-contiguous
    // operand alternates the two slabs of the pair, an n-contiguous one takes one slab per step.
    struct Pick { bool is_a; int slab_off, i; };
    auto pick = [](bool even, int q) -> Pick {
        const bool is_a = q < LA::L;
        const int r = is_a ? q : q - LA::L;
        const int L = is_a ? LA::L : LB::L;
        const bool transposed = is_a ? LA::TRANSPOSED : LB::TRANSPOSED;
        if (!PAIRED) return Pick{is_a, NS, r};
        const int first = even ? 4 : 3;                       // offset of the pair's even slab from kt
        if (transposed) return Pick{is_a, first + (even ? 0 : 1), r};
        return Pick{is_a, first + (r & 1), (even ? 0 : L / 2) + (r >> 1)};
    };
    const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa, a_bytes), rb0 = make_rsrc(pb, b_bytes);
    // steady state: the slab exists and lies wholly inside K; the k advance is the loads' scalar
    // offset, which the range check ignores (see load_to_lds_b128)
    // position in the ring of slab kt + d, given that of slab kt (d <= NS): no division in the loop
    auto ring_at = [](int ring, int d) { return ring + d >= NS ? ring + d - NS : ring + d; };
    auto issue_hot = [&](int kt, int ring, bool even, int q) {
        const Pick p = pick(even, q);
        const int t = kt + p.slab_off;
        char* stage = lds + ring_at(ring, p.slab_off) * C::STAGE;
        if (p.is_a) la.issue(false, p.i, ra0, stage, wave, tid, 0, K, (uint32_t)(t * a_step));
        else lb.issue(false, p.i, rb0, stage + C::A_BYTES, wave, tid, 0, K, (uint32_t)(t * b_step));
    };
    // first and last steps: a descriptor per slab (its range check cuts off k-rows past K), a
    // mask for the chunks of a partial slab, nothing for slabs past the end
    auto issue_checked = [&](int kt, bool even, int q) {
        const Pick p = pick(even, q);
        const int t = kt + p.slab_off;
        if (t >= k_tiles) return;
        char* stage = lds + (t % NS) * C::STAGE;
        if (p.is_a) {
            const __amdgpu_buffer_rsrc_t r = make_rsrc(pa + t * a_step, a_bytes - t * a_step);
            if (t < full_tiles) la.issue(false, p.i, r, stage, wave, tid, t * BK, K);
            else la.issue(true, p.i, r, stage, wave, tid, t * BK, K);
        } else {
            const __amdgpu_buffer_rsrc_t r = make_rsrc(pb + t * b_step, b_bytes - t * b_step);
            if (t < full_tiles) lb.issue(false, p.i, r, stage + C::A_BYTES, wave, tid, t * BK, K);
            else lb.issue(true, p.i, r, stage + C::A_BYTES, wave, tid, t * BK, K);
        }
    };

#define GEMM_WAIT_VM_BARRIER(N) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory")

    // Slot plan of a step (slot m follows MFMA m): barrier before MFMA BAR_SLOT; fragment q of the
    // next slab after MFMA BAR_SLOT + 2q; loads after the odd MFMAs in between, singly every
    // fourth slot or, paired, two every eighth.
    constexpr int BAR_SLOT = 4;
    constexpr int LOAD_FIRST = BAR_SLOT + 1, LOAD_EVERY = PAIRED ? 8 : 4, LOAD_GROUP = PAIRED ? 2 : 1;
    static_assert(BAR_SLOT + 2 * NR <= NM - 8, "the last fragment is read at least 8 MFMAs before the next step");
    static_assert(LOAD_FIRST + (LPT / LOAD_GROUP - 1) * LOAD_EVERY < NM, "all loads of a step fit in the step");
    // loads that may still be in flight when slab kt+1 must have landed
    constexpr int PENDING_EVEN = PAIRED ? 2 * LPT : (NS - 2) * LPT, PENDING_ODD = PAIRED ? LPT : (NS - 2) * LPT;

    auto step_hot = [&](int kt, int ring, auto parity) {
        constexpr bool EVEN = decltype(parity)::value == 0;
        constexpr int cur = EVEN ? 0 : 1, nxt = cur ^ 1;
        const int next = ring_at(ring, 1);
        run_mfmas(cur, [&](int m, int after) {
            if (!after) {
                if (m == BAR_SLOT) GEMM_WAIT_VM_BARRIER(EVEN ? PENDING_EVEN : PENDING_ODD);
                return;
            }
            if (m >= BAR_SLOT && (m - BAR_SLOT) % 2 == 0 && (m - BAR_SLOT) / 2 < NR) read_one(nxt, next, (m - BAR_SLOT) / 2);
            if (m >= LOAD_FIRST && (m - LOAD_FIRST) % LOAD_EVERY == 0 && (m - LOAD_FIRST) / LOAD_EVERY < LPT / LOAD_GROUP) {
#pragma unroll
                for (int u = 0; u < LOAD_GROUP; ++u) issue_hot(kt, ring, EVEN, (m - LOAD_FIRST) / LOAD_EVERY * LOAD_GROUP + u);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    auto step_edge = [&](int kt, auto parity) {
        constexpr bool EVEN = decltype(parity)::value == 0;
        constexpr int cur = EVEN ? 0 : 1, nxt = cur ^ 1;
        if (kt + 1 < k_tiles) {
            GEMM_WAIT_VM_BARRIER(0);
#pragma unroll
            for (int q = 0; q < LPT; ++q) issue_checked(kt, EVEN, q);
#pragma unroll
            for (int q = 0; q < NR; ++q) read_one(nxt, (kt + 1) % NS, q);
        }
        run_mfmas(cur, [](int, int) {});
    };
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;

    if (k_tiles > 0) {
        // slabs 0 .. 3: what the steps "before the first" would have requested
#pragma unroll
        for (int kt = -4; kt < 0; ++kt) {
            if (!PAIRED) {
#pragma unroll
                for (int q = 0; q < LPT; ++q) issue_checked(kt, true, q);
            } else if ((kt & 1) == 0) {
#pragma unroll
                for (int q = 0; q < LPT; ++q) issue_checked(kt, true, q);
            } else {
#pragma unroll
                for (int q = 0; q < LPT; ++q) issue_checked(kt, false, q);
            }
        }
        GEMM_WAIT_VM_BARRIER(0);
#pragma unroll
        for (int q = 0; q < NR; ++q) read_one(0, 0, q);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0, ring = 0;                            // ring = kt % NS
        for (; kt + 1 + NS < full_tiles; kt += 2) {      // the two steps request slabs up to kt + 5
            step_hot(kt, ring, Even{});
            step_hot(kt + 1, ring_at(ring, 1), Odd{});
            ring = ring_at(ring, 2);
        }
        for (; kt < k_tiles; kt += 2) {
            step_edge(kt, Even{});
            if (kt + 1 < k_tiles) step_edge(kt + 1, Odd{});
        }
    }
    // LDS is reused by the epilogue; the wait states let the last MFMAs retire before their results are read
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier\n\ts_nop 15\n\ts_nop 15" ::: "memory");
#undef GEMM_WAIT_VM_BARRIER

    // accumulator register v of lane l: row 4*(l/16) + v, column l%16 of its 16x16 tile
    const int c16 = lane & 15, g4 = lane >> 4;
    tile_epilogue_bands<C>(
        [&](auto band, char* region) {
            constexpr int b = decltype(band)::value;
#pragma unroll
            for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        *(float*)(region + ((16 * i2 + 4 * g4 + v) * EL::RS + j * 16 + c16) * 4) = acc[2 * b + i2][j][v];
        },
        lds, a, m0, n0, c_vec_ok);
}

template <class C>
hipError_t launch_dma16_variant(const Args& a, int group_m, hipStream_t stream) {
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(C::NT);
    const bool bf = a.dtype == DT_BF16;
    const bool akc = !a.transA, bkc = a.transB != 0;
    const int c_vec_ok = (a.ldc % 4 == 0) && ((uintptr_t)a.C % (a.out_dtype == DT_F32 ? 16 : 8) == 0);
#define GEMM_TILE_LAUNCH(BF, AKC, BKC) \
    hipLaunchKernelGGL((tile_dma16_kernel<C, BF, AKC, BKC>), grid, block, 0, stream, a, tiles_m, tiles_n, group_m, c_vec_ok)
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

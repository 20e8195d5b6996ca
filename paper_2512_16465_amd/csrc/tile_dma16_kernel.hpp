// Direct-to-LDS macro-tile kernel built on the 16x16x32 MFMA (bf16 / fp16, gfx950).
//
// Same operand movers, LDS layouts, ring of stages and slot-wise schedule as tile_dma_kernel.hpp;
// what changes is the matrix instruction.  v_mfma_f32_16x16x32 does the same work per cycle as
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

template <class C, bool IS_BF16, bool A_KC, bool B_KC>
__global__ __launch_bounds__(C::NT) void tile_dma16_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok) {
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::NT, NS = C::NS;
    constexpr int TM = C::WTM / 16, TN = C::WTN / 16;        // 16x16 accumulators per wave
    static_assert(TM == 8 && TN == 8, "the fragment waits below are written for a 128x128 wave sub-block");
    static_assert(NS >= 3, "the barrier's load count assumes at least two slabs of lookahead");
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
    constexpr int NKS = BK / 32;                  // k blocks (sub-steps) per slab
    constexpr int NM = TM * TN, NR = TM + TN;     // MFMAs and fragments per sub-step
    constexpr int LPT = LA::L + LB::L;
    constexpr int D = NS - 1;

    typename FA::Raw af[2][TM];                   // fragments of two consecutive sub-steps
    typename FB::Raw bf[2][TN];

    // Fragment q of a sub-step in the order the MFMAs first need them: A0, B0..B7, A1..A7.
    auto read_one = [&](int buf, int stage, int ks, int q) {
        const char* st = lds + stage * C::STAGE;
        if (q == 0) FA::read(st, fa[0], ks, af[buf][0]);
        else if (q <= TN) FB::read(st, fb[q - 1], ks, bf[buf][q - 1]);
        else FA::read(st, fa[q - TN], ks, af[buf][q - TN]);
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
    auto issue_one = [&](int q, __amdgpu_buffer_rsrc_t ra, __amdgpu_buffer_rsrc_t rb, char* stage, int k0, auto masked,
                         uint32_t soff_a = 0, uint32_t soff_b = 0) {
        constexpr bool M = decltype(masked)::value;
        if (q < LA::L) la.issue(M, q, ra, stage, wave, tid, k0, K, soff_a);
        else lb.issue(M, q - LA::L, rb, stage + C::A_BYTES, wave, tid, k0, K, soff_b);
    };
    auto issue_tile = [&](int t, auto masked) {
        const __amdgpu_buffer_rsrc_t ra = make_rsrc(pa + t * a_step, a_bytes - t * a_step);
        const __amdgpu_buffer_rsrc_t rb = make_rsrc(pb + t * b_step, b_bytes - t * b_step);
        char* stage = lds + (t % NS) * C::STAGE;
#pragma unroll
        for (int q = 0; q < LPT; ++q) issue_one(q, ra, rb, stage, t * BK, masked);
    };

#define GEMM_WAIT_VM_BARRIER(N) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory")

    // Slots of a k step: NKS * NM MFMAs.  The barrier of the step sits BAR_SLOT MFMAs into the last
    // sub-step; behind it the first fragments of the next slab are read, one per READ_EVERY slots.
    // The loads of slab kt+D go out one per LOAD_EVERY slots from the top of the step.
    constexpr int SLOTS = NKS * NM;
    constexpr int BAR_SLOT = 4;
    constexpr int BAR_POS = (NKS - 1) * NM + BAR_SLOT;
    constexpr int READ_EVERY = 2;                               // 16 fragments in 32 slots
    constexpr int LOAD_EVERY = SLOTS / LPT >= 4 ? 4 : SLOTS / LPT;
    constexpr int LOADS_BEFORE_BAR = (BAR_POS + LOAD_EVERY - 1) / LOAD_EVERY < LPT ? (BAR_POS + LOAD_EVERY - 1) / LOAD_EVERY : LPT;
    static_assert(BAR_SLOT + READ_EVERY * NR <= NM - 8, "the last fragment is read at least 8 MFMAs before the next sub-step");
    static_assert(LOAD_EVERY * LPT <= SLOTS, "all loads of a slab fit in the step");

    // Steady state: slabs kt+1 .. kt+D exist and need no mask; the k advance travels as the loads'
    // scalar offset (see tile_dma_kernel.hpp).  `base` is the parity of the step's first sub-step.
    const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa, a_bytes), rb0 = make_rsrc(pb, b_bytes);
    auto step_hot = [&](int kt, auto base_parity) {
        constexpr int P0 = decltype(base_parity)::value;
        const int stage = kt % NS, next = (kt + 1) % NS;
        const int t = kt + D;
        const uint32_t soff_a = (uint32_t)(t * a_step), soff_b = (uint32_t)(t * b_step);
        char* dst = lds + (t % NS) * C::STAGE;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = (P0 + ks) & 1, nxt = cur ^ 1;
            const bool last = ks == NKS - 1;
            run_mfmas(cur, [&](int m, int after) {
                const int slot = ks * NM + m;
                if (!after) {
                    // loads issued so far in this step: slots 0, LOAD_EVERY, ... below BAR_POS
                    if (last && m == BAR_SLOT) GEMM_WAIT_VM_BARRIER((D - 2) * LPT + LOADS_BEFORE_BAR);
                    return;
                }
                if (!last) {
                    if (m % READ_EVERY == 0 && m / READ_EVERY < NR) read_one(nxt, stage, ks + 1, m / READ_EVERY);
                } else if (m >= BAR_SLOT) {
                    const int mm = m - BAR_SLOT;
                    if (mm % READ_EVERY == 0 && mm / READ_EVERY < NR) read_one(nxt, next, 0, mm / READ_EVERY);
                }
                if (slot % LOAD_EVERY == 0 && slot / LOAD_EVERY < LPT)
                    issue_one(slot / LOAD_EVERY, ra0, rb0, dst, t * BK, std::false_type{}, soff_a, soff_b);
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };
    // the first and last steps: flags instead of assumptions, everything outstanding is awaited
    auto step_edge = [&](int kt, auto base_parity) {
        constexpr int P0 = decltype(base_parity)::value;
        const int stage = kt % NS, next = (kt + 1) % NS;
        const int t = kt + D;
        if (t < full_tiles) issue_tile(t, std::false_type{});
        else if (t < k_tiles) issue_tile(t, std::true_type{});
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = (P0 + ks) & 1, nxt = cur ^ 1;
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
    // With one sub-step per slab the fragment buffers alternate from step to step, so steps are
    // taken two at a time to keep the register names static.
    constexpr int STRIDE = (NKS & 1) ? 2 : 1;
    using Par0 = std::integral_constant<int, 0>;
    using Par1 = std::integral_constant<int, NKS & 1>;

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
        for (; kt + STRIDE - 1 + D < full_tiles; kt += STRIDE) {
            step_hot(kt, Par0{});
            if constexpr (STRIDE == 2) step_hot(kt + 1, Par1{});
        }
        for (; kt < k_tiles; kt += STRIDE) {
            step_edge(kt, Par0{});
            if constexpr (STRIDE == 2) {
                if (kt + 1 < k_tiles) step_edge(kt + 1, Par1{});
            }
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

// Direct-to-LDS macro-tile kernel whose operand loads ask the L2 for whole 128-byte lines.
//
// With BK = 32 a k-contiguous operand contributes 64 bytes per row and k step, half a cache line;
// the L2 serves a half-line request at the cost of a full one, and a 256x256 tile at full MFMA
// rate then needs more requests than the eight L2s deliver (measured on this part: 16 TB/s of
// half-line requests against 27 TB/s of full-line ones for the same tile stream).  This kernel
// keeps the 32-wide LDS stages and the slot-wise schedule of tile_dma_kernel.hpp but requests
// slabs in pairs (2j, 2j+1): the two loads that fetch the two halves of the same rows are
// issued back to back, and the L1 merges them into one line request (24 TB/s measured).
//
// Ring of 5 stages.  While slab kt is multiplied, slabs kt+1 .. kt+4 are resident or in flight:
//   odd  step kt: first half of the rows of pair (kt+3, kt+4) is requested,
//   even step kt: second half of the rows of pair (kt+2, kt+3).
// The stages those loads overwrite held slabs kt-2 and kt-1 (odd step), whose last readers passed
// the barrier of step kt-1.  The barrier of an odd step kt waits until pair (kt+1, kt+2) has
// landed (all its loads precede this step's in program order, and loads complete in order); the
// barrier of an even step only orders the readers of slab kt before the next overwrite.
// An n-contiguous operand already fetches whole lines; its two slabs simply go out one per step.
#pragma once
#include "tile_dma_kernel.hpp"

namespace gemm {
namespace tile {

template <class C, bool IS_BF16, bool A_KC, bool B_KC, bool PLAIN>
__global__ __launch_bounds__(C::NT) void tile_dma_pair_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok) {
    constexpr int BM = C::BM, BN = C::BN, BK = C::BK, NT = C::NT, TM = C::TM, TN = C::TN, NS = C::NS;
    static_assert(NS == 5, "the pairing schedule is written for a ring of five stages");
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
    static_assert(LA::L % 2 == 0 && LB::L % 2 == 0, "a slab is requested in two halves");
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
    constexpr int NKS = BK / 16;
    constexpr int NM = TM * TN, NR = TM + TN;
    constexpr int HL = LA::L + LB::L;             // loads per thread in one half of a pair
    constexpr int G = HL / 2;                     // issued two at a time

    typename LA::Raw af[2][TM];
    typename LB::Raw bf[2][TN];

    auto read_one = [&](int buf, int stage, int ks, int q) {
        const char* st = lds + stage * C::STAGE;
        if (q < TM) LA::read_frag(st, fa[q], ks, af[buf][q]);
        else LB::read_frag(st, fb[q - TM], ks, bf[buf][q - TM]);
    };
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
            const int i = m / TN, j = (i & 1) ? TN - 1 - m % TN : m % TN;
            acc[i][j] = mfma32<IS_BF16>(ua[i], ub[j], acc[i][j]);
            slot(m, 1);
        }
    };

    // Load q of half h of a pair: which operand, which slab of the pair (0 = even), which
    // instruction of that slab.  A k-contiguous operand alternates the two slabs so that both
    // halves of a line are requested back to back; an n-contiguous one sends the even slab in
    // the first half and the odd slab in the second.
    struct Pick { bool is_a; int parity, i; };
    auto pick = [](int h, int q) -> Pick {
        if (q < LA::L) {
            if (!LA::TRANSPOSED) return Pick{true, q & 1, h * (LA::L / 2) + (q >> 1)};
            return Pick{true, h, q};
        }
        const int r = q - LA::L;
        if (!LB::TRANSPOSED) return Pick{false, r & 1, h * (LB::L / 2) + (r >> 1)};
        return Pick{false, h, r};
    };
    // Where the two slabs of a pair come from and go to.  `exact` descriptors start at each slab
    // (the range check then also cuts off k-rows past K: first and last steps); otherwise both
    // slabs share the tile's descriptor and the k advance is the loads' scalar offset, which the
    // range check ignores - safe in the steady state, where each slab lies wholly inside K and
    // every lane whose own offset is in range addresses a row of the operand.
    struct PairRsrc { __amdgpu_buffer_rsrc_t a[2], b[2]; char* stage[2]; int k0[2]; uint32_t soff_a[2], soff_b[2]; };
    const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa, a_bytes), rb0 = make_rsrc(pb, b_bytes);
    auto pair_rsrc = [&](int j, auto exact) {
        PairRsrc r;
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int t = 2 * j + p;
            if (decltype(exact)::value) {
                r.a[p] = make_rsrc(pa + t * a_step, a_bytes - t * a_step);
                r.b[p] = make_rsrc(pb + t * b_step, b_bytes - t * b_step);
                r.soff_a[p] = r.soff_b[p] = 0;
            } else {
                r.a[p] = ra0;
                r.b[p] = rb0;
                r.soff_a[p] = (uint32_t)(t * a_step);
                r.soff_b[p] = (uint32_t)(t * b_step);
            }
            r.stage[p] = lds + (t % NS) * C::STAGE;
            r.k0[p] = t * BK;
        }
        return r;
    };
    auto issue_q = [&](const PairRsrc& r, int h, int q, auto masked) {
        constexpr bool M = decltype(masked)::value;
        const Pick p = pick(h, q);
        if (p.is_a) la.issue(M, p.i, r.a[p.parity], r.stage[p.parity], wave, tid, r.k0[p.parity], K, r.soff_a[p.parity]);
        else lb.issue(M, p.i, r.b[p.parity], r.stage[p.parity] + C::A_BYTES, wave, tid, r.k0[p.parity], K, r.soff_b[p.parity]);
    };
    // one half of pair j at once, for the first and last steps: slabs past the end are skipped,
    // a partial last slab is masked
    auto issue_half_checked = [&](int j, auto half) {
        constexpr int h = decltype(half)::value;
        if (2 * j >= k_tiles) return;
        const PairRsrc r = pair_rsrc(j, std::true_type{});
#pragma unroll
        for (int q = 0; q < HL; ++q) {
            const int t = 2 * j + pick(h, q).parity;     // parity is known at compile time
            if (t < full_tiles) issue_q(r, h, q, std::false_type{});
            else if (t < k_tiles) issue_q(r, h, q, std::true_type{});
        }
    };
    // what step kt requests: (pair, half)
    auto due_pair = [](int kt) { return (kt & 1) ? (kt + 3) / 2 : kt / 2 + 1; };

#define GEMM_WAIT_VM_BARRIER(N) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory")
#define GEMM_WAIT_LDS_BARRIER() asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

    constexpr int BAR_SLOT = NM / 4;                          // MFMAs of the last k-sub-step issued before the barrier
    constexpr int SLOTS = NKS * NM;                           // MFMAs (and slots) per step
    constexpr int BAR_POS = (NKS - 1) * NM + BAR_SLOT;        // slots that precede the barrier
    constexpr int BEFORE_BAR = 2 * ((BAR_POS * G) / SLOTS);   // loads of the step issued before its barrier

    // steady state: every slab requested exists and needs no mask
    auto step_hot = [&](int kt, auto parity) {
        constexpr int P = decltype(parity)::value;            // kt & 1
        const int stage = kt % NS, next = (kt + 1) % NS;
        const PairRsrc r = pair_rsrc(P ? (kt + 3) / 2 : kt / 2 + 1, std::false_type{});
        constexpr int h = P ? 0 : 1;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            const bool last = ks == NKS - 1;
            run_mfmas(cur, [&](int m, int after) {
                if (!after) {
                    if (last && m == BAR_SLOT) {
                        if (P) GEMM_WAIT_VM_BARRIER(BEFORE_BAR);
                        else GEMM_WAIT_LDS_BARRIER();
                    }
                    return;
                }
                if (!last) {
#pragma unroll
                    for (int q = (m * NR) / NM; q < ((m + 1) * NR) / NM; ++q) read_one(nxt, stage, ks + 1, q);
                } else if (m >= BAR_SLOT) {
                    constexpr int RS = NM - BAR_SLOT - NM / 4 > 0 ? NM - BAR_SLOT - NM / 4 : 1;
                    const int mm = m - BAR_SLOT;
                    if (mm < RS) {
#pragma unroll
                        for (int q = (mm * NR) / RS; q < ((mm + 1) * NR) / RS; ++q) read_one(nxt, next, 0, q);
                    }
                }
                const int slot = ks * NM + m;
#pragma unroll
                for (int g = (slot * G) / SLOTS; g < ((slot + 1) * G) / SLOTS; ++g) {
                    issue_q(r, h, 2 * g, std::false_type{});
                    issue_q(r, h, 2 * g + 1, std::false_type{});
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }
    };
    // the first and last steps: checks instead of assumptions, everything outstanding is awaited
    auto step_edge = [&](int kt) {
        const int stage = kt % NS, next = (kt + 1) % NS;
        if (kt & 1) issue_half_checked(due_pair(kt), std::integral_constant<int, 0>{});
        else issue_half_checked(due_pair(kt), std::integral_constant<int, 1>{});
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
        issue_half_checked(0, std::integral_constant<int, 0>{});
        issue_half_checked(0, std::integral_constant<int, 1>{});
        issue_half_checked(1, std::integral_constant<int, 0>{});
        GEMM_WAIT_VM_BARRIER(0);
#pragma unroll
        for (int q = 0; q < NR; ++q) read_one(0, 0, 0, q);
        __builtin_amdgcn_sched_barrier(0);
        int kt = 0;
        for (; kt + 6 <= full_tiles; kt += 2) {       // the steps request slabs up to kt + 5
            step_hot(kt, std::integral_constant<int, 0>{});
            step_hot(kt + 1, std::integral_constant<int, 1>{});
        }
        for (; kt < k_tiles; ++kt) step_edge(kt);
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS is reused by the epilogue
#undef GEMM_WAIT_VM_BARRIER
#undef GEMM_WAIT_LDS_BARRIER

    if constexpr (PLAIN) tile_epilogue_plain<C>(acc, a, m0, n0);
    else tile_epilogue<C>(acc, lds, a, m0, n0, c_vec_ok);
}

template <class C>
hipError_t launch_dma_pair_variant(const Args& a, int group_m, hipStream_t stream) {
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)a.batch), block(C::NT);
    const bool bf = a.dtype == DT_BF16;
    const bool akc = !a.transA, bkc = a.transB != 0;
    const int c_vec_ok = c_rows_take_vec4(a);
    const bool plain = plain_epilogue_applies<C>(a);
#define GEMM_TILE_LAUNCH(BF, AKC, BKC)                                                                             \
    do {                                                                                                           \
        if (plain)                                                                                                 \
            hipLaunchKernelGGL((tile_dma_pair_kernel<C, BF, AKC, BKC, true>), grid, block, 0, stream, a, tiles_m,  \
                               tiles_n, group_m, c_vec_ok);                                                        \
        else                                                                                                       \
            hipLaunchKernelGGL((tile_dma_pair_kernel<C, BF, AKC, BKC, false>), grid, block, 0, stream, a, tiles_m, \
                               tiles_n, group_m, c_vec_ok);                                                        \
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

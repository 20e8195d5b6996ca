// Persistent 128x128 tile kernel for short k loops (K <= 128, whole 32-wide slabs; bf16 / fp16).
//
// With a k loop of at most four slabs a tile is one trip to memory, half a microsecond of matrix
// arithmetic and a result to write: the per-head score products of attention are the model case (a
// batch of 2048 x 2048 x 128 products is 89 % result bytes).  Nothing in such a tile can be pipelined
// along k, and what the general tile kernels spend around their k loop (launch of a workgroup, ring
// fill, an epilogue staged in fp32 band by band) is here the whole cost.  What bounds this kernel is
// the path between a compute unit and the L2 (every tile fetches its operands from there and writes
// its results through it), so the kernel moves as few bytes over it as it can, in an order that keeps
// the memory channels evenly busy, and lets two workgroups per compute unit take turns:
//
//   a workgroup stays on its compute unit and walks a run of consecutive tiles down a column of tiles
//   of C; per tile it
//     multiplies pair by pair of slabs as they land in its 64 KiB of LDS (16x16x32 MFMA, four waves
//       of 64x64),
//     requests the operands of the next tile (direct-to-LDS loads) as soon as every wave has read this
//       tile's: all of A, and B only where the column ends (the panel of B stays in LDS otherwise),
//     applies alpha, the activation and the one rounding in the accumulator layout, brings 16
//       contiguous bytes of a row of C together in every lane (fp32: as they are; 16-bit: lanes trade
//       halves with v_permlane16_swap), then the two halves of each 128-byte line in one instruction
//       (a rotation within the 16-lane rows), and writes C from the registers: no pass through LDS.
//   The waits for the operands count this wave's operations in flight, loads and the younger stores
//   of the tile before.
//
// All LDS traffic is assembly: the compiler would make every LDS access wait for the direct-to-LDS
// loads in flight.  C is write-only here (beta == 0, no bias); calls with beta != 0, a bias, longer or
// ragged k, or rows of C that take no 16-byte stores go to the other tile kernels.
#pragma once
#include "tile_dma16_kernel.hpp"

namespace gemm {
namespace tile {

struct ShortK {
    static constexpr int BM = 128, BN = 128, BK = 32, NT = 256, WTM = 64, WTN = 64, TM = 4, TN = 4;
    static constexpr int SLAB = (BM + BN) * BK * 2;      // bytes of one 32-wide slab of both operands
    static constexpr int A_BYTES = BM * BK * 2;
    static constexpr int LDS_BYTES = 64 * 1024;          // two workgroups per compute unit
    static constexpr int MAX_SLABS = 4;
    // bytes of LDS a call needs: the operands of a tile
    static constexpr int lds_need(int slabs) { return slabs * SLAB; }
};

// Registers of a fragment between its LDS read and the wait for it.  The value of a k-contiguous
// operand is the one 16-byte register group that the read defines, and it stays whole until the wait
// has named it: a value taken apart before the wait (two halves, say) may be put together again by
// register copies that the compiler is free to place ahead of the wait, where they would copy what
// the registers held before.
struct ShortkRawKC { u32x4 q; };
struct ShortkRawMC { u32x2 lo, hi; };
template <int TILE, class F>
__device__ __forceinline__ void shortk_read(uint32_t addr, ShortkRawKC& r) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r.q) : "v"(addr), "n"(TILE * 1024));
}
template <int TILE, class F>
__device__ __forceinline__ void shortk_read(uint32_t addr, ShortkRawMC& r) {
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r.lo) : "v"(addr));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(addr), "n"(F::HALF_BYTES));
}
__device__ __forceinline__ void shortk_wait(ShortkRawKC (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(r[0].q), "+v"(r[1].q), "+v"(r[2].q), "+v"(r[3].q));
}
__device__ __forceinline__ void shortk_wait(ShortkRawMC (&r)[4]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(r[0].lo), "+v"(r[0].hi), "+v"(r[1].lo), "+v"(r[1].hi), "+v"(r[2].lo), "+v"(r[2].hi), "+v"(r[3].lo), "+v"(r[3].hi));
}
__device__ __forceinline__ u32x4 shortk_value(const ShortkRawKC& r) { return r.q; }
__device__ __forceinline__ u32x4 shortk_value(const ShortkRawMC& r) { return u32x4{r.lo.x, r.lo.y, r.hi.x, r.hi.y}; }

template <bool IS_BF16, bool A_KC, bool B_KC, int OUT>
__global__ __launch_bounds__(ShortK::NT, 2) void tile_shortk_kernel(Args a, int tiles_m, int tiles_n, int total_tiles, int slabs) {
    using S = ShortK;
    constexpr int OB = OUT == DT_F32 ? 4 : 2;                 // bytes per result element
    __shared__ __attribute__((aligned(1024))) char lds[S::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const uint32_t lds0 = (uint32_t)(uintptr_t)GEMM_LDS_PTR(lds);

    using LA = typename std::conditional<A_KC, DmaKC<S::BM, S::BK, S::NT, false>, DmaMC<S::BM, S::BK, S::NT>>::type;
    using LB = typename std::conditional<B_KC, DmaKC<S::BN, S::BK, S::NT, false>, DmaMC<S::BN, S::BK, S::NT>>::type;
    using FA = typename std::conditional<A_KC, Frag16KC<S::BM, S::BK>, Frag16MC<S::BM, S::BK>>::type;
    using FB = typename std::conditional<B_KC, Frag16KC<S::BN, S::BK>, Frag16MC<S::BN, S::BK>>::type;
    using RawA = typename std::conditional<A_KC, ShortkRawKC, ShortkRawMC>::type;
    using RawB = typename std::conditional<B_KC, ShortkRawKC, ShortkRawMC>::type;

    const int per_matrix = tiles_m * tiles_n;
    const int64_t in_b = 2, out_b = OB;
    struct Tile { int64_t m0, n0; const char* A; const char* B; char* C; };
    auto tile_of = [&](int t) __attribute__((always_inline)) {
        const int b = t / per_matrix, r = t - b * per_matrix;
        const int tn = r / tiles_m, tm = r - tn * tiles_m;          // consecutive tiles share a panel of B
        Tile x;
        x.m0 = (int64_t)tm * S::BM; x.n0 = (int64_t)tn * S::BN;
        x.A = (const char*)a.A + (int64_t)b * a.strideA * in_b;
        x.B = (const char*)a.B + (int64_t)b * a.strideB * in_b;
        x.C = (char*)a.C + (int64_t)b * a.strideC * out_b;
        return x;
    };
    // The movers' lane offsets depend on the tile only through the clamp of an edge tile of a row-contiguous
    // operand: kept for whole tiles, recomputed for the others.
    LA la_full;
    LB lb_full;
    la_full.init(tid, a.lda, S::BM);
    lb_full.init(tid, a.ldb, S::BN);
    const int64_t a_step = LA::k_step_bytes(a.lda), b_step = LB::k_step_bytes(a.ldb);
    auto slab_offset = [](int s) { return (uint32_t)(s * S::SLAB); };
    // Pair PAIR (slabs 2*PAIR, 2*PAIR+1, as far as the tile has them) of tile `x` into LDS: a descriptor per
    // slab, exact range checks.  Every thread issues the same number of loads per slab (LA::L for A, and LB::L for B where B is requested), whatever the tile.
    // Slabs go out in pairs: a k-contiguous operand contributes 64 bytes per row and slab, half a cache
    // line, and the two loads that fetch the two halves of the same rows, issued next to each other, are
    // merged into one line request on the way (the L2 serves a half-line request at the cost of a full one).
    auto request_pair = [&]<int SLABS, int PAIR>(const Tile& x, bool with_b) __attribute__((always_inline)) {
        constexpr int s = 2 * PAIR;
        if constexpr (s < SLABS) {
            constexpr bool TWO = s + 1 < SLABS;
            LA la = la_full;
            LB lb = lb_full;
            if (LA::TRANSPOSED && a.M - x.m0 < S::BM) la.init(tid, a.lda, (int)(a.M - x.m0));
            if (LB::TRANSPOSED && a.N - x.n0 < S::BN) lb.init(tid, a.ldb, (int)(a.N - x.n0));
            const char* pa = LA::tile_base(x.A, x.m0, a.lda);
            const char* pb = LB::tile_base(x.B, x.n0, a.ldb);
            const int64_t a_bytes = LA::total_bytes(a.M, a.K, a.lda) - (pa - x.A);
            const int64_t b_bytes = LB::total_bytes(a.N, a.K, a.ldb) - (pb - x.B);
            const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa + s * a_step, a_bytes - s * a_step);
            const __amdgpu_buffer_rsrc_t rb0 = make_rsrc(pb + s * b_step, b_bytes - s * b_step);
            const __amdgpu_buffer_rsrc_t ra1 = TWO ? make_rsrc(pa + (s + 1) * a_step, a_bytes - (s + 1) * a_step) : ra0;
            const __amdgpu_buffer_rsrc_t rb1 = TWO ? make_rsrc(pb + (s + 1) * b_step, b_bytes - (s + 1) * b_step) : rb0;
            char* dst0 = lds + slab_offset(s);
            char* dst1 = lds + slab_offset(s + 1);
#pragma unroll
            for (int i = 0; i < LA::L; ++i) {
                la.issue(false, i, ra0, dst0, wave, tid, s * S::BK, (int)a.K);
                if (TWO) la.issue(false, i, ra1, dst1, wave, tid, (s + 1) * S::BK, (int)a.K);
            }
            if (with_b) {
#pragma unroll
                for (int i = 0; i < LB::L; ++i) {
                    lb.issue(false, i, rb0, dst0 + S::A_BYTES, wave, tid, s * S::BK, (int)a.K);
                    if (TWO) lb.issue(false, i, rb1, dst1 + S::A_BYTES, wave, tid, (s + 1) * S::BK, (int)a.K);
                }
            }
        }
    };

    // fragment addresses of this lane in slab 0 of stage 0
    uint32_t fa[S::TM], fb[S::TN];
#pragma unroll
    for (int i = 0; i < S::TM; ++i) fa[i] = lds0 + FA::base(wm * S::WTM + (FA::PER_TILE_ADDRESS ? i * 16 : 0), lane);
#pragma unroll
    for (int j = 0; j < S::TN; ++j) fb[j] = lds0 + S::A_BYTES + FB::base(wn * S::WTN + (FB::PER_TILE_ADDRESS ? j * 16 : 0), lane);
    auto read_slab = [&](RawA (&af)[S::TM], RawB (&bf)[S::TN], uint32_t off) __attribute__((always_inline)) {
        [&]<int... T>(std::integer_sequence<int, T...>) __attribute__((always_inline)) {
            (shortk_read<T, FA>(fa[FA::PER_TILE_ADDRESS ? T : 0] + off, af[T]), ...);
            (shortk_read<T, FB>(fb[FB::PER_TILE_ADDRESS ? T : 0] + off, bf[T]), ...);
        }
        (std::make_integer_sequence<int, 4>{});
    };

    // What a wave has in flight when it starts on a tile, oldest first: the loads of the first pair of slabs,
    // the loads of the second pair, the stores of the tile before (see the tile loop).  Loads and stores of a
    // wave retire in the order of issue as far as the counter shows (the compiler's own waits rely on the same:
    // it waits for a load with vmcnt(1) while a younger store is in flight), so once at most Y operations are
    // outstanding everything but the Y youngest is done.  landed<Y>() waits for that, then meets the other waves.
    constexpr int NST = OB == 2 ? S::TM * S::TN / 2 : S::TM * S::TN;      // stores per wave and whole tile
    auto landed = [&]<int YOUNGER>() __attribute__((always_inline)) {
        static_assert(YOUNGER >= 0 && YOUNGER < 64, "the counter has six bits");
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(YOUNGER) : "memory");
    };

    const int c16 = lane & 15, g4 = lane >> 4;
    f32x4 acc[S::TM][S::TN];
    // The slab count is a template parameter: a fragment that has been requested from LDS and not yet waited
    // for must never cross a branch, where the compiler may copy its registers (before the data is there)
    // to merge the paths.
    auto multiply = [&]<int SLABS, int LOADS>() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < S::TM; ++i)
#pragma unroll
            for (int j = 0; j < S::TN; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        RawA af[2][S::TM];
        RawB bf[2][S::TN];
        landed.template operator()<(SLABS > 2 ? SLABS - 2 : 0) * LOADS + NST>();    // the first pair
        read_slab(af[0], bf[0], slab_offset(0));
        [&]<int... SL>(std::integer_sequence<int, SL...>) __attribute__((always_inline)) {
            ([&]() __attribute__((always_inline)) {
                constexpr int s = SL;
                shortk_wait(af[s & 1]);
                shortk_wait(bf[s & 1]);
                if constexpr (s + 1 < SLABS) {
                    if constexpr (s == 1) landed.template operator()<NST>();      // the second pair
                    read_slab(af[(s + 1) & 1], bf[(s + 1) & 1], slab_offset(s + 1));
                }
#pragma unroll
                for (int i = 0; i < S::TM; ++i) {
                    const u32x4 ua = shortk_value(af[s & 1][i]);
#pragma unroll
                    for (int j = 0; j < S::TN; ++j) {
                        const u32x4 ub = shortk_value(bf[s & 1][j]);
                        // B's fragment first: the block of C comes out transposed, four consecutive columns per lane
                        if constexpr (IS_BF16)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ub), __builtin_bit_cast(bf16x8, ua), acc[i][j], 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, ub), __builtin_bit_cast(f16x8, ua), acc[i][j], 0, 0, 0);
                    }
                }
            }(), ...);
        }
        (std::make_integer_sequence<int, SLABS>{});
    };

    // Accumulators -> C, without a pass through LDS.  With B's fragment first a lane of the accumulator layout
    // holds four consecutive columns of one row of a 16 x 16 block: row c16 of the block, columns 4*g4 .. +3,
    // where g4 numbers the wave's four rows of 16 lanes.  An fp32 C takes them as they are: 16 bytes per lane,
    // 64 contiguous bytes per row of C and instruction.  For a 16-bit C they are 8 bytes, and two neighbouring
    // blocks (columns 16j .. and 16j' .. of the same rows) trade halves first: v_permlane16_swap exchanges the
    // odd lane rows of its first operand with the even lane rows of its second, after which lane row 0 holds
    // columns 0-7 of block j, lane row 1 columns 0-7 of block j', lane rows 2 and 3 columns 8-15 of j and j':
    // 16 bytes per lane and again 64 contiguous bytes per row of C.  A second exchange (whole_lines below) makes
    // whole 128-byte lines of them.
    auto whole = [&](const Tile& x) { return x.m0 + S::BM <= a.M && x.n0 + S::BN <= a.N; };
    // A whole tile takes exactly NST store instructions per wave (assembly, so that the count is the source's
    // and not the compiler's); an edge tile takes as many as have a lane inside C.
    auto store16 = [&](bool inside_tile, bool lane_inside, char* p, u32x4 d) __attribute__((always_inline)) {
        // (a vector instruction that writes the data registers of a store of more than 8 bytes must stay two wait
        // states behind it; the compiler sees to that for its own stores and cannot know that this is one)
        if (inside_tile) asm volatile("global_store_dwordx4 %0, %1, off nt\n\ts_nop 1" ::"v"(p), "v"(d) : "memory");
        else if (lane_inside) __builtin_nontemporal_store(d, (u32x4*)p);
    };
    // Two 16-byte pieces per lane, `lower` 64 bytes before `upper` in the same row of C, held for rows c16 of a
    // block of 16 rows, become whole 128-byte lines: the two halves of each 16-lane row trade pieces (a rotation
    // by 8 within the row, written under a bank mask), after which lanes c16 < 8 hold `lower` and lanes
    // c16 >= 8 hold `upper` of the same eight rows, rows 0-7 in the first result and rows 8-15 in the second.
    // A store of 64-byte pieces is not only smaller: the L2 writes a line again when its other half arrives
    // (13 % more bytes written than C has for the batch of 32 products 2048 x 2048 x 128, 45 % with the two halves
    // stored back to back).
    auto whole_lines = [&](u32x4 lower, u32x4 upper, u32x4& rows_0_7, u32x4& rows_8_15) __attribute__((always_inline)) {
        constexpr int ROR8 = 0x128;         // row_ror:8
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            rows_0_7[q] = (uint32_t)__builtin_amdgcn_update_dpp((int)lower[q], (int)upper[q], ROR8, 0xf, 0xc, false);
            rows_8_15[q] = (uint32_t)__builtin_amdgcn_update_dpp((int)upper[q], (int)lower[q], ROR8, 0xf, 0x3, false);
        }
    };
    auto epilogue = [&](const Tile& x) __attribute__((always_inline)) {
        const float alpha = a.alpha;
        const int act = a.act;
        const bool inside = whole(x);
        const int r8 = c16 & 7, up = c16 >> 3;                      // row inside a half block; 1: this lane stores the upper piece
        const int64_t row0 = x.m0 + wm * S::WTM + r8;               // this lane's row in the first half of block row 0
        const int64_t colw = x.n0 + wn * S::WTN;                    // the wave's first column
        const int64_t row_step = (int64_t)16 * a.ldc * out_b, half_step = (int64_t)8 * a.ldc * out_b;
        if constexpr (OB == 4) {
            // a line is 32 columns: blocks j (lower piece) and j + 1 (upper piece)
            const int64_t col = colw + 16 * up + 4 * g4;
            char* p = x.C + (row0 * a.ldc + col) * out_b;
#pragma unroll
            for (int jp = 0; jp < S::TN / 2; ++jp) {
                f32x4 v[2][S::TM];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
#pragma unroll
                    for (int i = 0; i < S::TM; ++i) v[h][i] = alpha * acc[i][2 * jp + h];
                    apply_act4(v[h], act);
                }
#pragma unroll
                for (int i = 0; i < S::TM; ++i) {
                    u32x4 d0, d1;
                    whole_lines(__builtin_bit_cast(u32x4, v[0][i]), __builtin_bit_cast(u32x4, v[1][i]), d0, d1);
                    const bool cols_in = col + 32 * jp < a.N;
                    store16(inside, row0 + 16 * i < a.M && cols_in, p + i * row_step + jp * 32 * out_b, d0);
                    store16(inside, row0 + 16 * i + 8 < a.M && cols_in, p + i * row_step + half_step + jp * 32 * out_b, d1);
                }
            }
        } else {
            // a line is the wave's 64 columns: the pair of blocks 0, 1 (lower piece) and the pair 2, 3 (upper piece)
            static_assert(S::TN == 4, "two pairs of blocks make one line");
            const int64_t col = colw + 32 * up + 16 * (g4 & 1) + 8 * (g4 >> 1);
            char* p = x.C + (row0 * a.ldc + col) * out_b;
            u32x4 piece[2][S::TM];
#pragma unroll
            for (int jp = 0; jp < 2; ++jp) {
                u32x2 packed[2][S::TM];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    f32x4 v[S::TM];
#pragma unroll
                    for (int i = 0; i < S::TM; ++i) v[i] = alpha * acc[i][2 * jp + h];
                    apply_act4(v, act);
#pragma unroll
                    for (int i = 0; i < S::TM; ++i) {
                        if constexpr (OUT == DT_BF16) {
                            typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                            packed[h][i] = __builtin_bit_cast(u32x2, __builtin_convertvector(v[i], bf16x4));
                        } else {
                            typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
                            packed[h][i] = __builtin_bit_cast(u32x2, __builtin_convertvector(v[i], f16x4));
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < S::TM; ++i) {
                    const auto lo = __builtin_amdgcn_permlane16_swap(packed[0][i].x, packed[1][i].x, false, false);
                    const auto hi = __builtin_amdgcn_permlane16_swap(packed[0][i].y, packed[1][i].y, false, false);
                    piece[jp][i] = u32x4{lo[0], hi[0], lo[1], hi[1]};
                }
            }
            const bool cols_in = col < a.N;
#pragma unroll
            for (int i = 0; i < S::TM; ++i) {
                u32x4 d0, d1;
                whole_lines(piece[0][i], piece[1][i], d0, d1);
                store16(inside, row0 + 16 * i < a.M && cols_in, p + i * row_step, d0);
                store16(inside, row0 + 16 * i + 8 < a.M && cols_in, p + i * row_step + half_step, d1);
            }
        }
    };

    // The tile loop.  The operands of the next tile are requested as soon as every wave has read this tile's
    // (the epilogue needs no LDS), ahead of this tile's stores, so that they do not queue behind them.  The
    // multiplication's waits count NST younger stores; where the tile before was the first, or an edge tile
    // with fewer stores, everything in flight is awaited instead.
    // Which tiles a workgroup takes: a run of consecutive tiles.  Consecutive tiles share their panel of B
    // (until the column of tiles ends), which then stays where it is in LDS: only A is requested, half the
    // bytes.  Workgroups whose runs start in neighbouring columns of tiles walk down C side by side: what the
    // chip writes at any moment is spread over the width of C, and with it over the memory channels (runs along
    // the rows of C, with A staying, had every workgroup write the same few channels at once: 110 us for the
    // batch below instead of 68), and a panel of A is fetched once for the workgroups that need it together.
    // Workgroups are handed to the chip's XCDs in turn (workgroup b runs on XCD b mod 8), and each XCD has an L2
    // of its own: a matrix whose tiles are dealt out over all workgroups is fetched once by every XCD.  So the
    // tile list is first cut into eight contiguous parts, one per XCD, and each part into the runs of that
    // XCD's workgroups: the whole operands of a small matrix of a batch then come through one L2 only.
    constexpr int XCDS = 8;
    int first, last;
    {
        int wg = (int)blockIdx.x, wgs = (int)gridDim.x, lo = 0, hi = total_tiles;
        if (wgs % XCDS == 0) {
            const int xcd = wg % XCDS, part = (total_tiles + XCDS - 1) / XCDS;
            lo = xcd * part < total_tiles ? xcd * part : total_tiles;
            hi = lo + part < total_tiles ? lo + part : total_tiles;
            wg /= XCDS;
            wgs /= XCDS;
        }
        const int run = (hi - lo + wgs - 1) / wgs;
        first = lo + wg * run < hi ? lo + wg * run : hi;
        last = first + run < hi ? first + run : hi;
    }
    // The operands of the next tile are requested as soon as every wave has read this tile's (the epilogue
    // needs no LDS), ahead of this tile's stores, so that they do not queue behind them.  The multiplication's
    // waits count NST younger stores; where the tile before was the first, or an edge tile with fewer stores,
    // everything in flight is awaited instead.
    auto walk = [&]<int SLABS>() __attribute__((always_inline)) {
        int t = first;
        if (t >= last) return;
        Tile x = tile_of(t);
        bool with_b = true;
        request_pair.template operator()<SLABS, 0>(x, true);
        request_pair.template operator()<SLABS, 1>(x, true);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        while (true) {
            if (with_b) multiply.template operator()<SLABS, LA::L + LB::L>();
            else multiply.template operator()<SLABS, LA::L>();
            asm volatile("s_barrier" ::: "memory");                                   // the operands have been read by every wave
            const int tn = t + 1;
            const bool more = tn < last;
            Tile xn = x;
            if (more) {
                xn = tile_of(tn);
                with_b = xn.n0 != x.n0 || xn.B != x.B;
                request_pair.template operator()<SLABS, 0>(xn, with_b);
                request_pair.template operator()<SLABS, 1>(xn, with_b);
            }
            epilogue(x);
            if (!whole(x)) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            if (!more) break;
            x = xn;
            t = tn;
        }
    };
    switch (slabs) {
        case 1: walk.template operator()<1>(); break;
        case 2: walk.template operator()<2>(); break;
        case 3: walk.template operator()<3>(); break;
        case 4: walk.template operator()<4>(); break;
        default: break;
    }
}

inline int shortk_compute_units() {
    static int cus[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (!cus[dev]) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

// what the kernel takes beyond the preconditions of the tile family
inline bool shortk_supports(const Args& a) {
    if (a.dtype != DT_BF16 && a.dtype != DT_F16) return false;
    if (a.K % ShortK::BK != 0 || a.K > ShortK::MAX_SLABS * ShortK::BK || a.K <= 0) return false;
    if (a.beta != 0.0f || a.bias != nullptr || a.k_total != 0) return false;
    const int ob = elem_bytes(a.out_dtype);
    if (ShortK::lds_need((int)(a.K / ShortK::BK)) > ShortK::LDS_BYTES) return false;
    // 16-byte stores to C
    const int64_t per16 = 16 / ob;
    if (a.N % 8 != 0 || a.ldc % per16 != 0 || ((uintptr_t)a.C & 15)) return false;
    if (a.batch > 1 && (a.strideC * ob) % 16 != 0) return false;
    const int64_t tiles = ((a.M + 127) / 128) * ((a.N + 127) / 128) * a.batch;
    return tiles < ((int64_t)1 << 30);
}

// (a template, so that only the translation unit that calls it holds the kernels)
template <int UNUSED = 0>
hipError_t launch_shortk_variant(const Args& a, hipStream_t stream) {
    if (!shortk_supports(a)) return hipErrorInvalidValue;
    const int tiles_m = (int)((a.M + ShortK::BM - 1) / ShortK::BM), tiles_n = (int)((a.N + ShortK::BN - 1) / ShortK::BN);
    const int total = tiles_m * tiles_n * a.batch;
    const int cus = shortk_compute_units();
    const dim3 grid((unsigned)(total < 2 * cus ? total : 2 * cus)), block(ShortK::NT);
    const int slabs = (int)(a.K / ShortK::BK);
    const bool bf = a.dtype == DT_BF16, akc = !a.transA, bkc = a.transB != 0;
#define GEMM_SHORTK_LAUNCH(BF, AKC, BKC)                                                                                       \
    do {                                                                                                                       \
        if (a.out_dtype == DT_F32)                                                                                             \
            hipLaunchKernelGGL((tile_shortk_kernel<BF, AKC, BKC, DT_F32>), grid, block, 0, stream, a, tiles_m, tiles_n, total, slabs); \
        else if (a.out_dtype == DT_BF16)                                                                                       \
            hipLaunchKernelGGL((tile_shortk_kernel<BF, AKC, BKC, DT_BF16>), grid, block, 0, stream, a, tiles_m, tiles_n, total, slabs); \
        else                                                                                                                   \
            hipLaunchKernelGGL((tile_shortk_kernel<BF, AKC, BKC, DT_F16>), grid, block, 0, stream, a, tiles_m, tiles_n, total, slabs); \
    } while (0)
    if (bf) {
        if (akc && bkc) GEMM_SHORTK_LAUNCH(true, true, true);
        else if (akc && !bkc) GEMM_SHORTK_LAUNCH(true, true, false);
        else if (!akc && bkc) GEMM_SHORTK_LAUNCH(true, false, true);
        else GEMM_SHORTK_LAUNCH(true, false, false);
    } else {
        if (akc && bkc) GEMM_SHORTK_LAUNCH(false, true, true);
        else if (akc && !bkc) GEMM_SHORTK_LAUNCH(false, true, false);
        else if (!akc && bkc) GEMM_SHORTK_LAUNCH(false, false, true);
        else GEMM_SHORTK_LAUNCH(false, false, false);
    }
#undef GEMM_SHORTK_LAUNCH
    return hipGetLastError();
}

}  // namespace tile
}  // namespace gemm

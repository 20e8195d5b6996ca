// Persistent 128x128 tile kernel for short k loops (K <= 128, whole 32-wide slabs; bf16 / fp16).
//
// With a k loop of at most four slabs a tile is one trip to memory, half a microsecond of matrix
// arithmetic and a result to write: the per-head score products of attention are the model case (a
// batch of 2048 x 2048 x 128 products is 89 % result bytes).  Nothing in such a tile can be pipelined
// along k, and what the general tile kernels spend around their k loop (launch of a workgroup, ring
// fill, an epilogue staged in fp32 band by band) is here the whole cost.  This kernel keeps the
// instruction stream of a tile short and lets two workgroups per compute unit take turns:
//
//   a workgroup stays on its compute unit and walks a list of tiles; per tile it
//     requests all operands of the tile at once into its 64 KiB of LDS (direct-to-LDS loads),
//     multiplies slab by slab as they land (16x16x32 MFMA, four waves of 64x64),
//     applies alpha, the activation and the one rounding in the accumulator layout and parks the
//     results, in the type of C, where the operands were (a region per wave, swizzled in 16-byte units),
//     reads them back row by row and writes C with full 16-byte stores (128-byte row segments for
//     16-bit results).
//   While one workgroup of a compute unit waits for its operands or moves its results, the other
//   multiplies.  The waits for the operands count this wave's operations in flight; the stores of the
//   tile before are older than the loads and have had the loads' whole latency to retire.
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
    // bytes of LDS a call needs: the operands of a tile, then (in the same place) its staged results
    static constexpr int lds_need(int slabs, int out_bytes) { return slabs * SLAB > BM * BN * out_bytes ? slabs * SLAB : BM * BN * out_bytes; }
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
    constexpr int ROW_BYTES = S::WTN * OB;                    // a staged row of a wave: 128 or 256 bytes
    constexpr int UNITS = ROW_BYTES / 16;                     // 16-byte units per staged row
    constexpr int RPI = 64 / UNITS;                           // rows per read-back instruction
    __shared__ __attribute__((aligned(1024))) char lds[S::LDS_BYTES];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const uint32_t lds0 = (uint32_t)(uintptr_t)GEMM_LDS_PTR(lds);
    // staged results: the 64 x 64 quadrant of wave q at q * 64 rows
    const uint32_t staging0 = lds0 + (uint32_t)(wave * (S::WTM * ROW_BYTES));

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
        const int tm = r / tiles_n, tn = r - tm * tiles_n;          // consecutive tiles share a panel of A
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
    // all slabs of tile `x` into LDS: a descriptor per slab, exact range checks
    auto request = [&]<int SLABS>(const Tile& x) __attribute__((always_inline)) {
        LA la = la_full;
        LB lb = lb_full;
        if (LA::TRANSPOSED && a.M - x.m0 < S::BM) la.init(tid, a.lda, (int)(a.M - x.m0));
        if (LB::TRANSPOSED && a.N - x.n0 < S::BN) lb.init(tid, a.ldb, (int)(a.N - x.n0));
        const char* pa = LA::tile_base(x.A, x.m0, a.lda);
        const char* pb = LB::tile_base(x.B, x.n0, a.ldb);
        const int64_t a_bytes = LA::total_bytes(a.M, a.K, a.lda) - (pa - x.A);
        const int64_t b_bytes = LB::total_bytes(a.N, a.K, a.ldb) - (pb - x.B);
        // Slabs go out in pairs: a k-contiguous operand contributes 64 bytes per row and slab, half a cache
        // line, and the two loads that fetch the two halves of the same rows, issued next to each other, are
        // merged into one line request on the way (the L2 serves a half-line request at the cost of a full one).
#pragma unroll
        for (int s = 0; s < SLABS; s += 2) {
            const bool TWO = s + 1 < SLABS;          // (a constant once the loop is unrolled)
            const __amdgpu_buffer_rsrc_t ra0 = make_rsrc(pa + s * a_step, a_bytes - s * a_step);
            const __amdgpu_buffer_rsrc_t rb0 = make_rsrc(pb + s * b_step, b_bytes - s * b_step);
            const __amdgpu_buffer_rsrc_t ra1 = TWO ? make_rsrc(pa + (s + 1) * a_step, a_bytes - (s + 1) * a_step) : ra0;
            const __amdgpu_buffer_rsrc_t rb1 = TWO ? make_rsrc(pb + (s + 1) * b_step, b_bytes - (s + 1) * b_step) : rb0;
            char* dst = lds + s * S::SLAB;
#pragma unroll
            for (int i = 0; i < LA::L; ++i) {
                la.issue(false, i, ra0, dst, wave, tid, s * S::BK, (int)a.K);
                if (TWO) la.issue(false, i, ra1, dst + S::SLAB, wave, tid, (s + 1) * S::BK, (int)a.K);
            }
#pragma unroll
            for (int i = 0; i < LB::L; ++i) {
                lb.issue(false, i, rb0, dst + S::A_BYTES, wave, tid, s * S::BK, (int)a.K);
                if (TWO) lb.issue(false, i, rb1, dst + S::SLAB + S::A_BYTES, wave, tid, (s + 1) * S::BK, (int)a.K);
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

    // The slabs of a tile are requested at once and arrive pair after pair (64 KiB take the load path of a
    // compute unit half a microsecond); the multiplication starts on the first pair while the second is on its
    // way.  landed<Y>() waits until all but the Y last-requested loads of this wave have landed, then meets the
    // other waves.  The loads of a wave retire in order among themselves, so once at most Y operations are in
    // flight the older loads are done, whatever stores of the tile before are still among them.
    constexpr int LPS = LA::L + LB::L;          // loads per thread and slab
    auto landed = [&]<int YOUNGER>() __attribute__((always_inline)) {
        static_assert(YOUNGER >= 0 && YOUNGER < 64, "the counter has six bits");
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(YOUNGER) : "memory");
    };

    const int c16 = lane & 15, g4 = lane >> 4;
    f32x4 acc[S::TM][S::TN];
    // The slab count is a template parameter: a fragment that has been requested from LDS and not yet waited
    // for must never cross a branch, where the compiler may copy its registers (before the data is there)
    // to merge the paths.
    auto multiply = [&]<int SLABS>() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < S::TM; ++i)
#pragma unroll
            for (int j = 0; j < S::TN; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        RawA af[2][S::TM];
        RawB bf[2][S::TN];
        landed.template operator()<(SLABS > 2 ? SLABS - 2 : 0) * LPS>();
        read_slab(af[0], bf[0], 0u);
        [&]<int... SL>(std::integer_sequence<int, SL...>) __attribute__((always_inline)) {
            ([&]() __attribute__((always_inline)) {
                constexpr int s = SL;
                shortk_wait(af[s & 1]);
                shortk_wait(bf[s & 1]);
                if constexpr (s + 1 < SLABS) {
                    if constexpr (s == 1) landed.template operator()<0>();        // the second pair
                    read_slab(af[(s + 1) & 1], bf[(s + 1) & 1], (uint32_t)((s + 1) * S::SLAB));
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

    // Staged layout of a wave's 64 x 64 results: row r at r * ROW_BYTES, 16-byte unit u of the row at
    // position u xor (r mod UNITS').  A lane of the accumulator layout (row c16 of a block, columns
    // 4*g4 .. +3) writes 8 (16-bit results) or 16 bytes; the read-back takes whole units.
    auto unit_pos = [](int row, int unit) { return unit ^ (row & (UNITS - 1)); };
    // alpha, activation, rounding; accumulators -> staging
    auto stage_results = [&]() __attribute__((always_inline)) {
        const float alpha = a.alpha;
        const int act = a.act;
#pragma unroll
        for (int j = 0; j < S::TN; ++j) {
            f32x4 v[S::TM];
#pragma unroll
            for (int i = 0; i < S::TM; ++i) v[i] = alpha * acc[i][j];
            apply_act4(v, act);
#pragma unroll
            for (int i = 0; i < S::TM; ++i) {
                const int row = 16 * i + c16;
                const int byte_in_row = (16 * j + 4 * g4) * OB;
                const uint32_t addr = staging0 + (uint32_t)(row * ROW_BYTES + (unit_pos(row, byte_in_row >> 4) << 4) + (byte_in_row & 15));
                if constexpr (OUT == DT_F32) {
                    asm volatile("ds_write_b128 %0, %1" ::"v"(addr), "v"(v[i]) : "memory");
                } else if constexpr (OUT == DT_BF16) {
                    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
                    const u32x2 p = __builtin_bit_cast(u32x2, __builtin_convertvector(v[i], bf16x4));
                    asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(p) : "memory");
                } else {
                    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
                    const u32x2 p = __builtin_bit_cast(u32x2, __builtin_convertvector(v[i], f16x4));
                    asm volatile("ds_write_b64 %0, %1" ::"v"(addr), "v"(p) : "memory");
                }
            }
        }
    };
    // staging -> C: the wave's own quadrant, a lane moves one 16-byte unit of a row per trip
    auto write_results = [&](const Tile& x) __attribute__((always_inline)) {
        constexpr int TRIPS = S::WTM / RPI;
        const int rr = lane / UNITS, u = lane % UNITS;
        const int64_t col = x.n0 + wn * S::WTN + (u * 16) / OB;
        const int64_t row0 = x.m0 + wm * S::WTM + rr;
        u32x4 d[TRIPS];
#pragma unroll
        for (int it = 0; it < TRIPS; ++it) {
            const int row = it * RPI + rr;
            const uint32_t addr = staging0 + (uint32_t)(row * ROW_BYTES + (unit_pos(row, u) << 4));
            asm volatile("ds_read_b128 %0, %1" : "=v"(d[it]) : "v"(addr) : "memory");
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int it = 0; it < TRIPS; ++it) asm volatile("" : "+v"(d[it]));          // nothing that uses the data moves ahead of the wait
        char* p = x.C + (row0 * a.ldc + col) * out_b;
        const int64_t step = (int64_t)RPI * a.ldc * out_b;
        if (x.m0 + S::BM <= a.M && x.n0 + S::BN <= a.N) {          // whole tile inside C: no lane conditions
#pragma unroll
            for (int it = 0; it < TRIPS; ++it) __builtin_nontemporal_store(d[it], (u32x4*)(p + it * step));
        } else if (col < a.N) {                                      // N is a multiple of 8: a unit lies inside or outside as a whole
#pragma unroll
            for (int it = 0; it < TRIPS; ++it)
                if (row0 + it * RPI < a.M) __builtin_nontemporal_store(d[it], (u32x4*)(p + it * step));
        }
    };

    const int stride = (int)gridDim.x;
    auto walk = [&]<int SLABS>() __attribute__((always_inline)) {
        for (int t = (int)blockIdx.x; t < total_tiles; t += stride) {
            const Tile x = tile_of(t);
            request.template operator()<SLABS>(x);
            multiply.template operator()<SLABS>();
            asm volatile("s_barrier" ::: "memory");                                   // the operands have been read by every wave
            stage_results();
            write_results(x);
            asm volatile("s_barrier" ::: "memory");                                   // the staged results have been read back
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
    if (ShortK::lds_need((int)(a.K / ShortK::BK), ob) > ShortK::LDS_BYTES) return false;
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

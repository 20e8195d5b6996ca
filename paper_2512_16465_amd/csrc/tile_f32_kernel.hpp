// Macro-tile kernel for fp32 operands on the fp32 matrix instruction (gfx950).
//
// v_mfma_f32_32x32x2_f32 takes one float of A and one of B per lane (lane l: row / column l%32,
// k = l/32) and lasts 64 cycles: the fp32 matrix rate is a sixteenth of the bf16 one, so this
// kernel is bound by the matrix pipe by a wide margin and is kept simple - 128x128 tile, BK = 32,
// four waves of 64x64, operands staged global -> registers -> LDS in two stages, two workgroups
// per compute unit.
//
// The order of the k index inside a group of eight is free (both operands use the same), so
// lane half h takes k = 4h .. 4h+3 of the group over four consecutive MFMAs.  A k-contiguous
// operand then needs one 16-byte LDS read per 32 rows and group (rows padded to BK + 4 floats: the
// reads of 16 consecutive rows fall on distinct banks); an m/n-contiguous operand is kept as
// [k][row] and read one float at a time (32 consecutive lanes read 32 consecutive floats).  No
// transposition is needed for any of the four layouts.
//
// Edges as in the 16-bit kernels: loads past the end of an operand return zero through the
// buffer descriptor's range check; chunks of a k-contiguous operand past K are masked.
#pragma once
#include "tile_kernel.hpp"

namespace gemm {
namespace tile {

// SIDE = rows and columns of the workgroup tile: 128 (four waves of 64x64) or 64 (four waves of
// 32x32, for problems with too few 128x128 tiles to fill the chip).
template <int SIDE>
struct F32CfgT {
    static_assert(SIDE == 128 || SIDE == 64, "two tile sizes");
    static constexpr int BM = SIDE, BN = SIDE, BK = 32, WM = 2, WN = 2;
    static constexpr int NT = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int KC_STRIDE = BK + 4;          // floats per row of a k-contiguous slab in LDS
    static constexpr int MC_STRIDE = SIDE + 8;        // floats per k-row of an m/n-contiguous slab: the two lane halves read k-rows
                                                      // four apart, 4 * (SIDE + 8) floats = 32 banks (mod 64) from each other
    static constexpr int OPERAND_BYTES = SIDE * KC_STRIDE * 4 > BK * MC_STRIDE * 4 ? SIDE * KC_STRIDE * 4 : BK * MC_STRIDE * 4;
    static constexpr int STAGE = 2 * OPERAND_BYTES;
    static constexpr int WGS_PER_CU = SIDE == 128 ? 2 : 4;
};
using F32Cfg = F32CfgT<128>;

// One operand's slab: SIDE rows x BK k, L 16-byte chunks per thread.
template <bool KC, class F32Cfg>
struct F32Mover {
    static constexpr int L = F32Cfg::BM * F32Cfg::BK / 4 / F32Cfg::NT;   // chunks per thread
    static constexpr int CPR = F32Cfg::BK / 4;                      // 16-byte chunks per row of a k-contiguous slab
    static constexpr int CPK = F32Cfg::BM / 4;                      // 16-byte chunks per k-row of an m/n-contiguous slab
    uint32_t goff[L];      // byte offset of the chunk from the slab's first byte
    uint32_t loff[L];      // byte offset in the operand's LDS region
    u32x4 r[L];
    int valid_k;           // k values of the slab in r that lie inside K

    __device__ __forceinline__ void init(int tid, int64_t ld) {
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const uint32_t q = i * F32Cfg::NT + tid;
            if (KC) {
                const uint32_t row = q / CPR, c = q % CPR;             // CPR chunks cover a row's BK k
                goff[i] = (uint32_t)((row * ld + c * 4) * 4);
                loff[i] = (row * F32Cfg::KC_STRIDE + c * 4) * 4;
            } else {
                const uint32_t k = q / CPK, c = q % CPK;               // CPK chunks cover a k-row's columns
                goff[i] = (uint32_t)((k * ld + c * 4) * 4);
                loff[i] = (k * F32Cfg::MC_STRIDE + c * 4) * 4;
            }
        }
    }
    static __device__ __forceinline__ const char* tile_base(const void* p, int64_t first_row, int64_t ld) {
        return KC ? (const char*)p + first_row * ld * 4 : (const char*)p + first_row * 4;
    }
    static __device__ __forceinline__ int64_t k_step_bytes(int64_t ld) { return KC ? (int64_t)F32Cfg::BK * 4 : (int64_t)F32Cfg::BK * ld * 4; }
    static __device__ __forceinline__ int64_t total_bytes(int64_t rows, int64_t K, int64_t ld) {
        return KC ? ((rows - 1) * ld + K) * 4 : ((K - 1) * ld + rows) * 4;
    }
    // base = first byte of the slab, avail = bytes from there to the end of the operand.  Every
    // chunk is requested (one past the end of the operand reads as zero through the descriptor's
    // range check); the chunks of a k-contiguous operand that lie past K hold whatever follows the
    // row in memory and are cleared in lstore, once they have arrived -- clearing them here would
    // be a write to a register with a load in flight, which waits for the load.
    __device__ __forceinline__ void gload(const char* base, int64_t avail, int k0, int K) {
        const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(base, avail);
        valid_k = K - k0;
#pragma unroll
        for (int i = 0; i < L; ++i) r[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[i], 0, 0));
    }
    __device__ __forceinline__ void lstore(char* region, int tid) {
#pragma unroll
        for (int i = 0; i < L; ++i) {
            if (KC && valid_k < F32Cfg::BK) {                          // wave-uniform: only the last slab of a ragged K
                const int c = (i * F32Cfg::NT + tid) % CPR;
                if (c * 4 >= valid_k) r[i] = u32x4{0u, 0u, 0u, 0u};
            }
            *(u32x4*)(region + loff[i]) = r[i];
        }
    }
    // the four floats k = 8g + 4h + (0..3) of row `row` (tile-local) for lane half h
    static __device__ __forceinline__ f32x4 frag(const char* region, int row, int g, int h) {
        if (KC) return *(const f32x4*)(region + (row * F32Cfg::KC_STRIDE + 8 * g + 4 * h) * 4);
        f32x4 v;
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = *(const float*)(region + ((8 * g + 4 * h + j) * F32Cfg::MC_STRIDE + row) * 4);
        return v;
    }
};

template <class C, bool A_KC, bool B_KC>
__global__ __launch_bounds__(C::NT, C::WGS_PER_CU) void tile_f32_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok) {
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
    const int64_t m0 = (int64_t)tm * C::BM, n0 = (int64_t)tn * C::BN;
    const int K = (int)a.K;

    F32Mover<A_KC, C> la;
    F32Mover<B_KC, C> lb;
    la.init(tid, a.lda);
    lb.init(tid, a.ldb);
    const char* pa = F32Mover<A_KC, C>::tile_base(a.A, m0, a.lda);
    const char* pb = F32Mover<B_KC, C>::tile_base(a.B, n0, a.ldb);
    const int64_t a_step = F32Mover<A_KC, C>::k_step_bytes(a.lda), b_step = F32Mover<B_KC, C>::k_step_bytes(a.ldb);
    const int64_t a_bytes = F32Mover<A_KC, C>::total_bytes(a.M, a.K, a.lda) - (pa - (const char*)a.A);
    const int64_t b_bytes = F32Mover<B_KC, C>::total_bytes(a.N, a.K, a.ldb) - (pb - (const char*)a.B);

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int k_tiles = (K + C::BK - 1) / C::BK;
    auto gload = [&](int t) {
        la.gload(pa + t * a_step, a_bytes - t * a_step, t * C::BK, K);
        lb.gload(pb + t * b_step, b_bytes - t * b_step, t * C::BK, K);
    };
    auto lstore = [&](int stage) {
        la.lstore(lds + stage * C::STAGE, tid);
        lb.lstore(lds + stage * C::STAGE + C::OPERAND_BYTES, tid);
    };

    // Pipeline of one slab kt (G groups of 16 MFMAs): the next slab's global loads are issued at
    // its start and land in registers behind the MFMAs; the fragments of group g+1 are read from
    // LDS before the MFMAs of group g are issued; before the last group the next slab goes from
    // registers to the other LDS stage, the workgroup meets at the barrier, and the first
    // fragments of the next slab are read -- all of it behind the last group's MFMAs.  The other
    // stage is free at that point: its last readers took their fragments before the previous
    // barrier.
    constexpr int G = C::BK / 8;
    static_assert(G % 2 == 0, "fragment buffers alternate and group 0 uses buffer 0");
    f32x4 fa[2][C::TM], fb[2][C::TN];
    auto read_frags = [&](int buf, const char* stage, int g) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i) fa[buf][i] = F32Mover<A_KC, C>::frag(stage, wm * C::WTM + i * 32 + l32, g, lhi);
#pragma unroll
        for (int j = 0; j < C::TN; ++j) fb[buf][j] = F32Mover<B_KC, C>::frag(stage + C::OPERAND_BYTES, wn * C::WTN + j * 32 + l32, g, lhi);
    };
    if (k_tiles > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
        read_frags(0, lds, 0);
        for (int kt = 0; kt < k_tiles; ++kt) {
            const char* cur = lds + (kt & 1) * C::STAGE;
            const char* nxt = lds + ((kt + 1) & 1) * C::STAGE;
            const bool more = kt + 1 < k_tiles;
            if (more) gload(kt + 1);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                if (g + 1 < G) {
                    read_frags((g + 1) & 1, cur, g + 1);
                } else if (more) {
                    lstore((kt + 1) & 1);
                    __syncthreads();
                    read_frags(0, nxt, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < C::TM; ++i)
#pragma unroll
                        for (int j = 0; j < C::TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[g & 1][i][q], fb[g & 1][j][q], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    __syncthreads();                                      // LDS is reused by the epilogue
    tile_epilogue<C>(acc, lds, a, m0, n0, c_vec_ok);
}

template <class C>
inline hipError_t launch_f32_variant(const Args& a, int group_m, hipStream_t stream) {
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)a.batch), block(C::NT);
    const bool akc = !a.transA, bkc = a.transB != 0;
    const int c_vec_ok = c_rows_take_vec4(a);
#define GEMM_TILE_LAUNCH(AKC, BKC) \
    hipLaunchKernelGGL((tile_f32_kernel<C, AKC, BKC>), grid, block, 0, stream, a, tiles_m, tiles_n, group_m, c_vec_ok)
    if (akc && bkc) GEMM_TILE_LAUNCH(true, true);
    else if (akc && !bkc) GEMM_TILE_LAUNCH(true, false);
    else if (!akc && bkc) GEMM_TILE_LAUNCH(false, true);
    else GEMM_TILE_LAUNCH(false, false);
#undef GEMM_TILE_LAUNCH
    return hipGetLastError();
}

}  // namespace tile
}  // namespace gemm

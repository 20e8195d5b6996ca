// Macro-tile kernel for fp32 operands on the fp32 matrix instruction (gfx950).
//
// v_mfma_f32_32x32x2_f32 takes one float of A and one of B per lane (lane l: row / column l%32,
// k = l/32) and lasts 64 cycles: the fp32 matrix rate is a sixteenth of the bf16 one, so this
// kernel is bound by the matrix pipe by a wide margin and is kept simple - 128x128 tile, BK = 16,
// four waves of 64x64, operands staged global -> registers -> LDS in two stages, two workgroups
// per compute unit.
//
// The order of the k index inside a group of eight is free (both operands use the same), so
// lane half h takes k = 4h .. 4h+3 of the group over four consecutive MFMAs.  A k-contiguous
// operand then needs one 16-byte LDS read per 32 rows and group (rows padded to 20 floats: the
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

struct F32Cfg {
    static constexpr int BM = 128, BN = 128, BK = 16, WM = 2, WN = 2;
    static constexpr int NT = WM * WN * 64;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int KC_STRIDE = BK + 4;          // floats per row of a k-contiguous slab in LDS
    static constexpr int MC_STRIDE = 128 + 4;         // floats per k-row of an m/n-contiguous slab
    static constexpr int OPERAND_BYTES = 128 * KC_STRIDE * 4 > BK * MC_STRIDE * 4 ? 128 * KC_STRIDE * 4 : BK * MC_STRIDE * 4;
    static constexpr int STAGE = 2 * OPERAND_BYTES;
};

// One operand's slab: 128 rows x 16 k, two 16-byte chunks per thread.
template <bool KC>
struct F32Mover {
    static constexpr int L = 128 * F32Cfg::BK / 4 / F32Cfg::NT;     // chunks per thread
    uint32_t goff[L];      // byte offset of the chunk from the slab's first byte
    uint32_t loff[L];      // byte offset in the operand's LDS region
    u32x4 r[L];

    __device__ __forceinline__ void init(int tid, int64_t ld) {
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const uint32_t q = i * F32Cfg::NT + tid;
            if (KC) {
                const uint32_t row = q / 4, c = q % 4;                 // four chunks cover a row's 16 k
                goff[i] = (uint32_t)((row * ld + c * 4) * 4);
                loff[i] = (row * F32Cfg::KC_STRIDE + c * 4) * 4;
            } else {
                const uint32_t k = q / 32, c = q % 32;                 // 32 chunks cover a k-row's 128 columns
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
    // base = first byte of the slab, avail = bytes from there to the end of the operand
    __device__ __forceinline__ void gload(const char* base, int64_t avail, int tid, int k0, int K) {
        const __amdgpu_buffer_rsrc_t rsrc = make_rsrc(base, avail);
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const int c = (i * F32Cfg::NT + tid) % 4;
            if (!KC || k0 + c * 4 < K) r[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[i], 0, 0));
            else r[i] = u32x4{0u, 0u, 0u, 0u};
        }
    }
    __device__ __forceinline__ void lstore(char* region) const {
#pragma unroll
        for (int i = 0; i < L; ++i) *(u32x4*)(region + loff[i]) = r[i];
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

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(F32Cfg::NT, 2) void tile_f32_kernel(Args a, int tiles_m, int tiles_n, int group_m, int c_vec_ok) {
    using C = F32Cfg;
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

    F32Mover<A_KC> la;
    F32Mover<B_KC> lb;
    la.init(tid, a.lda);
    lb.init(tid, a.ldb);
    const char* pa = F32Mover<A_KC>::tile_base(a.A, m0, a.lda);
    const char* pb = F32Mover<B_KC>::tile_base(a.B, n0, a.ldb);
    const int64_t a_step = F32Mover<A_KC>::k_step_bytes(a.lda), b_step = F32Mover<B_KC>::k_step_bytes(a.ldb);
    const int64_t a_bytes = F32Mover<A_KC>::total_bytes(a.M, a.K, a.lda) - (pa - (const char*)a.A);
    const int64_t b_bytes = F32Mover<B_KC>::total_bytes(a.N, a.K, a.ldb) - (pb - (const char*)a.B);

    f32x16 acc[C::TM][C::TN];
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int k_tiles = (K + C::BK - 1) / C::BK;
    auto gload = [&](int t) {
        la.gload(pa + t * a_step, a_bytes - t * a_step, tid, t * C::BK, K);
        lb.gload(pb + t * b_step, b_bytes - t * b_step, tid, t * C::BK, K);
    };
    auto lstore = [&](int stage) {
        la.lstore(lds + stage * C::STAGE);
        lb.lstore(lds + stage * C::STAGE + C::OPERAND_BYTES);
    };

    if (k_tiles > 0) {
        gload(0);
        lstore(0);
        __syncthreads();
        for (int kt = 0; kt < k_tiles; ++kt) {
            const char* sa = lds + (kt & 1) * C::STAGE;
            const char* sb = sa + C::OPERAND_BYTES;
            if (kt + 1 < k_tiles) gload(kt + 1);          // in flight while this slab is multiplied
#pragma unroll
            for (int g = 0; g < C::BK / 8; ++g) {
                f32x4 fa[C::TM], fb[C::TN];
#pragma unroll
                for (int i = 0; i < C::TM; ++i) fa[i] = F32Mover<A_KC>::frag(sa, wm * C::WTM + i * 32 + l32, g, lhi);
#pragma unroll
                for (int j = 0; j < C::TN; ++j) fb[j] = F32Mover<B_KC>::frag(sb, wn * C::WTN + j * 32 + l32, g, lhi);
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < C::TM; ++i)
#pragma unroll
                        for (int j = 0; j < C::TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i][q], fb[j][q], acc[i][j], 0, 0, 0);
            }
            if (kt + 1 < k_tiles) {
                lstore((kt + 1) & 1);                     // the other stage: its readers passed the barrier of step kt-1
                __syncthreads();
            }
        }
    }
    __syncthreads();                                      // LDS is reused by the epilogue
    tile_epilogue<C>(acc, lds, a, m0, n0, c_vec_ok);
}

inline hipError_t launch_f32_variant(const Args& a, int group_m, hipStream_t stream) {
    using C = F32Cfg;
    const int tiles_m = (int)((a.M + C::BM - 1) / C::BM), tiles_n = (int)((a.N + C::BN - 1) / C::BN);
    const dim3 grid((unsigned)(tiles_m * tiles_n), (unsigned)a.batch), block(C::NT);
    const bool akc = !a.transA, bkc = a.transB != 0;
    const int c_vec_ok = c_rows_take_vec4(a);
#define GEMM_TILE_LAUNCH(AKC, BKC) \
    hipLaunchKernelGGL((tile_f32_kernel<AKC, BKC>), grid, block, 0, stream, a, tiles_m, tiles_n, group_m, c_vec_ok)
    if (akc && bkc) GEMM_TILE_LAUNCH(true, true);
    else if (akc && !bkc) GEMM_TILE_LAUNCH(true, false);
    else if (!akc && bkc) GEMM_TILE_LAUNCH(false, true);
    else GEMM_TILE_LAUNCH(false, false);
#undef GEMM_TILE_LAUNCH
    return hipGetLastError();
}

}  // namespace tile
}  // namespace gemm

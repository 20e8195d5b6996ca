// Table of macro-tile variants and the preconditions of the family.
#include "tile_kernel.hpp"

namespace gemm {

#define GEMM_TILE_VARIANT(IDX, NAME, KIND, BM, BN, BK, WM, WN, NS) \
    hipError_t launch_tile_variant_##IDX(const Args& a, int group_m, const TileSplit& split, hipStream_t stream);
#include "tile_variants.def"
#undef GEMM_TILE_VARIANT

namespace {

typedef hipError_t (*launch_fn)(const Args&, int, const TileSplit&, hipStream_t);

const TileVariantInfo kInfo[] = {
#define GEMM_TILE_VARIANT(IDX, NAME, KIND, BM, BN, BK, WM, WN, NS) {NAME, BM, BN, BK, (WM) * (WN) * 64, KIND},
#include "tile_variants.def"
#undef GEMM_TILE_VARIANT
};

const launch_fn kLaunch[] = {
#define GEMM_TILE_VARIANT(IDX, NAME, KIND, BM, BN, BK, WM, WN, NS) launch_tile_variant_##IDX,
#include "tile_variants.def"
#undef GEMM_TILE_VARIANT
};

constexpr int kNum = (int)(sizeof(kInfo) / sizeof(kInfo[0]));

}  // namespace

int tile_num_variants() { return kNum; }

const TileVariantInfo* tile_variant_info(int variant) {
    return (variant >= 0 && variant < kNum) ? &kInfo[variant] : nullptr;
}

// 16-byte vector loads along the contiguous dimension of each operand (8 elements of 16 bits,
// 4 of 32), 32-bit byte offsets inside a tile, and a 32-bit workgroup count.
bool tile_supports(const Args& a) {
    if (a.dtype != DT_BF16 && a.dtype != DT_F16 && a.dtype != DT_F32) return false;
    const int64_t chunk = a.dtype == DT_F32 ? 4 : 8;
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
    if (((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return false;
    if ((a.lda % chunk) || (a.ldb % chunk)) return false;
    if (a.lda > (1 << 22) || a.ldb > (1 << 22)) return false;
    if (a.K > (1 << 30)) return false;
    // the contiguous dimension of each operand must be whole 16-byte chunks
    if ((!a.transA ? a.K : a.M) % chunk) return false;
    if ((a.transB ? a.K : a.N) % chunk) return false;
    const int64_t tiles = ((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (tiles > (int64_t)1 << 30) return false;
    return true;
}

// A variant takes either 16-bit or 32-bit operands.  The direct-to-LDS variants mask lanes with a
// fixed out-of-range offset of 2 GiB - 16.
bool tile_variant_supports(const Args& a, int variant) {
    if (variant < 0 || variant >= kNum) return false;
    if ((kInfo[variant].kind == 4) != (a.dtype == DT_F32)) return false;
    if (kInfo[variant].kind == 0 || kInfo[variant].kind == 4) return true;
    if (kInfo[variant].kind == 5 && !shortk_call_fits(a)) return false;
    const int64_t a_bytes = ((a.transA ? a.K : a.M) * a.lda) * 2, b_bytes = ((a.transB ? a.N : a.K) * a.ldb) * 2;
    return a_bytes < 0x7ffffff0ll && b_bytes < 0x7ffffff0ll;
}

// The persistent short-k kernel (kind 5): whole slabs, K <= 128 (the operands of a tile inside 64 KiB of LDS),
// C write-only, no bias, stored in 16-byte pieces.  (Restated here from
// tile_shortk_kernel.hpp, which only the variant's own translation unit includes.)
bool shortk_call_fits(const Args& a) {
    if (a.K % 32 != 0 || a.K > 128 || a.beta != 0.0f || a.bias != nullptr || a.k_total != 0) return false;
    const int64_t ob = elem_bytes(a.out_dtype);
    if (a.N % 8 != 0 || a.ldc % (16 / ob) != 0 || ((uintptr_t)a.C & 15)) return false;
    if (a.batch > 1 && (a.strideC * ob) % 16 != 0) return false;
    return true;
}

bool tile_variant_splits(int variant) { return variant >= 0 && variant < kNum && kInfo[variant].kind == 3; }
bool tile_variant_slices(int variant) { return variant >= 0 && variant < kNum && kInfo[variant].kind != 3 && kInfo[variant].kind != 5; }

hipError_t launch_tile(const Args& a, int variant, int group_m, const TileSplit& split, hipStream_t stream) {
    if (variant < 0 || variant >= kNum) return hipErrorInvalidValue;
    if (split.parts > 1 && !tile_variant_splits(variant)) return hipErrorInvalidValue;
    return kLaunch[variant](a, group_m < 1 ? 1 : group_m, split, stream);
}

namespace {

// Adds the partial tiles of a split in the order of their k shares and applies the epilogue:
// one thread per four consecutive columns of a tile row.  The kernel is one round trip to memory
// long, so the loads of all shares (P > 0: their number is fixed at compile time; P == 0: any
// number, four at a time) and of C_in and bias are issued before the first use.
template <int P>
__global__ __launch_bounds__(256) void tile_split_reduce_kernel(Args a, int tiles_m, int tiles_n, int group_m, int first_tile,
                                                                int parts, const float* partials, int BM, int BN, int c_vec_ok) {
    int tm, tn;
    tile::tile_of_workgroup(first_tile + (int)blockIdx.x, tiles_m, tiles_n, group_m, tm, tn);
    const int idx = (int)blockIdx.y * 256 + (int)threadIdx.x;          // one of BM * BN / 4 vectors
    const int r = idx / (BN / 4), c = (idx % (BN / 4)) * 4;
    const int64_t row = (int64_t)tm * BM + r, col = (int64_t)tn * BN + c;
    if (row >= a.M || col >= a.N) return;
    const size_t tile_floats = (size_t)BM * BN;
    const float* p = partials + ((size_t)blockIdx.x * parts) * tile_floats + (size_t)r * BN + c;
    float c_in[4] = {0.0f, 0.0f, 0.0f, 0.0f}, bj[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    auto load_inputs = [&]() {
        const bool vec = c_vec_ok && col + 3 < a.N;
        if (vec && a.beta != 0.0f) {
            const int64_t ci = row * a.ldc + col;
            f32x4 v;
            if (a.out_dtype == DT_F32) v = tile::OutVec<DT_F32>::load4((const float*)a.C + ci);
            else if (a.out_dtype == DT_BF16) v = tile::OutVec<DT_BF16>::load4((const uint16_t*)a.C + ci);
            else v = tile::OutVec<DT_F16>::load4((const uint16_t*)a.C + ci);
#pragma unroll
            for (int e = 0; e < 4; ++e) c_in[e] = v[e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (col + e >= a.N) break;
            if (!vec && a.beta != 0.0f) c_in[e] = load_elem(a.C, a.out_dtype, row * a.ldc + col + e);
            if (a.bias) bj[e] = load_elem(a.bias, a.bias_dtype, col + e);
        }
    };
    f32x4 s;
    if constexpr (P > 0) {
        f32x4 v[P];
#pragma unroll
        for (int q = 0; q < P; ++q) v[q] = *(const f32x4*)(p + (size_t)q * tile_floats);
        load_inputs();
        s = v[0];
#pragma unroll
        for (int q = 1; q < P; ++q) s += v[q];
    } else {
        load_inputs();
        s = *(const f32x4*)p;
        int q = 1;
        for (; q + 4 <= parts; q += 4) {
            f32x4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *(const f32x4*)(p + (size_t)(q + u) * tile_floats);
#pragma unroll
            for (int u = 0; u < 4; ++u) s += v[u];
        }
        for (; q < parts; ++q) s += *(const f32x4*)(p + (size_t)q * tile_floats);
    }
    f32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = epilogue_value(s[e], a.alpha, a.beta, c_in[e], bj[e], a.act);
    if (c_vec_ok && col + 3 < a.N) {          // four outputs in one store
        const int64_t ci = row * a.ldc + col;
        if (a.out_dtype == DT_F32) tile::OutVec<DT_F32>::store4((float*)a.C + ci, o);
        else if (a.out_dtype == DT_BF16) tile::OutVec<DT_BF16>::store4((uint16_t*)a.C + ci, o);
        else tile::OutVec<DT_F16>::store4((uint16_t*)a.C + ci, o);
        return;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (col + e >= a.N) break;
        store_elem(a.C, a.out_dtype, row * a.ldc + col + e, o[e]);
    }
}

}  // namespace

hipError_t launch_tile_split_reduce(const Args& a, int variant, int group_m, const TileSplit& split, hipStream_t stream) {
    if (variant < 0 || variant >= kNum || split.parts <= 1) return hipErrorInvalidValue;
    const int BM = kInfo[variant].BM, BN = kInfo[variant].BN;
    const int tiles_m = (int)((a.M + BM - 1) / BM), tiles_n = (int)((a.N + BN - 1) / BN);
    const int tail = tiles_m * tiles_n - split.first_tile;
    if (tail <= 0) return hipSuccess;
    const dim3 grid((unsigned)tail, (unsigned)(BM * BN / 4 / 256)), block(256);
    const int gm = group_m < 1 ? 1 : group_m;
    const int c_vec_ok = c_rows_take_vec4(a);
#define GEMM_REDUCE_LAUNCH(P)                                                                                       \
    hipLaunchKernelGGL(tile_split_reduce_kernel<P>, grid, block, 0, stream, a, tiles_m, tiles_n, gm, split.first_tile, \
                       split.parts, (const float*)split.partials, BM, BN, c_vec_ok)
    switch (split.parts) {
        case 2: GEMM_REDUCE_LAUNCH(2); break;
        case 3: GEMM_REDUCE_LAUNCH(3); break;
        case 4: GEMM_REDUCE_LAUNCH(4); break;
        case 6: GEMM_REDUCE_LAUNCH(6); break;
        case 8: GEMM_REDUCE_LAUNCH(8); break;
        default: GEMM_REDUCE_LAUNCH(0); break;
    }
#undef GEMM_REDUCE_LAUNCH
    return hipGetLastError();
}

}  // namespace gemm

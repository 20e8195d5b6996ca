// Table of macro-tile variants and the preconditions of the family.
#include "common.hpp"

namespace gemm {

#define GEMM_TILE_VARIANT(IDX, NAME, KIND, BM, BN, BK, WM, WN, NS) \
    hipError_t launch_tile_variant_##IDX(const Args& a, int group_m, hipStream_t stream);
#include "tile_variants.def"
#undef GEMM_TILE_VARIANT

namespace {

typedef hipError_t (*launch_fn)(const Args&, int, hipStream_t);

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

// 16-byte vector loads along the contiguous dimension of each operand, 32-bit byte offsets
// inside a tile, and a 32-bit workgroup count.
bool tile_supports(const Args& a) {
    if (a.dtype != DT_BF16 && a.dtype != DT_F16) return false;
    if (a.M <= 0 || a.N <= 0 || a.K <= 0) return false;
    if (((uintptr_t)a.A & 15) || ((uintptr_t)a.B & 15)) return false;
    if ((a.lda & 7) || (a.ldb & 7)) return false;
    if (a.lda > (1 << 22) || a.ldb > (1 << 22)) return false;
    if (a.K > (1 << 30)) return false;
    // the contiguous dimension of each operand must be whole 16-byte chunks
    if (!a.transA ? (a.K & 7) : (a.M & 7)) return false;
    if (a.transB ? (a.K & 7) : (a.N & 7)) return false;
    const int64_t tiles = ((a.M + 127) / 128) * ((a.N + 127) / 128);
    if (tiles > (int64_t)1 << 30) return false;
    return true;
}

// The direct-to-LDS variants mask lanes with a fixed out-of-range offset of 2 GiB - 16.
bool tile_variant_supports(const Args& a, int variant) {
    if (variant < 0 || variant >= kNum) return false;
    if (kInfo[variant].kind == 0) return true;
    const int64_t a_bytes = ((a.transA ? a.K : a.M) * a.lda) * 2, b_bytes = ((a.transB ? a.N : a.K) * a.ldb) * 2;
    return a_bytes < 0x7ffffff0ll && b_bytes < 0x7ffffff0ll;
}

hipError_t launch_tile(const Args& a, int variant, int group_m, hipStream_t stream) {
    if (variant < 0 || variant >= kNum) return hipErrorInvalidValue;
    return kLaunch[variant](a, group_m < 1 ? 1 : group_m, stream);
}

}  // namespace gemm

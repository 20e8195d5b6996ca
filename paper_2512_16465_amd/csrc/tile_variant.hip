// Instantiates the macro-tile kernel for ONE tile variant; compiled once per variant with
// -DGEMM_TILE_VARIANT_INDEX=<n> so that the variants build in parallel.
#include "tile_kernel.hpp"

#ifndef GEMM_TILE_VARIANT_INDEX
#error "compile with -DGEMM_TILE_VARIANT_INDEX=<n>"
#endif

namespace gemm {

#define GEMM_CAT2(a, b) a##b
#define GEMM_CAT(a, b) GEMM_CAT2(a, b)

#define GEMM_TILE_VARIANT(IDX, NAME, BM, BN, BK, WM, WN)                                         \
    template <int I> struct VariantCfg##IDX { using type = tile::Cfg<BM, BN, BK, WM, WN>; };
#include "tile_variants.def"
#undef GEMM_TILE_VARIANT

hipError_t GEMM_CAT(launch_tile_variant_, GEMM_TILE_VARIANT_INDEX)(const Args& a, int group_m, hipStream_t stream) {
    using C = typename GEMM_CAT(VariantCfg, GEMM_TILE_VARIANT_INDEX)<0>::type;
    return tile::launch_variant<C>(a, group_m, stream);
}

}  // namespace gemm

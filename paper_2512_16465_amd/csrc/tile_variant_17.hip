// Tile variant 17 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 17
#include "tile_variant.inc"

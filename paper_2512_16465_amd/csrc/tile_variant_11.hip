// Tile variant 11 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 11
#include "tile_variant.inc"

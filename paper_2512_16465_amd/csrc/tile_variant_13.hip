// Tile variant 13 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 13
#include "tile_variant.inc"

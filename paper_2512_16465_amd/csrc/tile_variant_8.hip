// Tile variant 8 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 8
#include "tile_variant.inc"

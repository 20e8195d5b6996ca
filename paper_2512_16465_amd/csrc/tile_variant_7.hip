// Tile variant 7 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 7
#include "tile_variant.inc"

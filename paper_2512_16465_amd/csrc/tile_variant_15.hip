// Tile variant 15 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 15
#include "tile_variant.inc"

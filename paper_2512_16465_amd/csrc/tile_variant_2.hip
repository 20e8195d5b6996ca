// Tile variant 2 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 2
#include "tile_variant.inc"

// Tile variant 5 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 5
#include "tile_variant.inc"

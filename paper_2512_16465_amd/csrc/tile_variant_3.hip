// Tile variant 3 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 3
#include "tile_variant.inc"

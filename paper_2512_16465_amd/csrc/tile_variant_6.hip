// Tile variant 6 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 6
#include "tile_variant.inc"

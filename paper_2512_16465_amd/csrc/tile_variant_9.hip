// Tile variant 9 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 9
#include "tile_variant.inc"

// Tile variant 14 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 14
#include "tile_variant.inc"

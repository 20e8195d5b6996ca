// Tile variant 10 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 10
#include "tile_variant.inc"

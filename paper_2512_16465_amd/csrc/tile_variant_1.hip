// Tile variant 1 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 1
#include "tile_variant.inc"

// Tile variant 4 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 4
#include "tile_variant.inc"

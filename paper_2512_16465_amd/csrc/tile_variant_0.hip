// Tile variant 0 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 0
#include "tile_variant.inc"

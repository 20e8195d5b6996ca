// Tile variant 16 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 16
#include "tile_variant.inc"

// Tile variant 12 of tile_variants.def.
#define GEMM_TILE_VARIANT_INDEX 12
#include "tile_variant.inc"

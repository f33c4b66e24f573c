// MFMA tile kernels, f32 inputs, layout rc (A row-major, B column-major).
#define TILE_DT optiml::DT_F32
#define TILE_IS_F32 1
#define TILE_A_KC true
#define TILE_B_KC true
#define TILE_TAG "f32_rc"
#define TILE_SYMBOL kTile_f32_rc
#include "tile_instances.inc"

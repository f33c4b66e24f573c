// MFMA tile kernels, f32 inputs, layout cc (A column-major, B column-major).
#define TILE_DT optiml::DT_F32
#define TILE_IS_F32 1
#define TILE_A_KC false
#define TILE_B_KC true
#define TILE_TAG "f32_cc"
#define TILE_SYMBOL kTile_f32_cc
#include "tile_instances.inc"

// MFMA tile kernels, fp16 inputs, layout cc (A column-major, B column-major).
#define TILE_DT optiml::DT_F16
#define TILE_IS_F32 0
#define TILE_A_KC false
#define TILE_B_KC true
#define TILE_TAG "f16_cc"
#define TILE_SYMBOL kTile_f16_cc
#include "tile_instances.inc"

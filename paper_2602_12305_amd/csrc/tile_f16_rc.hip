// MFMA tile kernels, fp16 inputs, layout rc (A row-major, B column-major).
#define TILE_DT optiml::DT_F16
#define TILE_IS_F32 0
#define TILE_A_KC true
#define TILE_B_KC true
#define TILE_TAG "f16_rc"
#define TILE_SYMBOL kTile_f16_rc
#include "tile_instances.inc"

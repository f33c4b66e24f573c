// MFMA tile kernels, bf16 inputs, layout rc (A row-major, B column-major).
#define TILE_DT optiml::DT_BF16
#define TILE_IS_F32 0
#define TILE_A_KC true
#define TILE_B_KC true
#define TILE_TAG "bf16_rc"
#define TILE_SYMBOL kTile_bf16_rc
#include "tile_instances.inc"

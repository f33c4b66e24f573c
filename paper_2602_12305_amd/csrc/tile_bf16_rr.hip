// MFMA tile kernels, bf16 inputs, layout rr (A row-major, B row-major).
#define TILE_DT optiml::DT_BF16
#define TILE_IS_F32 0
#define TILE_A_KC true
#define TILE_B_KC false
#define TILE_TAG "bf16_rr"
#define TILE_SYMBOL kTile_bf16_rr
#include "tile_instances.inc"

// MFMA tile kernels, fp16 inputs, layout rr (A row-major, B row-major).
#define TILE_DT optiml::DT_F16
#define TILE_IS_F32 0
#define TILE_A_KC true
#define TILE_B_KC false
#define TILE_TAG "f16_rr"
#define TILE_SYMBOL kTile_f16_rr
#include "tile_instances.inc"

// MFMA tile kernels, f32 inputs, layout rr (A row-major, B row-major).
#define TILE_DT optiml::DT_F32
#define TILE_IS_F32 1
#define TILE_A_KC true
#define TILE_B_KC false
#define TILE_TAG "f32_rr"
#define TILE_SYMBOL kTile_f32_rr
#include "tile_instances.inc"

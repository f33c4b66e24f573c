// Ring-of-stages bf16 MFMA tile kernels, A row-major, B row-major.
#define RING_B_KC false
#define RING_TAG "bf16_rr"
#define RING_SYMBOL kRing_bf16_rr
#include "ring_instances.inc"

// Ring-of-stages bf16 MFMA tile kernels, A row-major, B column-major.
#define RING_B_KC true
#define RING_TAG "bf16_rc"
#define RING_SYMBOL kRing_bf16_rc
#include "ring_instances.inc"

// Ring-of-stages fp16 MFMA tile kernels, A row-major, B column-major.
#define RING_B_KC true
#define RING_DT DT_F16
#define RING_TAG "f16_rc"
#define RING_SYMBOL kRing_f16_rc
#include "ring_instances.inc"

// Ring-of-stages fp16 MFMA tile kernels, A row-major, B row-major.
#define RING_B_KC false
#define RING_DT DT_F16
#define RING_TAG "f16_rr"
#define RING_SYMBOL kRing_f16_rr
#include "ring_instances.inc"

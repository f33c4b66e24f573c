// Ring-of-stages MFMA tile kernels for 8-bit E5M2 operands (bf16 result), A row-major, B column-major.
#define RING_B_KC true
#define RING_DT DT_BF8
#define RING_TAG "bf8_rc"
#define RING_SYMBOL kRing_bf8_rc
#define RING_NO_PERSISTENT 1
#include "ring_instances.inc"

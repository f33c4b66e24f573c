// Ring-of-stages MFMA tile kernels for 8-bit E4M3 operands (bf16 result), A row-major, B column-major.
#define RING_B_KC true
#define RING_DT DT_F8
#define RING_TAG "f8_rc"
#define RING_SYMBOL kRing_f8_rc
#define RING_NO_PERSISTENT 1
#include "ring_instances.inc"

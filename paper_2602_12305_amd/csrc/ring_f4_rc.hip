// Ring-of-stages MFMA tile kernels for 4-bit E2M1 operands (bf16 result), A row-major, B column-major,
// two values to a byte along k.
#define RING_B_KC true
#define RING_DT DT_F4
#define RING_TAG "f4_rc"
#define RING_SYMBOL kRing_f4_rc
#define RING_E2M1 1
#include "ring_instances.inc"

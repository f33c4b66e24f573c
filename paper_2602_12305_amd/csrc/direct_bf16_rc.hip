// Direct-to-LDS bf16 MFMA tile kernels, A row-major, B column-major.
#define DIRECT_B_KC true
#define DIRECT_TAG "bf16_rc"
#define DIRECT_SYMBOL kDirect_bf16_rc
#include "direct_instances.inc"

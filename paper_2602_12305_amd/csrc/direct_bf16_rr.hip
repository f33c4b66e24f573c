// Direct-to-LDS bf16 MFMA tile kernels, A row-major, B row-major.
#define DIRECT_B_KC false
#define DIRECT_TAG "bf16_rr"
#define DIRECT_SYMBOL kDirect_bf16_rr
#include "direct_instances.inc"

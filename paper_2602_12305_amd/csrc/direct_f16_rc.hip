// Direct-to-LDS binary16 MFMA tile kernels, A row-major, B column-major.
#define DIRECT_B_KC true
#define DIRECT_DT DT_F16
#define DIRECT_TAG "f16_rc"
#define DIRECT_SYMBOL kDirect_f16_rc
#include "direct_instances.inc"

// Direct-to-LDS binary16 MFMA tile kernels, A row-major, B row-major.
#define DIRECT_B_KC false
#define DIRECT_DT DT_F16
#define DIRECT_TAG "f16_rr"
#define DIRECT_SYMBOL kDirect_f16_rr
#include "direct_instances.inc"

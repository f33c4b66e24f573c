// Ring-of-stages fp32 MFMA tile kernels, A row-major, B column-major.
#define RINGF_B_KC true
#define RINGF_TAG "f32_rc"
#define RINGF_SYMBOL kRing_f32_rc
#include "ringf_instances.inc"

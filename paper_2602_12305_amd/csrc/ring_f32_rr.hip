// Ring-of-stages fp32 MFMA tile kernels, A row-major, B row-major.
#define RINGF_B_KC false
#define RINGF_TAG "f32_rr"
#define RINGF_SYMBOL kRing_f32_rr
#include "ringf_instances.inc"

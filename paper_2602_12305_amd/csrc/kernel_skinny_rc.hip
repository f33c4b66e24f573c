// Table of the streaming kernels for a column-major B; the kernels are in kernel_skinny_rc.hpp.
#include "kernel_skinny_rc.hpp"

namespace optiml {
using namespace skinny_rc;

#define SKRC(DT, TAG, WN, WK, CG)                                                                       \
    {"skinnyrc_" TAG "_wn" #WN "_wk" #WK "_cg" #CG, supports<DT>, launch<DT, WN, WK, CG>, 0, 0,         \
     reinterpret_cast<const void *>(&skinny_rc_kernel<DT, WN, WK, CG>)}
#define SKRC_SET(DT, TAG) SKRC(DT, TAG, 1, 8, 4), SKRC(DT, TAG, 1, 4, 4), SKRC(DT, TAG, 2, 4, 2), SKRC(DT, TAG, 1, 8, 2)

// per dtype the first entry is the dispatcher's choice
const Variant *skinny_rc_variants()
{
    static const Variant v[kNumSkinnyRcVariants] = {SKRC_SET(DT_F32, "f32"), SKRC_SET(DT_BF16, "bf16"), SKRC_SET(DT_F16, "f16"),
                                                    SKRC_SET(DT_F8, "f8")};
    return v;
}

}  // namespace optiml

// Table of the streaming kernels for a column-major B; the kernels are in kernel_skinny_rc.hpp.
#include "kernel_skinny_rc.hpp"

namespace optiml {
using namespace skinny_rc;

#define SKRC(DT, TAG, WN, WK, CG, T)                                                                      \
    {"skinnyrc_" TAG "_wn" #WN "_wk" #WK "_cg" #CG "_t" #T, supports<DT>, launch<DT, WN, WK, CG, T>, 0, 0,  \
     reinterpret_cast<const void *>(&skinny_rc_kernel<DT, WN, WK, CG, T>)}
#define SKRC_SET(DT, TAG) SKRC(DT, TAG, 1, 4, 4, 4), SKRC(DT, TAG, 2, 2, 2, 8), SKRC(DT, TAG, 4, 1, 1, 16), SKRC(DT, TAG, 2, 4, 1, 16)

// per dtype the first entry is the dispatcher's choice
const Variant *skinny_rc_variants()
{
    static const Variant v[kNumSkinnyRcVariants] = {SKRC_SET(DT_F32, "f32"), SKRC_SET(DT_BF16, "bf16"), SKRC_SET(DT_F16, "f16"),
                                                    SKRC_SET(DT_F8, "f8")};
    return v;
}

}  // namespace optiml

// Table of the streaming kernels for a column-major B; the kernels are in kernel_skinny_rc.hpp.
#include "kernel_skinny_rc.hpp"

namespace optiml {
using namespace skinny_rc;

#define SKRC(DT, TAG, WN, WK, CG, T, ROLE)                                                                    \
    {"skinnyrc_" TAG "_wn" #WN "_wk" #WK "_cg" #CG "_t" #T, supports<DT>, launch<DT, WN, WK, CG, T>, 0, 0,  \
     reinterpret_cast<const void *>(&skinny_rc_kernel<DT, WN, WK, CG, T>), nullptr, true, nullptr, FAM_NONE, ROLE}
#define SKRC_DMA(DT, TAG, WK, CG, NS, ROLE)                                                                   \
    {"skinnyrc_" TAG "_dma_wk" #WK "_cg" #CG "_ns" #NS, supports_dma<DT>, launch_dma<DT, WK, CG, NS>, 0, 0,  \
     reinterpret_cast<const void *>(&skinny_rc_dma_kernel<DT, WK, CG, NS>), nullptr, true, nullptr, FAM_NONE, ROLE}
#define SKRC_SET(DT, TAG)                                                                                 \
    SKRC_DMA(DT, TAG, 4, 4, 2, ROLE_STREAM_DEFAULT), SKRC(DT, TAG, 1, 4, 4, 4, ROLE_STREAM_REGS),         \
    SKRC_DMA(DT, TAG, 4, 2, 3, ROLE_STREAM_NARROW), SKRC_DMA(DT, TAG, 2, 4, 4, ROLE_NONE)

// per dtype the first entry is the dispatcher's choice: staged through LDS by DMA, four waves, four column groups,
// two stages (160 KiB of LDS); the second is the register-only kernel (also the fallback when the 32-bit lane
// offsets of the DMA kernel do not reach)
const Variant *skinny_rc_variants()
{
    static const Variant v[kNumSkinnyRcVariants] = {SKRC_SET(DT_F32, "f32"), SKRC_SET(DT_BF16, "bf16"), SKRC_SET(DT_F16, "f16"),
                                                    SKRC_SET(DT_F8, "f8"), SKRC_SET(DT_F4, "f4"), SKRC_SET(DT_BF8, "bf8")};
    return v;
}

}  // namespace optiml

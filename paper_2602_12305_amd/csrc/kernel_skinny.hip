// Table of the streaming (skinny-M) kernel variants; the kernels are in kernel_skinny.hpp.
#include "kernel_skinny.hpp"

namespace optiml {
using namespace skinny;

#define SKINNY_IL(WN, WK, CG, NT, SPLIT, ROLE)                                                     \
    {"skinny_f32_wn" #WN "_wk" #WK "_cg" #CG "_nt" #NT "_split" #SPLIT "_il", skinny_supports,     \
     skinny_launch<WN, WK, CG, NT, SPLIT, true>, 0, 0,                                             \
     reinterpret_cast<const void *>(&skinny_kernel<WN, WK, CG, NT, true>), nullptr, true, nullptr, FAM_NONE, ROLE}
#define SKINNY(WN, WK, CG, NT, SPLIT, ROLE)                                                \
    {"skinny_f32_wn" #WN "_wk" #WK "_cg" #CG "_nt" #NT "_split" #SPLIT, skinny_supports, \
     skinny_launch<WN, WK, CG, NT, SPLIT>, 0, 0, reinterpret_cast<const void *>(&skinny_kernel<WN, WK, CG, NT>), nullptr, true, \
     nullptr, FAM_NONE, ROLE}

#define SKINNY_DMA(WK, CG, NS, NT, ROLE)                                                                   \
    {"skinny_f32_dma_wk" #WK "_cg" #CG "_ns" #NS "_nt" #NT, skinny_dma_supports, skinny_dma_launch<WK, CG, NS, NT>, 0, 0, \
     reinterpret_cast<const void *>(&skinny_dma_kernel<WK, CG, NS, NT>), nullptr, true, nullptr, FAM_NONE, ROLE}

// The dispatcher finds its entries by role, not by position: up to 16 rows the four-wave kernel that
// stages B through LDS by direct loads (128 columns a workgroup, B read with the non-temporal
// hint), more blocks of rows the same without the hint, and problems that would launch too few
// workgroups (or few blocks of rows over a small B) the one with 64 columns a workgroup, eight
// waves deep in k when B is smaller still.  The
// register-staged kernels stay for the sweep and the search (the eight-wave interleaved one is
// the point the tree search of paper_2602_12305_amd/search.py found on the 16 x 16384 x 16384 case).
const Variant *skinny_variants()
{
    static const Variant v[kNumSkinnyVariants] = {
        SKINNY_IL(1, 8, 2, 1, 0, ROLE_NONE), SKINNY(1, 4, 2, 0, 0, ROLE_NONE),
        SKINNY(1, 8, 2, 1, 0, ROLE_NONE),  SKINNY(1, 4, 2, 1, 0, ROLE_NONE),
        SKINNY(4, 1, 1, 1, 0, ROLE_NONE),  SKINNY(2, 4, 1, 1, 0, ROLE_NONE),
        SKINNY(1, 8, 1, 1, 1, ROLE_NONE),  SKINNY(1, 8, 1, 0, 1, ROLE_NONE),
        SKINNY(1, 16, 1, 1, 1, ROLE_NONE), SKINNY(1, 4, 1, 1, 2, ROLE_NONE),
        SKINNY(4, 4, 1, 1, 0, ROLE_NONE),  SKINNY(2, 2, 2, 1, 0, ROLE_NONE),
        SKINNY(1, 8, 2, 1, 2, ROLE_NONE),  SKINNY_IL(1, 8, 2, 1, 2, ROLE_NONE),
        SKINNY_IL(1, 4, 1, 1, 0, ROLE_NONE), SKINNY_IL(1, 8, 1, 1, 1, ROLE_NONE),
        SKINNY_DMA(4, 2, 2, 1, ROLE_STREAM_DEFAULT), SKINNY_DMA(8, 2, 2, 1, ROLE_NONE), SKINNY_DMA(4, 2, 4, 1, ROLE_NONE), SKINNY_DMA(4, 1, 4, 1, ROLE_NONE),
        SKINNY_DMA(4, 2, 2, 0, ROLE_STREAM_ROWS), SKINNY_DMA(4, 2, 4, 0, ROLE_NONE), SKINNY_DMA(4, 1, 4, 0, ROLE_STREAM_NARROW), SKINNY_DMA(8, 1, 2, 1, ROLE_STREAM_SMALL),
    };
    return v;
}

}  // namespace optiml

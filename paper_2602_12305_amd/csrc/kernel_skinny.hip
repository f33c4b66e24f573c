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

// The dispatcher finds its entries by role, not by position.  The first entry is its choice for at most 16 rows (eight waves deep in k, one
// workgroup per CU: the point the tree search of paper_2602_12305_amd/search.py found on the
// 16 x 16384 x 16384 case, here with the waves interleaved in k), the second (B loaded without the non-temporal hint) its choice for small
// problems of more rows; the rest are there for the sweep.
const Variant *skinny_variants()
{
    static const Variant v[kNumSkinnyVariants] = {
        SKINNY_IL(1, 8, 2, 1, 0, ROLE_STREAM_DEFAULT), SKINNY(1, 4, 2, 0, 0, ROLE_STREAM_ROWS),
        SKINNY(1, 8, 2, 1, 0, ROLE_NONE),  SKINNY(1, 4, 2, 1, 0, ROLE_NONE),
        SKINNY(4, 1, 1, 1, 0, ROLE_NONE),  SKINNY(2, 4, 1, 1, 0, ROLE_NONE),
        SKINNY(1, 8, 1, 1, 1, ROLE_NONE),  SKINNY(1, 8, 1, 0, 1, ROLE_STREAM_UNSPLIT),
        SKINNY(1, 16, 1, 1, 1, ROLE_NONE), SKINNY(1, 4, 1, 1, 2, ROLE_NONE),
        SKINNY(4, 4, 1, 1, 0, ROLE_NONE),  SKINNY(2, 2, 2, 1, 0, ROLE_NONE),
        SKINNY(1, 8, 2, 1, 2, ROLE_NONE),  SKINNY_IL(1, 8, 2, 1, 2, ROLE_NONE),
        SKINNY_IL(1, 4, 1, 1, 0, ROLE_STREAM_NARROW), SKINNY_IL(1, 8, 1, 1, 1, ROLE_NONE),
    };
    return v;
}

}  // namespace optiml

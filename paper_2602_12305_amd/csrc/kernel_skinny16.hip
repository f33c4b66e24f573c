// Table of the 16-bit streaming (skinny-M) kernel variants; the kernels are in kernel_skinny16.hpp.
#include "kernel_skinny16.hpp"

namespace optiml {
using namespace skinny16;

#define SK16(DT, TAG, WN, WK, CG, NT, SPLIT, IL, ILTAG, ROLE)                                                     \
    {"skinny_" TAG "_wn" #WN "_wk" #WK "_cg" #CG "_nt" #NT "_split" #SPLIT ILTAG, supports<DT>,              \
     launch<DT, WN, WK, CG, NT, SPLIT, IL>, 0, 0,                                                             \
     reinterpret_cast<const void *>(&skinny16_kernel<DT, WN, WK, CG, NT, IL>), nullptr, true, nullptr, FAM_NONE, ROLE}
#define SK16_SET(DT, TAG)                                                                                     \
    SK16(DT, TAG, 1, 4, 2, 1, 0, true, "_il", ROLE_STREAM_DEFAULT), SK16(DT, TAG, 1, 8, 1, 0, 0, true, "_il", ROLE_STREAM_ROWS), \
    SK16(DT, TAG, 1, 8, 1, 1, 0, true, "_il", ROLE_NONE), SK16(DT, TAG, 1, 4, 1, 1, 0, true, "_il", ROLE_STREAM_NARROW),  \
    SK16(DT, TAG, 1, 8, 1, 1, 0, false, "", ROLE_NONE),   SK16(DT, TAG, 2, 4, 1, 1, 0, false, "", ROLE_NONE),            \
    SK16(DT, TAG, 4, 1, 1, 1, 0, false, "", ROLE_NONE),   SK16(DT, TAG, 1, 4, 2, 1, 2, true, "_il", ROLE_NONE)

// Per dtype, the first entry is the dispatcher's choice: four waves interleaved in k, 512 bytes of
// each row of B per workgroup (measured best at 16 x 16384 x 16384 and for 32 and 64 rows; within
// 2 % of the best elsewhere); the rest are there for the sweep.
const Variant *skinny16_variants()
{
    static const Variant v[kNumSkinny16Variants] = {SK16_SET(DT_BF16, "bf16"), SK16_SET(DT_F16, "f16")};
    return v;
}

}  // namespace optiml

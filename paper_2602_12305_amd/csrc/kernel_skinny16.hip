// Table of the 16-bit streaming (skinny-M) kernel variants; the kernels are in kernel_skinny16.hpp.
#include "kernel_skinny16.hpp"

namespace optiml {
using namespace skinny16;

#define SK16(DT, TAG, WN, WK, CG, NT, SPLIT, IL, ILTAG, ROLE)                                                     \
    {"skinny_" TAG "_wn" #WN "_wk" #WK "_cg" #CG "_nt" #NT "_split" #SPLIT ILTAG, supports<DT>,              \
     launch<DT, WN, WK, CG, NT, SPLIT, IL>, 0, 0,                                                             \
     reinterpret_cast<const void *>(&skinny16_kernel<DT, WN, WK, CG, NT, IL>), nullptr, true, nullptr, FAM_NONE, ROLE}
#define SK16_SET(DT, TAG)                                                                                     \
    SK16(DT, TAG, 1, 4, 2, 1, 0, true, "_il", ROLE_STREAM_DEFAULT), SK16(DT, TAG, 1, 8, 1, 0, 0, true, "_il", ROLE_NONE), \
    SK16(DT, TAG, 1, 8, 1, 1, 0, true, "_il", ROLE_NONE), SK16(DT, TAG, 1, 4, 1, 1, 0, true, "_il", ROLE_NONE),  \
    SK16(DT, TAG, 1, 8, 1, 1, 0, false, "", ROLE_NONE),   SK16(DT, TAG, 2, 4, 1, 1, 0, false, "", ROLE_NONE),            \
    SK16(DT, TAG, 4, 1, 1, 1, 0, false, "", ROLE_NONE),   SK16(DT, TAG, 1, 4, 2, 1, 2, true, "_il", ROLE_NONE)

#define SK16_DMA(DT, TAG, WK, CG, NS, NT, ROLE)                                                                \
    {"skinny_" TAG "_dma_wk" #WK "_cg" #CG "_ns" #NS "_nt" #NT, dma_supports<DT>, dma_launch<DT, WK, CG, NS, NT>, 0, 0, \
     reinterpret_cast<const void *>(&skinny16_dma_kernel<DT, WK, CG, NS, NT>), nullptr, true, nullptr, FAM_NONE, ROLE}
#define SK16_DMA_SET(DT, TAG)                                                                                  \
    SK16_DMA(DT, TAG, 4, 2, 2, 1, ROLE_NONE), SK16_DMA(DT, TAG, 4, 2, 2, 0, ROLE_STREAM_ROWS), SK16_DMA(DT, TAG, 4, 1, 4, 0, ROLE_STREAM_NARROW), \
    SK16_DMA(DT, TAG, 4, 1, 4, 1, ROLE_NONE), SK16_DMA(DT, TAG, 8, 1, 2, 1, ROLE_STREAM_SMALL), SK16_DMA(DT, TAG, 8, 2, 2, 1, ROLE_NONE)

// The dispatcher finds its entries by role.  A large B under up to 16 rows keeps the register-staged
// kernel, four waves interleaved in k and 512 bytes of each row of B per workgroup (16 x 16384 x 16384:
// 85.4 us against 86.3 us for the kernel that stages B through LDS by direct loads).  The direct-load
// kernels, four waves deep in k, take the rest: 256 columns a workgroup without the non-temporal hint
// under more blocks of rows (32 x 16384 x 16384: 102 against 127 us), 128 columns a workgroup for every
// smaller B (16 x 8192 x 8192: 27.5 against 30.3 us, 16 x 4096 x 4096: 12.7 against 15.8 us, 64 x 8192 x
// 8192: 35.7 against 42.6 us), eight waves deep in k for a B of a few MiB.  The others are there for the
// sweep and the search.
const Variant *skinny16_variants()
{
    static const Variant v[kNumSkinny16Variants] = {SK16_SET(DT_BF16, "bf16"), SK16_DMA_SET(DT_BF16, "bf16"), SK16_SET(DT_F16, "f16"), SK16_DMA_SET(DT_F16, "f16")};
    return v;
}

}  // namespace optiml

// Matrix-pipe rate probe: what the MFMA units of this board sustain on operands of a given value
// distribution with no global-memory traffic at all - the measured counterpart of the published
// peak, as the plain copy kernel is for the HBM figure.  The paper scores kernels by "speed of
// light" percentages (section 3.2, profiling signals); on a power-limited board the reachable
// ceiling depends on how much the operand bits toggle (all-zero operands run near the clock limit,
// normally distributed ones well below) and on what else draws power next to the matrix pipe, and
// this probe measures both.
//
// One workgroup of four waves per compute unit, one wave per SIMD; `iters` rounds of sixteen
// 32x32x16 matrix instructions on sixteen independent accumulators.
//   lds_reads == 0: a lane reads eight 16-byte operand fragments once and rotates them after each
//     round so that both operands keep changing (the first operand held over four instructions,
//     as the tile kernels do): registers only.
//   lds_reads == 8, 12, 16: the operands of every k-step come from LDS (64 KiB filled once from
//     `operands`, 128-bit conflict-free reads), in the ratio of a 128x128, 128x64 or 64x64 wave
//     tile: TM + TN fragment reads for TM x TN instructions.
// The sum of the accumulators goes to `sink` so that nothing is optimised away.
#include "../../include/optiml.h"
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

template <int DT, int TM, int TN>
__global__ __launch_bounds__(256) void mfma_probe_kernel(const uintx4 *__restrict__ operands, float *__restrict__ sink, int iters)
{
    __shared__ __attribute__((aligned(16))) uintx4 lds[TM == 0 ? 1 : 4096];
    const int tid = threadIdx.x, lane = tid & 63;
    const size_t t = (size_t)blockIdx.x * 256 + tid;
    floatx16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    if constexpr (TM == 0) {
        uintx4 fa[4], fb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[i] = operands[t * 8 + i];
            fb[i] = operands[t * 8 + 4 + i];
        }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j * 4 + i] = mfma_32x32x16<DT>(fb[j], fa[i], acc[j * 4 + i]);
            const uintx4 first = fa[0];
            fa[0] = fa[1]; fa[1] = fa[2]; fa[2] = fa[3]; fa[3] = fb[0];
            fb[0] = fb[1]; fb[1] = fb[2]; fb[2] = fb[3]; fb[3] = first;
        }
    } else {
        for (int i = tid; i < 4096; i += 256) lds[i] = operands[(size_t)blockIdx.x * 4096 + i];
        __syncthreads();
        constexpr int KS = 16 / (TM * TN);          // k-steps per round of sixteen instructions
        int slot = 0;                               // 64 fragments of 64 lanes x 16 bytes, walked in turn
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                uintx4 a[TM], b[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) a[i] = lds[((slot + i) & 63) * 64 + lane];
#pragma unroll
                for (int j = 0; j < TN; ++j) b[j] = lds[((slot + TM + j) & 63) * 64 + lane];
                slot = (slot + TM + TN) & 63;
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int q = (ks * TM * TN + j * TM + i) & 15;
                        acc[q] = mfma_32x32x16<DT>(b[j], a[i], acc[q]);
                    }
            }
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[t] = s;
}

template <int DT>
void launch_probe(int lds_reads, unsigned groups, hipStream_t s, const uintx4 *operands, float *sink, int iters)
{
    if (lds_reads == 0) hipLaunchKernelGGL((mfma_probe_kernel<DT, 0, 0>), dim3(groups), dim3(256), 0, s, operands, sink, iters);
    else if (lds_reads == 8) hipLaunchKernelGGL((mfma_probe_kernel<DT, 4, 4>), dim3(groups), dim3(256), 0, s, operands, sink, iters);
    else if (lds_reads == 12) hipLaunchKernelGGL((mfma_probe_kernel<DT, 4, 2>), dim3(groups), dim3(256), 0, s, operands, sink, iters);
    else hipLaunchKernelGGL((mfma_probe_kernel<DT, 2, 2>), dim3(groups), dim3(256), 0, s, operands, sink, iters);
}

}  // namespace
}  // namespace optiml

extern "C" int optiml_mfma_probe(const void *operands, int64_t operand_bytes, float *sink, int64_t sink_floats,
                                 int64_t iters, int dtype, int lds_reads, double *flops, void *stream)
{
    using namespace optiml;
    if (iters < 0 || iters > 0x7fffffffLL || (dtype != DT_BF16 && dtype != DT_F16)) return OPTIML_ERR_INVALID_ARG;
    if (lds_reads != 0 && lds_reads != 8 && lds_reads != 12 && lds_reads != 16) return OPTIML_ERR_INVALID_ARG;
    if (!operands || !sink || (reinterpret_cast<uintptr_t>(operands) & 15u)) return OPTIML_ERR_INVALID_ARG;
    const int64_t groups = compute_units();
    if (operand_bytes < groups * 65536 || sink_floats < groups * 256) return OPTIML_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == DT_F16) launch_probe<DT_F16>(lds_reads, (unsigned)groups, s, static_cast<const uintx4 *>(operands), sink, (int)iters);
    else launch_probe<DT_BF16>(lds_reads, (unsigned)groups, s, static_cast<const uintx4 *>(operands), sink, (int)iters);
    if (flops) *flops = (double)groups * 4.0 * (double)iters * 16.0 * 32768.0;
    return hipGetLastError() == hipSuccess ? OPTIML_OK : OPTIML_ERR_HIP;
}

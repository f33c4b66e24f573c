// Matrix-pipe rate probe: what the MFMA units of this board sustain on operands of a given value
// distribution with no memory traffic at all - the measured counterpart of the published peak,
// as the plain copy kernel is for the HBM figure.  The paper scores kernels by "speed of light"
// percentages (section 3.2, profiling signals); on a power-limited board the reachable ceiling
// depends on how much the operand bits toggle (all-zero operands run near the clock limit,
// normally distributed ones well below), and this probe measures that ceiling.
//
// One workgroup of four waves per compute unit, one wave per SIMD.  A lane reads eight 16-byte
// operand fragments once, then issues `iters` rounds of sixteen 32x32x16 matrix instructions on
// sixteen independent accumulators (the first operand held over four instructions, as the tile
// kernels do) and rotates the eight fragments after each round so that both operands keep
// changing.  The sum of the accumulators goes to `sink` so that nothing is optimised away.
#include "../../include/optiml.h"
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

template <int DT>
__global__ __launch_bounds__(256) void mfma_probe_kernel(const uintx4 *__restrict__ operands, float *__restrict__ sink, int iters)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    uintx4 fa[4], fb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        fa[i] = operands[t * 8 + i];
        fb[i] = operands[t * 8 + 4 + i];
    }
    floatx16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[j * 4 + i] = mfma_32x32x16<DT>(fb[j], fa[i], acc[j * 4 + i]);
        const uintx4 first = fa[0];
        fa[0] = fa[1]; fa[1] = fa[2]; fa[2] = fa[3]; fa[3] = fb[0];
        fb[0] = fb[1]; fb[1] = fb[2]; fb[2] = fb[3]; fb[3] = first;
    }
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    sink[t] = s;
}

}  // namespace
}  // namespace optiml

extern "C" int optiml_mfma_probe(const void *operands, int64_t operand_bytes, float *sink, int64_t sink_floats,
                                 int64_t iters, int dtype, double *flops, void *stream)
{
    using namespace optiml;
    if (iters < 0 || iters > 0x7fffffffLL || (dtype != DT_BF16 && dtype != DT_F16)) return OPTIML_ERR_INVALID_ARG;
    if (!operands || !sink || (reinterpret_cast<uintptr_t>(operands) & 15u)) return OPTIML_ERR_INVALID_ARG;
    const int64_t groups = compute_units();
    if (operand_bytes < groups * 256 * 128 || sink_floats < groups * 256) return OPTIML_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == DT_F16)
        hipLaunchKernelGGL(mfma_probe_kernel<DT_F16>, dim3((unsigned)groups), dim3(256), 0, s,
                           static_cast<const uintx4 *>(operands), sink, (int)iters);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<DT_BF16>, dim3((unsigned)groups), dim3(256), 0, s,
                           static_cast<const uintx4 *>(operands), sink, (int)iters);
    if (flops) *flops = (double)groups * 4.0 * (double)iters * 16.0 * 32768.0;
    return hipGetLastError() == hipSuccess ? OPTIML_OK : OPTIML_ERR_HIP;
}

// Fused epilogue, evaluated in fp32 registers: z = acc + bias[j]; y = act(z);
// one rounding to the output type.  ReLU and the sigmoid follow the paper's
// Table 4 (tasks 10 and 1); SiLU is z*sigmoid(z); GELU is the tanh form, written
// through the identity 0.5*(1 + tanh(u)) = sigmoid(2u) so that large |z| cannot
// produce inf/inf.
#pragma once
#include "common.hpp"

namespace optiml {

__device__ __forceinline__ float sigmoidf_(float x)
{
    // expf(-x) overflows to +inf for x < -88.7 and the quotient is then +0: the right limit
    return 1.0f / (1.0f + expf(-x));
}

__device__ __forceinline__ float apply_act(float z, int act)
{
    switch (act) {
    case ACT_RELU:
        return z > 0.0f ? z : 0.0f;
    case ACT_SILU:
        return z * sigmoidf_(z);
    case ACT_GELU_TANH: {
        const float c2 = 1.5957691216057308f;   // 2*sqrt(2/pi)
        const float u2 = c2 * fmaf(0.044715f * z * z, z, z);
        return z * sigmoidf_(u2);
    }
    default:
        return z;
    }
}

// fp32 -> bf16 bits, round to nearest even; NaN stays a (quiet) NaN
__device__ __forceinline__ unsigned short f32_to_bf16(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u)
        return (unsigned short)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

__device__ __forceinline__ float bf16_to_f32(unsigned short b)
{
    return __uint_as_float(((unsigned int)b) << 16);
}

}  // namespace optiml

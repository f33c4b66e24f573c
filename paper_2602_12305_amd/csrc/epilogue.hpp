// Fused epilogue, evaluated in fp32 registers: z = acc + bias[j]; y = act(z);
// one rounding to the output type.  ReLU and the sigmoid follow the paper's
// Table 4 (tasks 10 and 1); SiLU is z*sigmoid(z); GELU is the tanh form, written
// through the identity 0.5*(1 + tanh(u)) = sigmoid(2u) so that large |z| cannot
// produce inf/inf.
#pragma once
#include <type_traits>

#include "common.hpp"

namespace optiml {

// exp(-x) to about 2 ulp from the hardware base-2 exponential: the product -x*log2(e) is
// formed with its rounding error (fma) and the error is applied as a first-order correction.
// Saturates to +inf / 0 outside the fp32 range, which is what the sigmoid below wants.
__device__ __forceinline__ float exp_neg(float x)
{
    const float l2e_hi = -1.44269502162933349609375f;     // -log2(e) rounded to fp32
    const float l2e_lo = -1.925963033500011e-08f;          // -(log2(e) - fp32(log2(e)))
    const float t = x * l2e_hi;
    float r = fmaf(x, l2e_hi, -t) + x * l2e_lo;            // what the rounded product lost
    r = __builtin_isinf(t) ? 0.0f : r;                     // infinite x (or product): inf - inf above
    const float p = __builtin_amdgcn_exp2f(t);
    return p * fmaf(r, 0.693147180559945f, 1.0f);          // 2^(t+r) = 2^t (1 + r ln 2 + ...); inf stays inf
}

__device__ __forceinline__ float sigmoidf_(float x)
{
    // exp(-x) overflows to +inf for x < -88.7 and the reciprocal is then +0: the right limit.
    // v_rcp_f32 is accurate to 1 ulp.
    return __builtin_amdgcn_rcpf(1.0f + exp_neg(x));
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

// The same activations for results that are rounded to bf16 or fp16 (relative step 2^-8 / 2^-11): the
// exponential is the bare v_exp_f32 of -x*log2(e), whose argument rounding costs at most
// 6e-8*|x| of relative error, orders below either output format's resolution.
__device__ __forceinline__ float sigmoid_bf16out(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x * -1.44269502162933349609375f));
}

__device__ __forceinline__ float apply_act_bf16out(float z, int act)
{
    switch (act) {
    case ACT_RELU:
        return z > 0.0f ? z : 0.0f;
    case ACT_SILU:
        return z * sigmoid_bf16out(z);
    case ACT_GELU_TANH:
        return z * sigmoid_bf16out(1.5957691216057308f * fmaf(0.044715f * z * z, z, z));
    default:
        return z;
    }
}

// Calls f(std::integral_constant<int, ACT>{}) with the run-time activation code turned into a
// compile-time constant.  The tile kernels wrap their whole epilogue in this: a switch per
// output element compiles to a compare-and-branch chain per element (measured: 6.6 us per
// 256x256 tile, more than the arithmetic), one switch per tile costs nothing.
template <class F>
__device__ __forceinline__ void dispatch_act(int act, F &&f)
{
    switch (act) {
    case ACT_RELU: f(std::integral_constant<int, ACT_RELU>{}); break;
    case ACT_SILU: f(std::integral_constant<int, ACT_SILU>{}); break;
    case ACT_GELU_TANH: f(std::integral_constant<int, ACT_GELU_TANH>{}); break;
    default: f(std::integral_constant<int, ACT_NONE>{}); break;
    }
}

// One 32x32x64 matrix instruction on E4M3 (DT_F8, format code 0) or E5M2 (DT_BF8, format code 1) operands given
// as two 16-byte halves each (the scale operands of the builtin are zero: the unscaled instruction).  E2M3 (DT_F6,
// code 2) and E3M2 (DT_BF6, code 3): a lane's operand is 32 values in the first 24 of the 32 bytes, a little-endian
// stream of 6-bit codes; the last two registers are not read.
template <int DT> struct F8F6F4Code { static constexpr int value = DT == DT_BF8 ? 1 : DT == DT_F6 ? 2 : DT == DT_BF6 ? 3 : 0; };
template <int DT, class V4, class ACC> __device__ __forceinline__ ACC mfma_32x32x64_f8(V4 a_lo, V4 a_hi, V4 b_lo, V4 b_hi, ACC c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef int intx8_ __attribute__((ext_vector_type(8)));
    const intx8_ a = intx8_{(int)a_lo[0], (int)a_lo[1], (int)a_lo[2], (int)a_lo[3], (int)a_hi[0], (int)a_hi[1], (int)a_hi[2], (int)a_hi[3]};
    const intx8_ b = intx8_{(int)b_lo[0], (int)b_lo[1], (int)b_lo[2], (int)b_lo[3], (int)b_hi[0], (int)b_hi[1], (int)b_hi[2], (int)b_hi[3]};
    constexpr int F = F8F6F4Code<DT>::value;
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, F, F, 0, 0, 0, 0);
#else
    return c;
#endif
}

// The same with block scales: byte 0 of sa / sb is an E8M0 scale of this lane's row of the first / second operand,
// in lanes 0-31 that of k 0-31 of the 64, in lanes 32-63 that of k 32-63
template <int DT, class V4, class ACC>
__device__ __forceinline__ ACC mfma_32x32x64_f8_scaled(V4 a_lo, V4 a_hi, V4 b_lo, V4 b_hi, ACC c, unsigned sa, unsigned sb)
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef int intx8_ __attribute__((ext_vector_type(8)));
    const intx8_ a = intx8_{(int)a_lo[0], (int)a_lo[1], (int)a_lo[2], (int)a_lo[3], (int)a_hi[0], (int)a_hi[1], (int)a_hi[2], (int)a_hi[3]};
    const intx8_ b = intx8_{(int)b_lo[0], (int)b_lo[1], (int)b_lo[2], (int)b_lo[3], (int)b_hi[0], (int)b_hi[1], (int)b_hi[2], (int)b_hi[3]};
    constexpr int F = F8F6F4Code<DT>::value;
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, F, F, 0, (int)sa, 0, (int)sb);
#else
    return c;
#endif
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

// two fp32 -> two bf16 packed in one dword (lo in bits 0..15), round to nearest even:
// the conversion instruction of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ unsigned int f32x2_to_bf16x2(float lo, float hi)
{
    typedef float floatx2_ __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_ __attribute__((ext_vector_type(2)));
    const bf16x2_ v = __builtin_convertvector(floatx2_{lo, hi}, bf16x2_);
    return __builtin_bit_cast(unsigned int, v);
}

__device__ __forceinline__ float bf16_to_f32(unsigned short b)
{
    return __uint_as_float(((unsigned int)b) << 16);
}

// IEEE binary16 storage: the hardware conversions round to nearest even (the default mode).
__device__ __forceinline__ unsigned int f32x2_to_f16x2(float lo, float hi)
{
    typedef float floatx2_ __attribute__((ext_vector_type(2)));
    typedef _Float16 halfx2_ __attribute__((ext_vector_type(2)));
    const halfx2_ v = __builtin_convertvector(floatx2_{lo, hi}, halfx2_);
    return __builtin_bit_cast(unsigned int, v);
}

__device__ __forceinline__ unsigned short f32_to_f16(float f)
{
    return __builtin_bit_cast(unsigned short, (_Float16)f);
}

__device__ __forceinline__ float f16_to_f32(unsigned short b)
{
    return (float)__builtin_bit_cast(_Float16, b);
}

// OCP 8-bit E4M3 (bias 7, no infinities, NaN = S.1111.111, subnormals f * 2^-9) to fp32, exactly
__device__ __forceinline__ float f8e4m3_to_f32(unsigned char b)
{
    const unsigned e = (b >> 3) & 15u, f = b & 7u;
    float v;
    if (e == 15u && f == 7u) v = __builtin_nanf("");
    else if (e == 0u) v = (float)f * 0.001953125f;                                   // f * 2^-9
    else v = __uint_as_float(((e + 120u) << 23) | (f << 20));                        // 1.f * 2^(e-7)
    return (b & 0x80u) ? -v : v;
}

// OCP 8-bit E5M2 (bias 15, infinities and NaNs as in binary16, of which it is the upper byte) to fp32, exactly
__device__ __forceinline__ float f8e5m2_to_f32(unsigned char b)
{
    const unsigned e = (b >> 2) & 31u, f = b & 3u;
    float v;
    if (e == 31u) v = f ? __builtin_nanf("") : __builtin_inff();
    else if (e == 0u) v = (float)f * 1.52587890625e-05f;                             // f * 2^-16
    else v = __uint_as_float(((e + 112u) << 23) | (f << 21));                        // 1.f * 2^(e-15)
    return (b & 0x80u) ? -v : v;
}

// OCP 4-bit E2M1 (bias 1, no infinities or NaN): sign, then 0, 0.5, 1, 1.5, 2, 3, 4, 6
__device__ __forceinline__ float f4e2m1_to_f32(unsigned int code)
{
    const unsigned e = (code >> 1) & 3u, f = code & 1u;
    const float v = e == 0u ? 0.5f * (float)f : __uint_as_float(((e + 126u) << 23) | (f << 22));   // 1.f * 2^(e-1)
    return (code & 8u) ? -v : v;
}

// OCP 6-bit E2M3 (bias 1) and E3M2 (bias 3), no infinities or NaN; the low six bits of `code`
__device__ __forceinline__ float f6e2m3_to_f32(unsigned int code)
{
    const unsigned e = (code >> 3) & 3u, f = code & 7u;
    const float v = e == 0u ? 0.125f * (float)f : __uint_as_float(((e + 126u) << 23) | (f << 20));   // 1.f * 2^(e-1)
    return (code & 32u) ? -v : v;
}
__device__ __forceinline__ float f6e3m2_to_f32(unsigned int code)
{
    const unsigned e = (code >> 2) & 7u, f = code & 3u;
    const float v = e == 0u ? 0.0625f * (float)f : __uint_as_float(((e + 124u) << 23) | (f << 21));  // 1.f * 2^(e-3)
    return (code & 32u) ? -v : v;
}
// element i of a dense array of 6-bit codes: bits 6 i .. 6 i + 5 of its little-endian bit stream
__device__ __forceinline__ unsigned int six_bit_code(const unsigned char *base, int64_t i)
{
    const int64_t bit = 6 * i, byte = bit >> 3;
    const unsigned sh = (unsigned)(bit & 7);
    unsigned v = base[byte];
    if (sh > 2u) v |= (unsigned)base[byte + 1] << 8;             // the code runs into the next byte
    return (v >> sh) & 63u;
}

// The two 16-bit storage types share every kernel; these pick the conversions and the matrix
// instruction (same shape, same register layout) by the dtype code.
template <int DT> __device__ __forceinline__ unsigned int pack2_16(float lo, float hi)
{
    return DT == DT_F16 ? f32x2_to_f16x2(lo, hi) : f32x2_to_bf16x2(lo, hi);      // DT_F8 stores bf16
}
template <int DT> __device__ __forceinline__ unsigned short to_16(float f)
{
    return DT == DT_F16 ? f32_to_f16(f) : f32_to_bf16(f);
}
template <int DT> __device__ __forceinline__ float from_16(unsigned short b)
{
    return DT == DT_F16 ? f16_to_f32(b) : bf16_to_f32(b);
}
template <int DT, class V4, class ACC> __device__ __forceinline__ ACC mfma_32x32x16(V4 a, V4 b, ACC c)
{
    typedef __bf16 bf16x8_ __attribute__((ext_vector_type(8), unused));
    typedef _Float16 halfx8_ __attribute__((ext_vector_type(8), unused));
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (DT == DT_F4) {
        // 16 bytes per lane = 32 E2M1 values of k = this lane's half of one 64-deep instruction, with both
        // block scales at 2^0 (E8M0 127).  Format code 4 = E2M1 for either operand; only the low four
        // registers of the eight-register operands are read for it.
        typedef int intx8_ __attribute__((ext_vector_type(8)));
        typedef int intx4_ __attribute__((ext_vector_type(4)));
        const intx4_ a4 = __builtin_bit_cast(intx4_, a), b4 = __builtin_bit_cast(intx4_, b);
        const intx8_ a8 = {a4[0], a4[1], a4[2], a4[3], 0, 0, 0, 0}, b8 = {b4[0], b4[1], b4[2], b4[3], 0, 0, 0, 0};
        return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a8, b8, c, 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    } else if constexpr (DT == DT_F8) {
        // 16 bytes per lane = 16 E4M3 values of k: two instructions of 8 each.  Which k a lane's
        // byte stands for only has to agree between the two operands, and it does: both come from
        // the same chunk and byte of their rows.
        typedef long longx2_ __attribute__((ext_vector_type(2)));
        const longx2_ a2 = __builtin_bit_cast(longx2_, a), b2 = __builtin_bit_cast(longx2_, b);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a2[0], b2[0], c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a2[1], b2[1], c, 0, 0, 0);
    } else if constexpr (DT == DT_BF8) {
        // the same with E5M2 operands
        typedef long longx2_ __attribute__((ext_vector_type(2)));
        const longx2_ a2 = __builtin_bit_cast(longx2_, a), b2 = __builtin_bit_cast(longx2_, b);
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf8_bf8(a2[0], b2[0], c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x16_bf8_bf8(a2[1], b2[1], c, 0, 0, 0);
    } else if constexpr (DT == DT_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(halfx8_, a), __builtin_bit_cast(halfx8_, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_, a), __builtin_bit_cast(bf16x8_, b), c, 0, 0, 0);
#else
    return c;
#endif
}

}  // namespace optiml

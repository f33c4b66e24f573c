/*
 * CPU oracle for the fused dense contraction  Y = act(A.B + bias).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is
 * compared against; nothing on the product path may call it, and it shares no
 * code, header, table or constant with the HIP sources.
 *
 * What it computes is the plain definition: the paper's Matrix Multiplication
 * task (Table 4, task 2: A is M x K, B is K x N, C = A x B is M x N) in the
 * row-major indexing of the naive kernel of its matmul case study (appendix
 * "One-task kernel snapshots", first listing: C[row,col] = sum_k A[row,k] *
 * B[k,col]), valid for any M, N as in the second listing's guard.  The fused
 * epilogue adds a length-N bias broadcast down the rows and applies ReLU
 * (Table 4, task 10: max(0,x)), SiLU x*sigmoid(x) with the sigmoid of Table 4,
 * task 1 (1/(1+exp(-x))), or the tanh form of GELU,
 *     0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) )).
 * Bias, SiLU, GELU, bf16 storage and batching are not in the paper; they are
 * the standard definitions named by this repository's benchmark configuration.
 *
 * Arithmetic: the stored fp32 / bf16 / fp16 / 8-bit E4M3 or E5M2 / 6-bit E2M3 or E3M2 / 4-bit E2M1 inputs are widened exactly to fp64; every
 * product of two of them is exact in fp64 (at most 48 significant bits); the
 * sum runs over k ascending in one fp64 accumulator starting from +0.0; the
 * bias is added after the sum; activations use fp64 libm.  The result is kept
 * in fp64 (no rounding to the output type), so it stands for the exact value
 * to within about K * 2^-53 * sum|a b|.
 *
 * Loop nests.  When B's rows are contiguous (B stored K x N) the nest is
 * i, k, j with a row of N accumulators, when B's columns are contiguous
 * (B stored N x K) it is i, j, k.  Either way each output entry receives the
 * same sequence of fp64 operations: acc += a[i,k]*b[k,j] for k = 0..K-1.
 * OpenMP only distributes (batch, row) pairs over threads.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2, ORACLE_F8E4M3 = 3, ORACLE_F4E2M1 = 4, ORACLE_F8E5M2 = 5,
       ORACLE_F6E2M3 = 6, ORACLE_F6E3M2 = 7 };
enum { ORACLE_ACT_NONE = 0, ORACLE_ACT_RELU = 1, ORACLE_ACT_GELU_TANH = 2, ORACLE_ACT_SILU = 3 };
/* bit 0 of layout: B is column-major; bit 1: A is column-major */

/* IEEE 754 binary16 (1 sign, 5 exponent bits with bias 15, 10 fraction bits) to double, exactly:
 * exponent field 0 is a subnormal f * 2^-24, field 31 is infinity (f = 0) or NaN. */
double oracle_f16_to_double(uint16_t h)
{
    const int sign = h >> 15, e = (h >> 10) & 31, f = h & 1023;
    double v;
    if (e == 0)
        v = ldexp((double)f, -24);
    else if (e == 31)
        v = f ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + f), e - 25);
    return sign ? -v : v;
}

/* OCP 8-bit floating point E4M3 (1 sign, 4 exponent bits with bias 7, 3 fraction bits; the "FN"
 * variant: no infinities, the single NaN pattern S.1111.111, largest finite 448) to double,
 * exactly: exponent field 0 is a subnormal f * 2^-9. */
double oracle_f8e4m3_to_double(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 3) & 15, f = b & 7;
    double v;
    if (e == 15 && f == 7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)f, -9);
    else
        v = ldexp((double)(8 + f), e - 10);
    return sign ? -v : v;
}

/* OCP 8-bit floating point E5M2 (1 sign, 5 exponent bits with bias 15, 2 fraction bits: binary16 cut after
 * its second fraction bit) to double, exactly: exponent field 0 is a subnormal f * 2^-16, field 31 is infinity
 * (f = 0) or NaN; largest finite 57344. */
double oracle_f8e5m2_to_double(uint8_t b)
{
    const int sign = b >> 7, e = (b >> 2) & 31, f = b & 3;
    double v;
    if (e == 31)
        v = f ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)f, -16);
    else
        v = ldexp((double)(4 + f), e - 17);
    return sign ? -v : v;
}

/* OCP 4-bit floating point E2M1 (1 sign, 2 exponent bits with bias 1, 1 fraction bit; no infinities, no NaN)
 * to double, exactly: exponent field 0 is a subnormal f * 2^-1, else (2 + f) * 2^(e - 2).  The sixteen codes
 * are 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives.  Only the low four bits of `nibble` are read. */
double oracle_f4e2m1_to_double(uint8_t nibble)
{
    const int sign = (nibble >> 3) & 1, e = (nibble >> 1) & 3, f = nibble & 1;
    const double v = e == 0 ? ldexp((double)f, -1) : ldexp((double)(2 + f), e - 2);
    return sign ? -v : v;
}

/* OCP 6-bit floating point E2M3 (1 sign, 2 exponent bits with bias 1, 3 fraction bits; no infinities, no NaN) to
 * double, exactly: exponent field 0 is a subnormal f * 2^-3, else (8 + f) * 2^(e - 4); largest 7.5.  Only the low
 * six bits of `code` are read. */
double oracle_f6e2m3_to_double(uint8_t code)
{
    const int sign = (code >> 5) & 1, e = (code >> 3) & 3, f = code & 7;
    const double v = e == 0 ? ldexp((double)f, -3) : ldexp((double)(8 + f), e - 4);
    return sign ? -v : v;
}

/* OCP 6-bit floating point E3M2 (1 sign, 3 exponent bits with bias 3, 2 fraction bits; no infinities, no NaN) to
 * double, exactly: exponent field 0 is a subnormal f * 2^-4, else (4 + f) * 2^(e - 5); largest 28. */
double oracle_f6e3m2_to_double(uint8_t code)
{
    const int sign = (code >> 5) & 1, e = (code >> 2) & 7, f = code & 3;
    const double v = e == 0 ? ldexp((double)f, -4) : ldexp((double)(4 + f), e - 5);
    return sign ? -v : v;
}

/* Element idx of an array of 6-bit codes stored densely: the array is one little-endian bit stream (bit b of the
 * stream is bit b % 8 of byte b / 8) and element idx occupies its bits 6 idx .. 6 idx + 5, so four elements fill
 * three bytes. */
static uint8_t six_bits(const void *base, int64_t idx)
{
    const uint8_t *p = (const uint8_t *)base;
    const int64_t bit = 6 * idx;                     /* first bit of the element in the stream */
    const int sh = (int)(bit % 8);
    unsigned v = p[bit / 8] >> sh;                   /* the 8 - sh bits of its first byte from there upwards */
    if (sh > 2)                                      /* fewer than six: the rest are the low bits of the next byte */
        v |= (unsigned)p[bit / 8 + 1] << (8 - sh);
    return (uint8_t)(v & 63u);
}

/* OCP E8M0 block scale (8 exponent bits with bias 127, no sign, no fraction): 2^(e - 127); 255 is NaN. */
double oracle_e8m0_to_double(uint8_t e)
{
    return e == 255 ? NAN : ldexp(1.0, (int)e - 127);
}

static double widen(const void *base, int64_t idx, int dtype)
{
    /* E2M1: two elements to a byte, element idx in the low (idx even) or high (idx odd) four bits */
    if (dtype == ORACLE_F4E2M1)
        return oracle_f4e2m1_to_double((uint8_t)(((const uint8_t *)base)[idx >> 1] >> ((idx & 1) * 4)));
    if (dtype == ORACLE_F6E2M3)
        return oracle_f6e2m3_to_double(six_bits(base, idx));
    if (dtype == ORACLE_F6E3M2)
        return oracle_f6e3m2_to_double(six_bits(base, idx));
    if (dtype == ORACLE_F32)
        return (double)((const float *)base)[idx];
    if (dtype == ORACLE_F16)
        return oracle_f16_to_double(((const uint16_t *)base)[idx]);
    if (dtype == ORACLE_F8E4M3)
        return oracle_f8e4m3_to_double(((const uint8_t *)base)[idx]);
    if (dtype == ORACLE_F8E5M2)
        return oracle_f8e5m2_to_double(((const uint8_t *)base)[idx]);
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

double oracle_act(double z, int act)
{
    switch (act) {
    case ORACLE_ACT_NONE:
        return z;
    case ORACLE_ACT_RELU:
        return z > 0.0 ? z : 0.0;
    case ORACLE_ACT_GELU_TANH: {
        const double pi = 3.14159265358979323846;
        const double c = sqrt(2.0 / pi);
        return 0.5 * z * (1.0 + tanh(c * (z + 0.044715 * z * z * z)));
    }
    case ORACLE_ACT_SILU:
        return z * (1.0 / (1.0 + exp(-z)));
    default:
        return NAN;
    }
}

/* Round a double to the nearest bf16 (ties to even), straight from the fp64
 * value so that no intermediate fp32 rounding can double-round.  Returns the
 * 16 bits.  Overflow gives infinity; NaN gives a quiet NaN. */
uint16_t oracle_bf16_from_double(double x)
{
    if (isnan(x))
        return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0)
        return sign;
    if (isinf(a))
        return sign | 0x7F80;
    int e;
    (void)frexp(a, &e);                /* a = m * 2^e, m in [0.5, 1) */
    int exp_unb = e - 1;               /* a = (2m) * 2^(e-1), 2m in [1, 2) */
    int q;                             /* a is rounded to a multiple of 2^q */
    if (exp_unb < -126)
        q = -126 - 7;                  /* subnormal spacing 2^-133 */
    else
        q = exp_unb - 7;               /* 8 significant bits */
    double scaled = ldexp(a, -q);      /* exact */
    double r = nearbyint(scaled);      /* default rounding mode: nearest even */
    double v = ldexp(r, q);
    if (v >= ldexp(1.0, 128))
        return sign | 0x7F80;
    /* v is exactly representable in bf16, hence in fp32 */
    float f = (float)v;
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    return sign | (uint16_t)(bits >> 16);
}

/* Round a double to the nearest binary16 (ties to even), straight from the fp64 value.
 * 11 significant bits, smallest normal 2^-14, subnormal spacing 2^-24, largest finite 65504;
 * a value that rounds to 2^16 or more gives infinity; NaN gives a quiet NaN. */
uint16_t oracle_f16_from_double(double x)
{
    if (isnan(x))
        return 0x7E00;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (a == 0.0)
        return sign;
    if (isinf(a))
        return sign | 0x7C00;
    int e;
    (void)frexp(a, &e);
    int exp_unb = e - 1;                               /* a in [2^exp_unb, 2^(exp_unb+1)) */
    int q = exp_unb < -14 ? -24 : exp_unb - 10;        /* a is rounded to a multiple of 2^q */
    double r = nearbyint(ldexp(a, -q));                /* default rounding mode: nearest even */
    double v = ldexp(r, q);
    if (v >= 65536.0)
        return sign | 0x7C00;
    if (v < ldexp(1.0, -14))                           /* subnormal (or zero): the count of 2^-24 steps */
        return sign | (uint16_t)r;
    (void)frexp(v, &e);                                /* rounding may have carried into the next binade */
    int field = e - 1 + 15;
    uint16_t frac = (uint16_t)(ldexp(v, 10 - (e - 1)) - 1024.0);
    return sign | (uint16_t)(field << 10) | frac;
}

/*
 * Full evaluation.
 *   A      : A[i,k] at A[b*strideA + i*lda + k]   (A row-major)  or  [.. + k*lda + i] (column-major)
 *   B      : B[k,j] at B[b*strideB + k*ldb + j]   (B row-major)  or  [.. + j*ldb + k] (column-major)
 *   bias   : bias[j] at bias[b*strideBias + j], fp32, NULL = zeros
 *   Y      : fp64, Y[(b*M + i)*N + j] = act(z)
 *   absden : optional fp64 of the same shape, |bias_j| + sum_k |a_ik b_kj|
 * Returns 0, or -1 on a bad enum / negative size.
 */
int oracle_gemm_epilogue(int64_t batch, int64_t M, int64_t N, int64_t K,
                         const void *A, int64_t lda, int64_t strideA,
                         const void *B, int64_t ldb, int64_t strideB,
                         const float *bias, int64_t strideBias,
                         double *Y, double *absden,
                         int layout, int dtype, int act)
{
    if (batch < 0 || M < 0 || N < 0 || K < 0 || layout < 0 || layout > 3 ||
        (dtype < ORACLE_F32 || dtype > ORACLE_F6E3M2) || act < 0 || act > 3)
        return -1;
    const int a_col = (layout >> 1) & 1, b_col = layout & 1;
    const int64_t rows = batch * M;

#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        double *den = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t bi = 0; bi < rows; ++bi) {
            const int64_t b = bi / M, i = bi % M;
            const int64_t a0 = b * strideA, b0 = b * strideB;
            if (!b_col) {
                for (int64_t j = 0; j < N; ++j) { acc[j] = 0.0; den[j] = 0.0; }
                for (int64_t k = 0; k < K; ++k) {
                    const double a = widen(A, a0 + (a_col ? k * lda + i : i * lda + k), dtype);
                    const int64_t brow = b0 + k * ldb;
                    for (int64_t j = 0; j < N; ++j) {
                        const double p = a * widen(B, brow + j, dtype);
                        acc[j] += p;
                        den[j] += fabs(p);
                    }
                }
            } else {
                for (int64_t j = 0; j < N; ++j) {
                    double s = 0.0, d = 0.0;
                    const int64_t bcol = b0 + j * ldb;
                    for (int64_t k = 0; k < K; ++k) {
                        const double a = widen(A, a0 + (a_col ? k * lda + i : i * lda + k), dtype);
                        const double p = a * widen(B, bcol + k, dtype);
                        s += p;
                        d += fabs(p);
                    }
                    acc[j] = s;
                    den[j] = d;
                }
            }
            for (int64_t j = 0; j < N; ++j) {
                const double bj = bias ? (double)bias[b * strideBias + j] : 0.0;
                const double z = acc[j] + bj;
                Y[bi * N + j] = oracle_act(z, act);
                if (absden)
                    absden[bi * N + j] = den[j] + fabs(bj);
            }
        }
        free(acc);
        free(den);
    }
    return 0;
}

/*
 * Sampled evaluation: the same definition at `count` chosen entries
 * (sb[t], si[t], sj[t]); Y[t] and absden[t] (optional) receive the values.
 */
int oracle_gemm_epilogue_sampled(int64_t count, const int64_t *sb, const int64_t *si, const int64_t *sj,
                                 int64_t batch, int64_t M, int64_t N, int64_t K,
                                 const void *A, int64_t lda, int64_t strideA,
                                 const void *B, int64_t ldb, int64_t strideB,
                                 const float *bias, int64_t strideBias,
                                 double *Y, double *absden,
                                 int layout, int dtype, int act)
{
    if (count < 0 || batch < 0 || M < 0 || N < 0 || K < 0 || layout < 0 || layout > 3 ||
        (dtype < ORACLE_F32 || dtype > ORACLE_F6E3M2) || act < 0 || act > 3)
        return -1;
    for (int64_t t = 0; t < count; ++t)
        if (sb[t] < 0 || sb[t] >= batch || si[t] < 0 || si[t] >= M || sj[t] < 0 || sj[t] >= N)
            return -1;
    const int a_col = (layout >> 1) & 1, b_col = layout & 1;

#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t t = 0; t < count; ++t) {
        const int64_t b = sb[t], i = si[t], j = sj[t];
        const int64_t a0 = b * strideA, b0 = b * strideB;
        double s = 0.0, d = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const double a = widen(A, a0 + (a_col ? k * lda + i : i * lda + k), dtype);
            const double bb = widen(B, b0 + (b_col ? j * ldb + k : k * ldb + j), dtype);
            const double p = a * bb;
            s += p;
            d += fabs(p);
        }
        const double bj = bias ? (double)bias[b * strideBias + j] : 0.0;
        Y[t] = oracle_act(s + bj, act);
        if (absden)
            absden[t] = d + fabs(bj);
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Block-scaled operands (the OCP microscaling formats): every 32 consecutive k of a row of A and of a column
 * of B share one E8M0 scale,
 *     z_ij = bias_j + sum_k (sA[i][k / 32] a_ik) (sB[j][k / 32] b_kj),   y_ij = act(z_ij),
 * with a, b in E4M3, E5M2, E2M3, E3M2 or E2M1 storage (dtype), decoded exactly; a scaled element is a power of two times a
 * short significand, exact in fp64, and so is every product; one fp64 accumulator per output, k ascending,
 * bias after the sum.  scaleA is [M][ceil(K / 32)], scaleB [N][ceil(K / 32)] (row-major bytes); A and B in
 * the layouts of oracle_gemm_epilogue, leading dimensions in elements.  Y fp64 [M][N].
 * Returns 0, or -1 on a bad enum / negative size.
 */
int oracle_gemm_epilogue_mx(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const uint8_t *scaleA,
                            const void *B, int64_t ldb, const uint8_t *scaleB, const float *bias, double *Y,
                            int layout, int dtype, int act)
{
    if (M < 0 || N < 0 || K < 0 || layout < 0 || layout > 3 || (dtype < ORACLE_F8E4M3 || dtype > ORACLE_F6E3M2) ||
        act < 0 || act > 3)
        return -1;
    const int a_col = (layout >> 1) & 1, b_col = layout & 1;
    const int64_t blocks = (K + 31) / 32;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const double a = oracle_e8m0_to_double(scaleA[i * blocks + k / 32]) * widen(A, a_col ? k * lda + i : i * lda + k, dtype);
                const double b = oracle_e8m0_to_double(scaleB[j * blocks + k / 32]) * widen(B, b_col ? j * ldb + k : k * ldb + j, dtype);
                s += a * b;
            }
            Y[i * N + j] = oracle_act(s + (bias ? (double)bias[j] : 0.0), act);
        }
    return 0;
}

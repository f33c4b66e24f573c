/*
 * CPU oracle for multi-head self-attention (paper Table 4, task 6): for query, key and value
 * matrices Q, K, V of N rows and d_model columns (row-major, one sequence per batch entry) and h
 * heads of width d_k = d_model / h,
 *
 *     head_i = softmax( Q_i K_i^T / sqrt(d_k) ) V_i,     MultiHead = Concat(head_1 .. head_h),
 *
 * where Q_i, K_i, V_i are columns [i d_k, (i+1) d_k) of Q, K, V and the softmax runs over the
 * keys of one query.  No projections, no mask (the task names none).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is compared
 * against; nothing on the product path may call it, and it shares no code, header, table
 * or constant with the HIP sources.
 *
 * Arithmetic: inputs (fp32, or bf16 / binary16 widened exactly) in fp64.  Per (batch, head, query): the
 * scores s_n = (sum_c q_c k_nc) / sqrt(d_k) over keys n ascending, each dot product over c
 * ascending (products exact in fp64); the maximum score; weights exp(s_n - max); their sum;
 * then for every output column the sum over keys n ascending of weight_n * v_nc, divided by the
 * weight sum.  Kept in fp64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

double oracle_f16_to_double(uint16_t h);      /* oracle_gemm.c */

/* dtype 0: fp32; 1: bf16 bit patterns; 2: IEEE binary16 bit patterns */
static double widen_a(const void *base, int64_t idx, int dtype)
{
    if (dtype == 0) return (double)((const float *)base)[idx];
    if (dtype == 2) return oracle_f16_to_double(((const uint16_t *)base)[idx]);
    uint32_t bits = (uint32_t)((const uint16_t *)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

/* out[b][n][c], fp64, same shape as the inputs; returns 0, or -1 on bad arguments / no memory */
int oracle_mhsa(int64_t batch, int64_t N, int64_t d_model, int64_t heads, const void *Q, const void *K, const void *V,
                int dtype, double *out)
{
    if (batch < 0 || N < 0 || d_model < 1 || heads < 1 || d_model % heads != 0 || dtype < 0 || dtype > 2) return -1;
    const int64_t dk = d_model / heads;
    const double scale = 1.0 / sqrt((double)dk);
    int failed = 0;
#pragma omp parallel
    {
        double *w = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        if (!w) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(static)
        for (int64_t b = 0; b < batch; ++b)
            for (int64_t h = 0; h < heads; ++h) {
                if (!w) continue;
                const int64_t base = b * N * d_model + h * dk;
                for (int64_t i = 0; i < N; ++i) {
                    double mx = -INFINITY;
                    for (int64_t n = 0; n < N; ++n) {
                        double s = 0.0;
                        for (int64_t c = 0; c < dk; ++c)
                            s += widen_a(Q, base + i * d_model + c, dtype) * widen_a(K, base + n * d_model + c, dtype);
                        w[n] = s * scale;
                        mx = w[n] > mx ? w[n] : mx;
                    }
                    double sum = 0.0;
                    for (int64_t n = 0; n < N; ++n) {
                        w[n] = exp(w[n] - mx);
                        sum += w[n];
                    }
                    for (int64_t c = 0; c < dk; ++c) {
                        double o = 0.0;
                        for (int64_t n = 0; n < N; ++n) o += w[n] * widen_a(V, base + n * d_model + c, dtype);
                        out[base + i * d_model + c] = o / sum;
                    }
                }
            }
        free(w);
    }
    return failed ? -1 : 0;
}

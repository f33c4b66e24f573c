/*
 * CPU oracle for the bandwidth-bound siblings of the contraction, all on fp32 arrays:
 *   sigmoid  (paper Table 4, task 1):   y_i = 1 / (1 + exp(-x_i))
 *   ReLU     (Table 4, task 10):        y_i = max(0, x_i)
 *   sum      (Table 4, task 14):        s = sum_i x_i
 *   dot      (Table 4, task 15):        s = sum_i x_i * y_i
 *   MSE      (Table 4, task 7):         s = (1/n) sum_i (x_i - y_i)^2
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the GPU library is compared
 * against; nothing on the product path may call it, and it shares no code, header, table
 * or constant with the HIP sources.
 *
 * Arithmetic: inputs are widened exactly to fp64.  Element-wise results are computed with
 * fp64 libm and kept in fp64.  For the reductions every term is formed in fp64 - a product
 * of two fp32 values is exact, a difference of two fp32 values is rounded once (relative
 * 2^-53), its square once more - and the terms are added in index order inside blocks of
 * 65,536 elements, then the block sums in block order: a fixed order whatever the thread
 * count, with error at most (65,536 + n/65,536) * 2^-53 * sum|term| (4e-12 of sum|term|
 * at n = 2^28), five orders below fp32 resolution.  The value is kept in fp64; MSE of an
 * empty array is 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

enum { ORACLE_EW_RELU = 0, ORACLE_EW_SIGMOID = 1 };
enum { ORACLE_RED_SUM = 0, ORACLE_RED_DOT = 1, ORACLE_RED_MSE = 2 };

void oracle_elementwise(int64_t n, const float *x, int op, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        const double v = (double)x[i];
        y[i] = op == ORACLE_EW_RELU ? (v > 0.0 ? v : 0.0) : 1.0 / (1.0 + exp(-v));
    }
}

static double term(const float *x, const float *y, int64_t i, int op)
{
    const double a = (double)x[i];
    if (op == ORACLE_RED_SUM) return a;
    const double b = (double)y[i];
    if (op == ORACLE_RED_DOT) return a * b;
    return (a - b) * (a - b);
}

double oracle_reduce(int64_t n, const float *x, const float *y, int op)
{
    enum { BLOCK = 65536 };
    const int64_t blocks = (n + BLOCK - 1) / BLOCK;
    double *part = (double *)malloc(sizeof(double) * (size_t)(blocks > 0 ? blocks : 1));
    if (!part) return NAN;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < blocks; ++b) {
        const int64_t lo = b * BLOCK, hi = lo + BLOCK < n ? lo + BLOCK : n;
        double s = 0.0;
        for (int64_t i = lo; i < hi; ++i) s += term(x, y, i, op);
        part[b] = s;
    }
    double total = 0.0;
    for (int64_t b = 0; b < blocks; ++b) total += part[b];
    free(part);
    if (op == ORACLE_RED_MSE) total = n > 0 ? total / (double)n : 0.0;
    return total;
}

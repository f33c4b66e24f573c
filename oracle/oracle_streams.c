/*
 * CPU oracle for the bandwidth-bound siblings of the contraction, all on fp32 arrays:
 *   sigmoid  (paper Table 4, task 1):   y_i = 1 / (1 + exp(-x_i))
 *   ReLU     (Table 4, task 10):        y_i = max(0, x_i)
 *   sum      (Table 4, task 14):        s = sum_i x_i
 *   dot      (Table 4, task 15):        s = sum_i x_i * y_i
 *   MSE      (Table 4, task 7):         s = (1/n) sum_i (x_i - y_i)^2
 *   cross-entropy (Table 4, task 17):   L = (1/N) sum_j ( log(sum_k exp(z_jk)) - z_{j, y_j} )
 *                                       for logits Z (N x C, row-major) and labels y_j in [0, C)
 *   LayerNorm (Table 4, task 4):        y = (x - mean) / sqrt(var + eps) over all features of one
 *                                       sample (rows of length L), mean and biased variance of
 *                                       that row; the task states no eps and no scale / shift:
 *                                       eps is an argument, there is no affine part
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
#include <string.h>

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

/*
 * Cross-entropy.  Per row: the maximum m is found first, the sum of exp(z - m) runs over k
 * ascending in fp64, the loss is log(sum) - (z_y - m): the stable form the task prescribes,
 * with the exact difference z_y - m taken first so that large logits cost no accuracy.  Row
 * losses are added in row order inside blocks of 4,096 rows, block sums in block order.  A label
 * outside [0, C) makes the result NaN.  N == 0 gives 0.
 */
double oracle_cross_entropy(int64_t N, int64_t C, const float *z, const int32_t *labels)
{
    enum { BLOCK = 4096 };
    const int64_t blocks = (N + BLOCK - 1) / BLOCK;
    double *part = (double *)malloc(sizeof(double) * (size_t)(blocks > 0 ? blocks : 1));
    if (!part) return NAN;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < blocks; ++b) {
        const int64_t lo = b * BLOCK, hi = lo + BLOCK < N ? lo + BLOCK : N;
        double s = 0.0;
        for (int64_t j = lo; j < hi; ++j) {
            const float *row = z + j * C;
            if (labels[j] < 0 || labels[j] >= C) { s = NAN; continue; }
            double m = (double)row[0];
            for (int64_t k = 1; k < C; ++k) m = (double)row[k] > m ? (double)row[k] : m;
            double e = 0.0;
            for (int64_t k = 0; k < C; ++k) e += exp((double)row[k] - m);
            s += log(e) - ((double)row[labels[j]] - m);
        }
        part[b] = s;
    }
    double total = 0.0;
    for (int64_t b = 0; b < blocks; ++b) total += part[b];
    free(part);
    return N > 0 ? total / (double)N : 0.0;
}

/*
 * The same loss for logits that are already fp64 (the fused contraction + cross-entropy keeps its
 * logits unrounded): identical steps, no conversion.
 */
double oracle_cross_entropy_f64(int64_t N, int64_t C, const double *z, const int32_t *labels)
{
    enum { BLOCK = 4096 };
    const int64_t blocks = (N + BLOCK - 1) / BLOCK;
    double *part = (double *)malloc(sizeof(double) * (size_t)(blocks > 0 ? blocks : 1));
    if (!part) return NAN;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < blocks; ++b) {
        const int64_t lo = b * BLOCK, hi = lo + BLOCK < N ? lo + BLOCK : N;
        double s = 0.0;
        for (int64_t j = lo; j < hi; ++j) {
            const double *row = z + j * C;
            if (labels[j] < 0 || labels[j] >= C) { s = NAN; continue; }
            double m = row[0];
            for (int64_t k = 1; k < C; ++k) m = row[k] > m ? row[k] : m;
            double e = 0.0;
            for (int64_t k = 0; k < C; ++k) e += exp(row[k] - m);
            s += log(e) - (row[labels[j]] - m);
        }
        part[b] = s;
    }
    double total = 0.0;
    for (int64_t b = 0; b < blocks; ++b) total += part[b];
    free(part);
    return N > 0 ? total / (double)N : 0.0;
}

/*
 * The per-row losses of the same cross-entropy on fp64 logits, loss_j = log(sum_k exp(z_jk)) -
 * z_{j, y_j} with the row maximum taken out first (same steps as above, nothing summed over rows):
 * what the fused contraction + cross-entropy is compared with row by row.  A label outside [0, C)
 * gives NaN for that row.
 */
void oracle_cross_entropy_rows_f64(int64_t N, int64_t C, const double *z, const int32_t *labels, double *loss)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < N; ++j) {
        const double *row = z + j * C;
        if (labels[j] < 0 || labels[j] >= C) { loss[j] = NAN; continue; }
        double m = row[0];
        for (int64_t k = 1; k < C; ++k) m = row[k] > m ? row[k] : m;
        double e = 0.0;
        for (int64_t k = 0; k < C; ++k) e += exp(row[k] - m);
        loss[j] = log(e) - (row[labels[j]] - m);
    }
}

/*
 * LayerNorm of `rows` samples of `len` features each.  Two passes per row in fp64: the mean
 * (sum in index order / len), then the biased variance as the mean of squared deviations from
 * that mean (not E[x^2] - mean^2), then y = (x - mean) / sqrt(var + eps).  Results kept in fp64.
 */
void oracle_layernorm(int64_t rows, int64_t len, const float *x, double eps, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + r * len;
        double *yr = y + r * len;
        double s = 0.0;
        for (int64_t i = 0; i < len; ++i) s += (double)xr[i];
        const double mean = s / (double)len;
        double q = 0.0;
        for (int64_t i = 0; i < len; ++i) q += ((double)xr[i] - mean) * ((double)xr[i] - mean);
        const double rstd = 1.0 / sqrt(q / (double)len + eps);
        for (int64_t i = 0; i < len; ++i) yr[i] = ((double)xr[i] - mean) * rstd;
    }
}

/*
 * The same LayerNorm for rows that are already fp64 (the contraction fused with LayerNorm keeps
 * its products unrounded): identical steps, no conversion.
 */
void oracle_layernorm_f64(int64_t rows, int64_t len, const double *x, double eps, double *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * len;
        double *yr = y + r * len;
        double s = 0.0;
        for (int64_t i = 0; i < len; ++i) s += xr[i];
        const double mean = s / (double)len;
        double q = 0.0;
        for (int64_t i = 0; i < len; ++i) q += (xr[i] - mean) * (xr[i] - mean);
        const double rstd = 1.0 / sqrt(q / (double)len + eps);
        for (int64_t i = 0; i < len; ++i) yr[i] = (xr[i] - mean) * rstd;
    }
}

/*
 * Transpose (Table 4, task 8): dst[j][i] = src[i][j] for a rows x cols row-major matrix of
 * elements of `esize` bytes; dst is cols x rows row-major.  Bytes are moved, never interpreted.
 */
void oracle_transpose(int64_t rows, int64_t cols, const void *src, void *dst, int64_t esize)
{
    const char *s = (const char *)src;
    char *d = (char *)dst;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j)
            memcpy(d + (j * rows + i) * esize, s + (i * cols + j) * esize, (size_t)esize);
}

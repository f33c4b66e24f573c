// Row-wise bandwidth-bound siblings on fp32 arrays (paper Table 4): categorical cross-entropy
// (task 17: mean over rows of log(sum_k exp(z_jk)) - z_{j, y_j}) and LayerNorm over all features
// of a sample (task 4: (x - mean) / sqrt(var + eps) per row, biased variance, no scale / shift).
//
// Both read every input byte once when they can and walk memory in block order (see
// kernel_streams.hip for why that matters on this board).
//
// Cross-entropy.  A wave owns a row at a time; a lane holds up to 32 logits of a 2048-column
// slice in registers, takes the slice's maximum, and folds the slice into a running (max, sum)
// pair: sum = sum * exp(max_old - max_new) + sum_k exp(z_k - max_new), one exponential per
// logit.  Lanes are merged with the same rule by a butterfly; the row's loss is
// log(sum) - (z_y - max) in fp64; row losses are added in fp64 in a fixed order (wave, then
// workgroup, then a second small kernel over the per-workgroup partials).  For fewer than 64
// classes a lane owns a whole row instead.
//
// LayerNorm.  Rows of at most 8192 features: one workgroup per row keeps the row in registers
// (one read, one write).  Longer rows are cut into chunks of 16,384 features, one workgroup each:
// a first kernel leaves per-chunk sums of d = x - x_row[0] and d^2 in fp64 (shifting by the
// row's first element keeps the variance from cancelling when |mean| >> std), a second kernel
// adds a row's chunk sums in a fixed order and normalises its chunk: x is read twice (12 bytes
// per element against 8 algorithmic).  Running the two kernels over groups of rows small enough
// for the 256 MiB Infinity Cache was measured and bought nothing (4.1 - 4.3 TB/s of algorithmic
// bytes for any group size from 32 MiB up), so groups are 256 MiB only to bound the workspace.
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;

bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

// ---- cross-entropy ---------------------------------------------------------------------------

struct MaxSum {
    float m, s;
};

__device__ __forceinline__ MaxSum merge(MaxSum a, MaxSum b)
{
    if (b.s == 0.0f) return a;               // a side that has seen nothing (a real side has s >= 1)
    if (a.s == 0.0f) return b;
    const float m = a.m > b.m ? a.m : b.m;
    // exp_neg(x) = exp(-x)
    return MaxSum{m, a.s * exp_neg(m - a.m) + b.s * exp_neg(m - b.m)};
}

// loss of one row from the merged (max, sum), in fp64; NaN for a label outside [0, C)
__device__ __forceinline__ double row_loss(MaxSum r, const float *row, int64_t C, int label)
{
    if (label < 0 || label >= C) return __builtin_nan("");
    return log((double)r.s) - ((double)row[label] - (double)r.m);
}

// WAVE_ROWS: a wave per row (C >= 64); rows_per_group rows per workgroup, taken by its 4 waves in turn.
// VEC: rows are 16-byte aligned (base aligned, ld % 4 == 0).
template <bool VEC>
__global__ __launch_bounds__(kThreads) void ce_wave_rows_kernel(const float *__restrict__ z, int64_t ld,
                                                                const int *__restrict__ labels, int64_t N, int64_t C,
                                                                int rows_per_group, double *__restrict__ partial)
{
    __shared__ double wave_sum[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_group;
    double acc = 0.0;
    for (int64_t j = row0 + wave; j < row0 + rows_per_group && j < N; j += kThreads / 64) {
        const float *row = z + j * ld;
        MaxSum r{-__builtin_inff(), 0.0f};
        if (VEC) {
            constexpr int U = 8;                          // 8 x 64 lanes x 4 = 2048 columns per slice
            const int64_t c4 = C / 4;
            const floatx4 *row4 = reinterpret_cast<const floatx4 *>(row);
            // Rows are walked in slices of 2048 columns, row j starting 5 j slices in and wrapping:
            // with a power-of-two row pitch the waves in flight would otherwise all sit at the same
            // offset within their rows, i.e. on the same few memory channels.
            const int64_t slices = (c4 + U * 64 - 1) / (U * 64);
            const int64_t start = slices > 0 ? (j * 5) % slices : 0;
            // the loads of slice it + 1 are in flight while slice it is summed
            auto fetch = [&](int64_t it, floatx4 (&v)[U]) {
                const int64_t sl = it + start < slices ? it + start : it + start - slices;
                const int64_t base = lane + sl * (U * 64);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool in = base + u * 64 < c4;
                    v[u] = in ? __builtin_nontemporal_load(row4 + base + u * 64)
                              : floatx4{-__builtin_inff(), -__builtin_inff(), -__builtin_inff(), -__builtin_inff()};
                }
            };
            auto fold = [&](const floatx4 (&v)[U]) {
                float mx = -__builtin_inff();
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) mx = v[u][e] > mx ? v[u][e] : mx;
                if (mx == -__builtin_inff()) return;        // nothing (or only -inf) in this lane's part
                const float m = r.m > mx ? r.m : mx;
                float s = r.s * exp_neg(m - r.m);
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) s += exp_neg(m - v[u][e]);
                r = MaxSum{m, s};
            };
            floatx4 va[U], vb[U];
            if (slices > 0) fetch(0, va);
            for (int64_t it = 0; it < slices; it += 2) {
                if (it + 1 < slices) fetch(it + 1, vb);
                fold(va);
                if (it + 1 < slices) {
                    if (it + 2 < slices) fetch(it + 2, va);
                    fold(vb);
                }
            }
            for (int64_t k = 4 * c4 + lane; k < C; k += 64) r = merge(r, MaxSum{row[k], 1.0f});
        } else {
            for (int64_t k = lane; k < C; k += 64) r = merge(r, MaxSum{row[k], 1.0f});
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            MaxSum o{__shfl_xor(r.m, off, 64), __shfl_xor(r.s, off, 64)};
            r = merge(r, o);
        }
        if (lane == 0) acc += row_loss(r, row, C, labels[j]);
    }
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wave_sum[0];
        for (int w = 1; w < kThreads / 64; ++w) t += wave_sum[w];
        partial[blockIdx.x] = t;
    }
}

// 64 <= C <= 1024, rows 16-byte aligned: LPR lanes per row (several rows per wave), U vectors of four per lane, so
// that a lane has no more empty slots than a factor of two - the wave-per-row kernel above spends 32 exponentials
// per lane and row whatever C is (0.29 TB/s at C = 64, 1.1 at 256, 3.7 at 1000).
template <int LPR, int U>
__global__ __launch_bounds__(kThreads) void ce_group_rows_kernel(const float *__restrict__ z, int64_t ld,
                                                                 const int *__restrict__ labels, int64_t N, int64_t C,
                                                                 int rows_per_group, double *__restrict__ partial)
{
    __shared__ double wave_sum[kThreads / 64];
    constexpr int GPW = 64 / LPR, GROUPS = (kThreads / 64) * GPW;      // rows per wave, rows in flight per workgroup
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, gl = lane % LPR, g = lane / LPR;
    const int64_t row0 = (int64_t)blockIdx.x * rows_per_group;
    const int64_t c4 = C / 4;
    double acc = 0.0;
    for (int64_t j = row0 + wave * GPW + g; j < row0 + rows_per_group && j < N; j += GROUPS) {
        const float *row = z + j * ld;
        const floatx4 *row4 = reinterpret_cast<const floatx4 *>(row);
        floatx4 v[U];
        float mx = -__builtin_inff();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool in = gl + u * LPR < c4;
            v[u] = in ? __builtin_nontemporal_load(row4 + gl + u * LPR)
                      : floatx4{-__builtin_inff(), -__builtin_inff(), -__builtin_inff(), -__builtin_inff()};
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = v[u][e] > mx ? v[u][e] : mx;
        }
        MaxSum r{-__builtin_inff(), 0.0f};
        if (mx != -__builtin_inff()) {
            float s = 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) s += exp_neg(mx - v[u][e]);
            r = MaxSum{mx, s};
        }
        for (int64_t k = 4 * c4 + gl; k < C; k += LPR) r = merge(r, MaxSum{row[k], 1.0f});
#pragma unroll
        for (int off = LPR / 2; off >= 1; off >>= 1) {
            MaxSum o{__shfl_xor(r.m, off, 64), __shfl_xor(r.s, off, 64)};
            r = merge(r, o);
        }
        if (gl == 0) acc += row_loss(r, row, C, labels[j]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) wave_sum[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wave_sum[0];
        for (int w = 1; w < kThreads / 64; ++w) t += wave_sum[w];
        partial[blockIdx.x] = t;
    }
}

// C < 64: a lane per row; workgroup b takes rows [256 b, 256 b + 256)
__global__ __launch_bounds__(kThreads) void ce_lane_rows_kernel(const float *__restrict__ z, int64_t ld,
                                                                const int *__restrict__ labels, int64_t N, int64_t C,
                                                                double *__restrict__ partial)
{
    __shared__ double wave_sum[kThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t j = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    double loss = 0.0;
    if (j < N) {
        const float *row = z + j * ld;
        float m = row[0];
        for (int64_t k = 1; k < C; ++k) m = row[k] > m ? row[k] : m;
        float s = 0.0f;
        for (int64_t k = 0; k < C; ++k) s += exp_neg(m - row[k]);
        loss = row_loss(MaxSum{m, s}, row, C, labels[j]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) loss += __shfl_xor(loss, off, 64);
    if (lane == 0) wave_sum[wave] = loss;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wave_sum[0];
        for (int w = 1; w < kThreads / 64; ++w) t += wave_sum[w];
        partial[blockIdx.x] = t;
    }
}

// out = (sum of the partials, thread t adding partials t, t + 1024, ... in order, then a fixed
// tree) / N
constexpr int kFinalThreads = 1024;
__global__ __launch_bounds__(kFinalThreads) void mean_of_partials_kernel(const double *__restrict__ partial, int count,
                                                                         int64_t N, float *__restrict__ out)
{
    __shared__ double tree[kFinalThreads];
    double c = 0.0;
    for (int i = threadIdx.x; i < count; i += kFinalThreads) c += partial[i];
    tree[threadIdx.x] = c;
    __syncthreads();
    for (int half = kFinalThreads / 2; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) tree[threadIdx.x] += tree[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (float)(N > 0 ? tree[0] / (double)N : 0.0);
}

// ---- LayerNorm -------------------------------------------------------------------------------

// sum over the workgroup of two fp64 values, fixed order (butterfly in the wave, waves in order);
// every thread gets the result
template <int THREADS = kThreads>
__device__ __forceinline__ void block_sum2(double &a, double &b, double (*scratch)[2])
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        a += __shfl_xor(a, off, 64);
        b += __shfl_xor(b, off, 64);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();                         // scratch may still be read from a previous call
    if (lane == 0) { scratch[wave][0] = a; scratch[wave][1] = b; }
    __syncthreads();
    a = scratch[0][0]; b = scratch[0][1];
    for (int w = 1; w < THREADS / 64; ++w) { a += scratch[w][0]; b += scratch[w][1]; }
}

// One workgroup of THREADS per row.  VEC: the row, at most THREADS * U * 4 features, is read once
// and held in registers (8 bytes of traffic per feature); scalar: it is read three times.
template <bool VEC, int THREADS, int U>
__global__ __launch_bounds__(THREADS) void layernorm_short_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                  int64_t len, double eps)
{
    constexpr int kThreads = THREADS;
    __shared__ double scratch[kThreads / 64][2];
    const float *xr = x + (int64_t)blockIdx.x * len;
    float *yr = y + (int64_t)blockIdx.x * len;
    const double inv_len = 1.0 / (double)len;
    if (VEC) {
        const int64_t n4 = len / 4;                      // len % 4 == 0 here
        const floatx4 *x4 = reinterpret_cast<const floatx4 *>(xr);
        floatx4 v[U];
        double s = 0.0, unused = 0.0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = threadIdx.x + u * kThreads;
            v[u] = i < n4 ? __builtin_nontemporal_load(x4 + i) : floatx4{0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 4; ++e) s += (double)v[u][e];
        }
        block_sum2<THREADS>(s, unused, scratch);
        const double mean = s * inv_len;
        double q = 0.0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = threadIdx.x + u * kThreads;
            if (i < n4) {
#pragma unroll
                for (int e = 0; e < 4; ++e) q += ((double)v[u][e] - mean) * ((double)v[u][e] - mean);
            }
        }
        unused = 0.0;
        block_sum2<THREADS>(q, unused, scratch);
        const double rstd = 1.0 / sqrt(q * inv_len + eps);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = threadIdx.x + u * kThreads;
            if (i < n4) {
                floatx4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = (float)(((double)v[u][e] - mean) * rstd);
                __builtin_nontemporal_store(r, reinterpret_cast<floatx4 *>(yr) + i);
            }
        }
    } else {
        double s = 0.0, unused = 0.0;
        for (int64_t i = threadIdx.x; i < len; i += kThreads) s += (double)xr[i];
        block_sum2<THREADS>(s, unused, scratch);
        const double mean = s * inv_len;
        double q = 0.0;
        for (int64_t i = threadIdx.x; i < len; i += kThreads) q += ((double)xr[i] - mean) * ((double)xr[i] - mean);
        unused = 0.0;
        block_sum2<THREADS>(q, unused, scratch);
        const double rstd = 1.0 / sqrt(q * inv_len + eps);
        for (int64_t i = threadIdx.x; i < len; i += kThreads) yr[i] = (float)(((double)xr[i] - mean) * rstd);
    }
}


// rows of at most 2048 features (len % 4 == 0, 16-byte aligned): one wave per row, four rows per workgroup, the row
// in registers, sums by butterfly across the wave only - no LDS, no barrier.  A workgroup per row leaves such rows
// at 4.2 TB/s (8 KiB of work per workgroup).
template <int U>                 // vectors of four per lane: len <= 256 U
__global__ __launch_bounds__(kThreads) void layernorm_wave_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                  int64_t rows, int64_t len, double eps)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t row = (int64_t)blockIdx.x * (kThreads / 64) + wave;
    if (row >= rows) return;
    const floatx4 *x4 = reinterpret_cast<const floatx4 *>(x + row * len);
    floatx4 *y4 = reinterpret_cast<floatx4 *>(y + row * len);
    const int64_t n4 = len / 4;
    const double inv_len = 1.0 / (double)len;
    floatx4 v[U];
    double s = 0.0;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = lane + 64 * u;
        v[u] = i < n4 ? __builtin_nontemporal_load(x4 + i) : floatx4{0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 4; ++e) s += (double)v[u][e];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    const double mean = s * inv_len;
    double q = 0.0;
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (lane + 64 * u < n4) {
#pragma unroll
            for (int e = 0; e < 4; ++e) q += ((double)v[u][e] - mean) * ((double)v[u][e] - mean);
        }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) q += __shfl_xor(q, off, 64);
    const double rstd = 1.0 / sqrt(q * inv_len + eps);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int64_t i = lane + 64 * u;
        if (i < n4) {
            floatx4 r;
#pragma unroll
            for (int e = 0; e < 4; ++e) r[e] = (float)(((double)v[u][e] - mean) * rstd);
            __builtin_nontemporal_store(r, y4 + i);
        }
    }
}

// long rows, first kernel: stats[(row * chunks + c) * 2 + {0, 1}] = sum of d, sum of d^2 over the
// chunk, d = x - x_row[0]; pivots[row] = x_row[0] (y may be x: the second kernel must not read it there).  Plain loads: the data is meant to stay in cache for the second kernel.
template <bool VEC>
__global__ __launch_bounds__(kThreads) void layernorm_stats_kernel(const float *__restrict__ x, int64_t len, int64_t chunks,
                                                                   int64_t kChunk, double *__restrict__ stats,
                                                                   double *__restrict__ pivots)
{
    __shared__ double scratch[kThreads / 64][2];
    const int64_t row = blockIdx.x / chunks, c = blockIdx.x % chunks;
    const float *xr = x + row * len;
    const double pivot = (double)xr[0];
    const int64_t lo = c * kChunk, hi = lo + kChunk < len ? lo + kChunk : len;
    double s = 0.0, q = 0.0;
    if (VEC) {
        const floatx4 *x4 = reinterpret_cast<const floatx4 *>(xr);
        for (int64_t base = lo / 4 + threadIdx.x; base < hi / 4; base += 8 * kThreads) {
            floatx4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t i = base + u * kThreads;
                v[u] = i < hi / 4 ? x4[i] : floatx4{(float)pivot, (float)pivot, (float)pivot, (float)pivot};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const double d = (double)v[u][e] - pivot;
                    s += d;
                    q += d * d;
                }
        }
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) {
            const double d = (double)xr[i] - pivot;
            s += d;
            q += d * d;
        }
    }
    block_sum2(s, q, scratch);
    if (threadIdx.x == 0) {
        stats[2 * blockIdx.x] = s;
        stats[2 * blockIdx.x + 1] = q;
        if (c == 0) pivots[row] = pivot;
    }
}

// long rows, second kernel: add the row's chunk sums (fixed order), normalise this chunk
template <bool VEC>
__global__ __launch_bounds__(kThreads) void layernorm_apply_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                   int64_t len, int64_t chunks, int64_t kChunk,
                                                                   const double *__restrict__ stats,
                                                                   const double *__restrict__ pivots, double eps,
                                                                   const unsigned *__restrict__ done)
{
    if (done != nullptr && done[blockIdx.x] != 0u) return;      // normalised by the one-pass kernel already
    const int64_t row = blockIdx.x / chunks, c = blockIdx.x % chunks;
    const float *xr = x + row * len;
    float *yr = y + row * len;
    __shared__ double scratch[kThreads / 64][2];
    double s = 0.0, q = 0.0;                              // thread t: chunks t, t + 256, ... in order
    for (int64_t i = threadIdx.x; i < chunks; i += kThreads) {
        s += stats[2 * (row * chunks + i)];
        q += stats[2 * (row * chunks + i) + 1];
    }
    block_sum2(s, q, scratch);
    const double inv_len = 1.0 / (double)len;
    const double dm = s * inv_len;                        // mean - pivot
    const double mean = pivots[row] + dm;
    double var = q * inv_len - dm * dm;                   // shifted-data formula
    var = var > 0.0 ? var : 0.0;
    const double rstd = 1.0 / sqrt(var + eps);
    const int64_t lo = c * kChunk, hi = lo + kChunk < len ? lo + kChunk : len;
    if (VEC) {
        const floatx4 *x4 = reinterpret_cast<const floatx4 *>(xr);
        floatx4 *y4 = reinterpret_cast<floatx4 *>(yr);
        for (int64_t base = lo / 4 + threadIdx.x; base < hi / 4; base += 8 * kThreads) {
            floatx4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t i = base + u * kThreads;
                v[u] = i < hi / 4 ? __builtin_nontemporal_load(x4 + i) : floatx4{0, 0, 0, 0};
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int64_t i = base + u * kThreads;
                if (i < hi / 4) {
                    floatx4 r;
#pragma unroll
                    for (int e = 0; e < 4; ++e) r[e] = (float)(((double)v[u][e] - mean) * rstd);
                    __builtin_nontemporal_store(r, y4 + i);
                }
            }
        }
    } else {
        for (int64_t i = lo + threadIdx.x; i < hi; i += kThreads) yr[i] = (float)(((double)xr[i] - mean) * rstd);
    }
}

// Long rows in ONE pass over x.  A workgroup keeps a chunk of 8 Ki features in registers (8 vectors a thread),
// publishes the chunk's (sum of d, sum of d^2), announces itself on the row's counter and waits until all the
// row's chunks have done so; then every workgroup adds the row's chunk sums in the same fixed order and normalises
// from registers: 8 bytes of traffic per feature instead of 12.
//   * The grid is persistent: no larger than what the device holds at once, a multiple of the chunks per row where
//     that fits, each workgroup taking chunk after chunk (index += grid size), so that the workgroups of a row
//     reach it together whatever order the hardware starts workgroups in.
//   * Signalling through a memory system that is saturated with the rows themselves takes microseconds per round
//     trip, so a workgroup has TWO chunks in flight: it loads and publishes its next chunk before it waits for the
//     row of the current one, and the wait is hidden behind that load.
//   * Other work on the device can still keep part of the grid from running, so the wait is bounded (`wait_clocks`
//     shader clocks): a workgroup that gives up leaves its chunk to layernorm_apply_kernel, which runs afterwards
//     over all chunks and skips those marked done.  `arrived` and `done` start at zero.
constexpr int64_t kOnePassChunk = 8192, kOnePassMaxChunks = 512;     // rows of up to 4 Mi features; beyond, two kernels are faster

__global__ __launch_bounds__(kThreads, 4) void layernorm_onepass_kernel(const float *__restrict__ x, float *__restrict__ y, int64_t len,
                                                                        int64_t chunks, int64_t tasks, double *stats, double *pivots,
                                                                        unsigned long long *arrived, unsigned *done, double eps,
                                                                        long long wait_clocks)
{
    __shared__ double scratch[kThreads / 64][2];
    __shared__ int ready;
    constexpr int U = (int)(kOnePassChunk / 4 / kThreads);      // vectors a thread holds of one chunk
    auto count_of = [&](int64_t task) __attribute__((always_inline)) {                   // vectors in the chunk
        const int64_t lo = (task % chunks) * kOnePassChunk;
        return ((lo + kOnePassChunk < len ? lo + kOnePassChunk : len) - lo) / 4;        // len % 4 == 0 here
    };
    // the chunk into registers, its sums published, its arrival counted
    auto take = [&](floatx4 (&v)[U], float &pivot, int64_t task) __attribute__((always_inline)) {
        const int64_t row = task / chunks, c = task % chunks;
        const float *xr = x + row * len;
        pivot = xr[0];
        const int64_t n4 = count_of(task);
        const floatx4 *x4 = reinterpret_cast<const floatx4 *>(xr + c * kOnePassChunk);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = threadIdx.x + u * kThreads;
            v[u] = i < n4 ? __builtin_nontemporal_load(x4 + i) : floatx4{pivot, pivot, pivot, pivot};
        }
        double s = 0.0, q = 0.0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double d = (double)v[u][e] - (double)pivot;
                s += d;
                q += d * d;
            }
            __builtin_amdgcn_sched_barrier(0);           // one vector at a time: the doubles are not kept
        }
        block_sum2(s, q, scratch);
        if (threadIdx.x == 0) {
            // Only relaxed device-scope atomics cross between workgroups here: they are performed at the memory
            // side, past the per-XCD L2s, and cost nothing else (an acquire or release at device scope would
            // invalidate or write back a whole L2 for every workgroup and poll).  Order comes from completion:
            // the two exchanges have returned their old values, so they are done, before the counter is bumped,
            // and a reader loads the sums only after it has seen the full count.  Such atomics on ONE address
            // take about 0.1 us each, one after the other, so a row counts its arrivals in 32 places (16 words of
            // 64 bits, a count in each half), which one 16-lane load reads back.
            const double old_s = __hip_atomic_exchange(stats + 2 * task, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const double old_q = __hip_atomic_exchange(stats + 2 * task + 1, q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (c == 0) pivots[row] = (double)pivot;     // for the second kernel: y may be x, and x[row][0] gone by then
            asm volatile("" :: "v"(old_s), "v"(old_q) : "memory");       // both have returned
            const unsigned long long old_n = __hip_atomic_fetch_add(arrived + row * 16 + ((c & 31) >> 1), (c & 1) ? 1ull << 32 : 1ull,
                                                                    __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("" :: "v"(old_n) : "memory");
        }
    };
    // wait for the chunk's row, normalise from registers
    auto finish = [&](floatx4 (&v)[U], float pivot, int64_t task) __attribute__((always_inline)) {
        const int64_t row = task / chunks, c = task % chunks;
        if (threadIdx.x < 64) {
            const unsigned long long *row_count = arrived + row * 16;
            const long long t0 = (long long)__builtin_amdgcn_s_memtime();
            int ok = 0;
            for (;;) {
                const unsigned long long w = threadIdx.x < 16 ? __hip_atomic_load(row_count + threadIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0ull;
                unsigned seen = (unsigned)(w & 0xffffffffull) + (unsigned)(w >> 32);
#pragma unroll
                for (int off = 8; off >= 1; off >>= 1) seen += __shfl_xor(seen, off, 64);
                seen = __builtin_amdgcn_readfirstlane(seen);
                if (seen >= (unsigned)chunks) { ok = 1; break; }
                if ((long long)__builtin_amdgcn_s_memtime() - t0 >= wait_clocks) break;
                // every poll of a row goes to the same two lines in memory: sleep longer while many are missing
                for (unsigned k = 0; k <= ((unsigned)chunks - seen) / 32u; ++k) __builtin_amdgcn_s_sleep(4);
            }
            asm volatile("" ::: "memory");
            if (threadIdx.x == 0) ready = ok;
        }
        __syncthreads();
        const bool go = ready != 0;
        __syncthreads();                                  // `ready` is free again
        if (!go) return;                                  // the second kernel normalises this chunk
        double s = 0.0, q = 0.0;                          // thread t: chunks t, t + 256, ... in order, as the apply kernel
        for (int64_t i = threadIdx.x; i < chunks; i += kThreads) {
            s += __hip_atomic_load(stats + 2 * (row * chunks + i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            q += __hip_atomic_load(stats + 2 * (row * chunks + i) + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        block_sum2(s, q, scratch);
        const double inv_len = 1.0 / (double)len;
        const double dm = s * inv_len;                    // mean - pivot
        const double mean = (double)pivot + dm;
        double var = q * inv_len - dm * dm;               // shifted-data formula
        var = var > 0.0 ? var : 0.0;
        const double rstd = 1.0 / sqrt(var + eps);
        const int64_t n4 = count_of(task);
        floatx4 *y4 = reinterpret_cast<floatx4 *>(y + row * len + c * kOnePassChunk);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = threadIdx.x + u * kThreads;
            if (i < n4) {
                floatx4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float f = v[u][e];
                    asm volatile("" : "+v"(f));          // convert again here rather than keep 64 doubles from the first pass
                    r[e] = (float)(((double)f - mean) * rstd);
                }
                __builtin_nontemporal_store(r, y4 + i);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (threadIdx.x == 0) done[task] = 1u;
    };

    floatx4 va[U], vb[U];
    float pa = 0.0f, pb = 0.0f;
    int64_t t = blockIdx.x;
    if (t < tasks) take(va, pa, t);
    while (t < tasks) {
        int64_t tn = t + gridDim.x;
        if (tn < tasks) take(vb, pb, tn);
        finish(va, pa, t);
        t = tn;
        if (t >= tasks) break;
        tn = t + gridDim.x;
        if (tn < tasks) take(va, pa, tn);
        finish(vb, pb, t);
        t = tn;
    }
}

__global__ __launch_bounds__(kThreads) void zero_words_kernel(unsigned *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0u;
}

long long g_wait_clocks = 1ll << 22;       // about 2 ms: a row's loads take microseconds

}  // namespace

void set_wait_limit(long long clocks) { g_wait_clocks = clocks < 0 ? 0 : clocks; }

hipError_t launch_cross_entropy(int64_t N, int64_t C, const float *z, int64_t ld, const int *labels, float *loss,
                                hipStream_t stream)
{
    int64_t grid = 0;
    int rows_per_group = 0;
    if (N > 0) {
        if (C < 64) {
            grid = (N + kThreads - 1) / kThreads;
        } else {
            // about 64 KiB of logits per workgroup, a multiple of its 4 waves
            int64_t r = (16384 + C - 1) / C;
            r = (r + 3) / 4 * 4;
            rows_per_group = (int)(r < 4 ? 4 : (r > 1024 ? 1024 : r));
            grid = (N + rows_per_group - 1) / rows_per_group;
        }
    }
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    void *ws = nullptr;
    hipError_t e = workspace(sizeof(double) * (size_t)(grid > 0 ? grid : 1), &ws, stream);
    if (e != hipSuccess) return e;
    double *partial = static_cast<double *>(ws);
    if (grid > 0) {
        if (C < 64) {
            hipLaunchKernelGGL(ce_lane_rows_kernel, dim3((unsigned)grid), dim3(kThreads), 0, stream, z, ld, labels, N, C,
                               partial);
        } else if (aligned16(z) && ld % 4 == 0 && C <= 1024) {
            const dim3 g((unsigned)grid), b(kThreads);
            if (C <= 64) hipLaunchKernelGGL((ce_group_rows_kernel<16, 1>), g, b, 0, stream, z, ld, labels, N, C, rows_per_group, partial);
            else if (C <= 128) hipLaunchKernelGGL((ce_group_rows_kernel<16, 2>), g, b, 0, stream, z, ld, labels, N, C, rows_per_group, partial);
            else if (C <= 256) hipLaunchKernelGGL((ce_group_rows_kernel<16, 4>), g, b, 0, stream, z, ld, labels, N, C, rows_per_group, partial);
            else if (C <= 512) hipLaunchKernelGGL((ce_group_rows_kernel<32, 4>), g, b, 0, stream, z, ld, labels, N, C, rows_per_group, partial);
            else hipLaunchKernelGGL((ce_group_rows_kernel<64, 4>), g, b, 0, stream, z, ld, labels, N, C, rows_per_group, partial);
        } else if (aligned16(z) && ld % 4 == 0) {
            hipLaunchKernelGGL(ce_wave_rows_kernel<true>, dim3((unsigned)grid), dim3(kThreads), 0, stream, z, ld, labels, N,
                               C, rows_per_group, partial);
        } else {
            hipLaunchKernelGGL(ce_wave_rows_kernel<false>, dim3((unsigned)grid), dim3(kThreads), 0, stream, z, ld, labels,
                               N, C, rows_per_group, partial);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(mean_of_partials_kernel, dim3(1), dim3(kFinalThreads), 0, stream, partial, (int)grid, N, loss);
    return hipGetLastError();
}

hipError_t launch_layernorm(int64_t rows, int64_t len, const float *x, float *y, float eps, hipStream_t stream)
{
    const bool vec = aligned16(x) && aligned16(y) && len % 4 == 0;
    if (len <= 8192 || (vec && len <= 32768)) {
        if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
        const dim3 grid((unsigned)rows);
        const double e64 = (double)eps;
        if (vec && len <= 2048) {
            const dim3 g((unsigned)((rows + kThreads / 64 - 1) / (kThreads / 64))), b(kThreads);
            if (len <= 256) hipLaunchKernelGGL(layernorm_wave_kernel<1>, g, b, 0, stream, x, y, rows, len, e64);
            else if (len <= 512) hipLaunchKernelGGL(layernorm_wave_kernel<2>, g, b, 0, stream, x, y, rows, len, e64);
            else if (len <= 1024) hipLaunchKernelGGL(layernorm_wave_kernel<4>, g, b, 0, stream, x, y, rows, len, e64);
            else hipLaunchKernelGGL(layernorm_wave_kernel<8>, g, b, 0, stream, x, y, rows, len, e64);
        } else if (!vec) hipLaunchKernelGGL((layernorm_short_kernel<false, kThreads, 8>), grid, dim3(kThreads), 0, stream, x, y, len, e64);
        else if (len <= 4096) hipLaunchKernelGGL((layernorm_short_kernel<true, kThreads, 8>), grid, dim3(kThreads), 0, stream, x, y, len, e64);
        // rows that a 1024-thread workgroup still holds in registers: one pass instead of the
        // two kernels below
        // (16 vectors a thread would spill)
        else if (len <= 16384) hipLaunchKernelGGL((layernorm_short_kernel<true, 512, 8>), grid, dim3(512), 0, stream, x, y, len, e64);
        else hipLaunchKernelGGL((layernorm_short_kernel<true, 1024, 8>), grid, dim3(1024), 0, stream, x, y, len, e64);
        return hipGetLastError();
    }
    if (vec && (len + kOnePassChunk - 1) / kOnePassChunk <= kOnePassMaxChunks) {
        const int64_t chunks = (len + kOnePassChunk - 1) / kOnePassChunk, blocks = rows * chunks;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        // workspace: 2 doubles per chunk, a pivot per row, 16 words of 64 bits of arrival counts per row, a flag per chunk
        const size_t words = (size_t)(32 * rows + blocks);
        void *ws = nullptr;
        hipError_t e = workspace(sizeof(double) * (2 * (size_t)blocks + (size_t)rows) + sizeof(unsigned) * words, &ws, stream);
        if (e != hipSuccess) return e;
        double *stats = static_cast<double *>(ws), *pivots = stats + 2 * blocks;
        unsigned long long *arrived = reinterpret_cast<unsigned long long *>(pivots + rows);
        unsigned *done = reinterpret_cast<unsigned *>(arrived + 16 * rows);
        hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)((words + kThreads - 1) / kThreads)), dim3(kThreads), 0, stream,
                           reinterpret_cast<unsigned *>(arrived), (int64_t)words);
        // persistent grid: what the device holds at once, rounded down to whole rows
        static const int per_cu = [] {
            int n = 0;
            return hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, layernorm_onepass_kernel, kThreads, 0) == hipSuccess && n > 0 ? n : 1;
        }();
        int64_t grid = (int64_t)per_cu * compute_units();
        if (grid > chunks) grid -= grid % chunks;
        if (grid > blocks) grid = blocks;
        hipLaunchKernelGGL(layernorm_onepass_kernel, dim3((unsigned)grid), dim3(kThreads), 0, stream, x, y, len, chunks, blocks,
                           stats, pivots, arrived, done, (double)eps, g_wait_clocks);
        hipLaunchKernelGGL(layernorm_apply_kernel<true>, dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, y, len, chunks,
                           kOnePassChunk, stats, pivots, (double)eps, done);
        return hipGetLastError();
    }
    // Chunk and group sizes from a sweep on 64 rows of 4 Mi features: 16 Ki features per workgroup and
    // groups of 256 MiB gave 4.3 TB/s of algorithmic bytes; 8 - 32 Ki and 32 MiB - everything stayed
    // within 8 % of that, 16 MiB groups (too few workgroups per launch) fell to 2.9 TB/s.
    const int64_t kChunk = 16384, group_bytes = int64_t(256) << 20;
    const int64_t chunks = (len + kChunk - 1) / kChunk;
    // groups of rows: statistics, then normalisation, group by group
    int64_t group = group_bytes / (len * 4);
    group = group < 1 ? 1 : group;
    if (group * chunks > 0x7fffffffLL) return hipErrorInvalidValue;
    void *ws = nullptr;
    hipError_t e = workspace(sizeof(double) * (2 * (size_t)(group * chunks) + (size_t)group), &ws, stream);
    if (e != hipSuccess) return e;
    double *stats = static_cast<double *>(ws), *pivots = stats + 2 * group * chunks;
    for (int64_t r0 = 0; r0 < rows; r0 += group) {
        const int64_t nr = rows - r0 < group ? rows - r0 : group;
        const dim3 grid((unsigned)(nr * chunks)), block(kThreads);
        const float *xg = x + r0 * len;
        float *yg = y + r0 * len;
        if (vec) {
            hipLaunchKernelGGL(layernorm_stats_kernel<true>, grid, block, 0, stream, xg, len, chunks, kChunk, stats, pivots);
            hipLaunchKernelGGL(layernorm_apply_kernel<true>, grid, block, 0, stream, xg, yg, len, chunks, kChunk, stats, pivots, (double)eps, nullptr);
        } else {
            hipLaunchKernelGGL(layernorm_stats_kernel<false>, grid, block, 0, stream, xg, len, chunks, kChunk, stats, pivots);
            hipLaunchKernelGGL(layernorm_apply_kernel<false>, grid, block, 0, stream, xg, yg, len, chunks, kChunk, stats, pivots, (double)eps, nullptr);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace optiml

// Bandwidth-bound siblings of the contraction on fp32 arrays (paper Table 4): element-wise ReLU
// (task 10) and sigmoid (task 1); sum (task 14), dot product (task 15) and mean squared error
// (task 7) as reductions to one value.
//
// All of them touch every input byte once: 128-bit non-temporal loads and stores, eight loads
// in flight per lane before the first use.  What matters most is the ORDER in which the chip
// as a whole walks memory: workgroup b owns the b-th contiguous block (32 KiB element-wise,
// 256 KiB for the reductions), so the workgroups resident at any moment cover one compact
// window of each array.  With the usual grid-size stride (every workgroup striding over the
// whole array) the same loads and stores reach 4.4 TB/s read+write and 5.5 TB/s read-only on
// this board; block order reaches 6.4 and 7.1 TB/s (measured with a working copy of these
// kernels; DRAM pages and read/write turnarounds, presumably).  The reductions
// accumulate in fp64 (one conversion and one fp64 add or fma per element is a twentieth of the
// fp64 rate at full HBM speed), which makes the result the correctly rounded fp32 of the exact
// sum up to fp64 rounding - no tolerance depends on n - and they are deterministic: lane sums,
// then wave, workgroup and grid sums, each in a fixed order, the last by a second small kernel
// over the per-workgroup partials in the library's workspace.  (Letting the last workgroup to
// finish add the partials instead was tried: the device-scope fence every workgroup then needs
// before it takes its ticket writes back the L2 of its XCD, and 8192 of those made the sum 3.5
// times slower.)  No atomics.
#include "common.hpp"
#include "epilogue.hpp"
#include "../../include/optiml.h"

namespace optiml {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;

template <int OP>
__device__ __forceinline__ float ew(float v)
{
    return OP == OPTIML_EW_RELU ? (v > 0.0f ? v : 0.0f) : sigmoidf_(v);
}

// VEC: both arrays 16-byte aligned -> 128-bit accesses for the first n/4*4 elements, workgroup b
// taking vectors [b * kBlock, (b + 1) * kBlock); otherwise one element per thread and step.
constexpr int kUnroll = 8, kBlock = kUnroll * kThreads;

template <int OP, bool VEC>
__global__ __launch_bounds__(kThreads) void elementwise_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                               int64_t n)
{
    if (VEC) {
        const int64_t n4 = n / 4, base = (int64_t)blockIdx.x * kBlock + threadIdx.x;
        const floatx4 *x4 = reinterpret_cast<const floatx4 *>(x);
        floatx4 *y4 = reinterpret_cast<floatx4 *>(y);
        floatx4 v[kUnroll];
        if (base + (kUnroll - 1) * kThreads < n4) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(x4 + base + u * kThreads);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                floatx4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = ew<OP>(v[u][e]);
                __builtin_nontemporal_store(r, y4 + base + u * kThreads);
            }
        } else {
            for (int u = 0; u < kUnroll; ++u) {
                const int64_t i = base + u * kThreads;
                if (i >= n4) break;
                const floatx4 a = x4[i];
                floatx4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = ew<OP>(a[e]);
                y4[i] = r;
            }
        }
        const int64_t j = 4 * n4 + threadIdx.x;          // at most three trailing elements
        if (blockIdx.x == 0 && j < n) y[j] = ew<OP>(x[j]);
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) y[i] = ew<OP>(x[i]);
    }
}

template <int OP>
__device__ __forceinline__ double red_term(float a, float b)
{
    if (OP == OPTIML_RED_SUM) return (double)a;
    if (OP == OPTIML_RED_DOT) return (double)a * (double)b;
    const double d = (double)a - (double)b;
    return d * d;
}

// partial[blockIdx.x] = sum of this workgroup's terms: kRedIter consecutive blocks of kBlock
// vectors.  Order: per lane eight interleaved chains over its vectors in index order, combined
// ((0+1)+(2+3))+((4+5)+(6+7)); lanes by a butterfly over the wave (fixed pattern); waves in wave
// order.
constexpr int kRedIter = 8;

template <int OP, bool VEC>
__global__ __launch_bounds__(kThreads) void reduce_partial_kernel(const float *__restrict__ x,
                                                                  const float *__restrict__ y, int64_t n,
                                                                  double *__restrict__ partial)
{
    __shared__ double wave_sum[kThreads / 64];
    double acc[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc[u] = 0.0;
    if (VEC) {
        const int64_t n4 = n / 4;
        const floatx4 *x4 = reinterpret_cast<const floatx4 *>(x);
        const floatx4 *y4 = reinterpret_cast<const floatx4 *>(y);
        for (int it = 0; it < kRedIter; ++it) {
            const int64_t base = ((int64_t)blockIdx.x * kRedIter + it) * kBlock + threadIdx.x;
            if (base + (kUnroll - 1) * kThreads < n4) {
                floatx4 a[kUnroll], b[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; ++u) {
                    a[u] = __builtin_nontemporal_load(x4 + base + u * kThreads);
                    if (OP != OPTIML_RED_SUM) b[u] = __builtin_nontemporal_load(y4 + base + u * kThreads);
                }
#pragma unroll
                for (int u = 0; u < kUnroll; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        acc[u] += red_term<OP>(a[u][e], OP != OPTIML_RED_SUM ? b[u][e] : 0.0f);
            } else {
                for (int u = 0; u < kUnroll; ++u) {
                    const int64_t i = base + u * kThreads;
                    if (i >= n4) break;
                    const floatx4 a = x4[i];
                    floatx4 b = floatx4{0, 0, 0, 0};
                    if (OP != OPTIML_RED_SUM) b = y4[i];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[u] += red_term<OP>(a[e], b[e]);
                }
            }
        }
        const int64_t j = 4 * n4 + threadIdx.x;          // at most three trailing elements
        if (blockIdx.x == 0 && j < n) acc[0] += red_term<OP>(x[j], OP != OPTIML_RED_SUM ? y[j] : 0.0f);
    } else {
        const int64_t stride = (int64_t)gridDim.x * kThreads;
        for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride)
            acc[0] += red_term<OP>(x[i], OP != OPTIML_RED_SUM ? y[i] : 0.0f);
    }
    double s = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) wave_sum[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wave_sum[0];
        for (int w = 1; w < kThreads / 64; ++w) t += wave_sum[w];
        partial[blockIdx.x] = t;
    }
}

// out = fp32 of the sum of the partials, divided by n for the mean squared error.  1024 threads;
// thread t adds partials t, t + 1024, ... in order (loads issued four at a time), then a fixed
// tree over the threads.
constexpr int kFinalThreads = 1024;

__global__ __launch_bounds__(kFinalThreads) void reduce_final_kernel(const double *__restrict__ partial, int count,
                                                                     int64_t n, int op, float *__restrict__ out)
{
    __shared__ double tree[kFinalThreads];
    double c[4] = {0.0, 0.0, 0.0, 0.0};
    for (int i = threadIdx.x; i < count; i += 4 * kFinalThreads) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * kFinalThreads < count) c[u] += partial[i + u * kFinalThreads];
    }
    tree[threadIdx.x] = (c[0] + c[1]) + (c[2] + c[3]);
    __syncthreads();
    for (int half = kFinalThreads / 2; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) tree[threadIdx.x] += tree[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        double t = tree[0];
        if (op == OPTIML_RED_MSE) t = n > 0 ? t / (double)n : 0.0;
        *out = (float)t;
    }
}

bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

// one workgroup per block of `vectors_per_group` 128-bit vectors (vector path); the scalar path
// strides over the array with a few workgroups per CU
int64_t grid_for(int64_t n, bool vec, int64_t vectors_per_group)
{
    if (vec) {
        const int64_t g = (n / 4 + vectors_per_group - 1) / vectors_per_group;
        return g > 0 ? g : 1;
    }
    const int64_t by_size = (n + kThreads - 1) / kThreads, cap = (int64_t)compute_units() * 8;
    return by_size < cap ? by_size : cap;
}

}  // namespace

hipError_t launch_elementwise(int64_t n, const float *x, float *y, int op, hipStream_t stream)
{
    const bool vec = aligned16(x) && aligned16(y);
    const dim3 grid((unsigned)grid_for(n, vec, kBlock)), block(kThreads);
    if (op == OPTIML_EW_RELU) {
        if (vec) hipLaunchKernelGGL((elementwise_kernel<OPTIML_EW_RELU, true>), grid, block, 0, stream, x, y, n);
        else hipLaunchKernelGGL((elementwise_kernel<OPTIML_EW_RELU, false>), grid, block, 0, stream, x, y, n);
    } else {
        if (vec) hipLaunchKernelGGL((elementwise_kernel<OPTIML_EW_SIGMOID, true>), grid, block, 0, stream, x, y, n);
        else hipLaunchKernelGGL((elementwise_kernel<OPTIML_EW_SIGMOID, false>), grid, block, 0, stream, x, y, n);
    }
    return hipGetLastError();
}

template <int OP>
static hipError_t launch_partial(bool vec, int grid, hipStream_t stream, const float *x, const float *y, int64_t n,
                                 double *partial)
{
    if (vec) hipLaunchKernelGGL((reduce_partial_kernel<OP, true>), dim3(grid), dim3(kThreads), 0, stream, x, y, n, partial);
    else hipLaunchKernelGGL((reduce_partial_kernel<OP, false>), dim3(grid), dim3(kThreads), 0, stream, x, y, n, partial);
    return hipGetLastError();
}

hipError_t launch_reduce(int64_t n, const float *x, const float *y, int op, float *out, hipStream_t stream)
{
    const bool vec = aligned16(x) && (op == OPTIML_RED_SUM || aligned16(y));
    const int grid = n > 0 ? (int)grid_for(n, vec, (int64_t)kBlock * kRedIter) : 0;
    void *ws = nullptr;
    hipError_t e = workspace(sizeof(double) * (size_t)(grid > 0 ? grid : 1), &ws, stream);
    if (e != hipSuccess) return e;
    double *partial = static_cast<double *>(ws);
    if (grid > 0) {
        if (op == OPTIML_RED_SUM) e = launch_partial<OPTIML_RED_SUM>(vec, grid, stream, x, y, n, partial);
        else if (op == OPTIML_RED_DOT) e = launch_partial<OPTIML_RED_DOT>(vec, grid, stream, x, y, n, partial);
        else e = launch_partial<OPTIML_RED_MSE>(vec, grid, stream, x, y, n, partial);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(reduce_final_kernel, dim3(1), dim3(kFinalThreads), 0, stream, partial, grid, n, op, out);
    return hipGetLastError();
}

}  // namespace optiml

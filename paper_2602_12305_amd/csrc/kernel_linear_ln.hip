// The contraction followed by LayerNorm over each row of the product (paper Table 4, task 2 into
// task 4):
//     y[i][j] = (z[i][j] - mean_i) / sqrt(var_i + eps),   z = A.B + bias,
// mean_i and the biased variance var_i over the N entries of row i; no scale or shift.
//
// A row's statistics need the whole row, which spans many tiles, so the normalisation is a second
// pass.  What is fused is the reduction: the ring kernels' EPI == 2 epilogue writes z UNROUNDED
// (fp32) and, from the registers that hold it, leaves per row and wave-wide slice of columns the
// slice's mean and its sum of squared deviations from that mean.  gln_finish_kernel then merges a
// row's slices (fp64, pairwise-update formula, fixed order), and streams z once: subtract,
// scale, round ONCE to the storage type.  fp32 storage: z sits in Y itself and is normalised in
// place; 16-bit storage: z sits in the workspace (4 bytes per entry) and Y receives 16-bit values,
// so the product is never rounded to 16 bits before it is normalised.
// Fallback (shapes the ring kernels do not take): a workgroup per row forms the row's z in fp32,
// one column per thread; the finishing kernel then takes the row's statistics itself (two passes).
#include "kernel_ring_f32.hpp"

namespace optiml {
namespace {

template <typename E> __device__ __forceinline__ float widen_ln(E v);
template <> __device__ __forceinline__ float widen_ln<float>(float v) { return v; }
template <> __device__ __forceinline__ float widen_ln<unsigned short>(unsigned short v) { return bf16_to_f32(v); }
template <> __device__ __forceinline__ float widen_ln<_Float16>(_Float16 v) { return (float)v; }

// Fallback: workgroup = row i; thread t forms z_ij for j = t, t + 256, ... (guarded scalar loads, any
// layout and alignment, K = 0 gives the bias)
template <typename E>
__global__ __launch_bounds__(256) void gln_fallback_kernel(Problem p, float *Z, int64_t ldz)
{
    const int64_t i = blockIdx.x;
    const E *A = static_cast<const E *>(p.A), *B = static_cast<const E *>(p.B);
    const bool a_col = (p.layout & 2) != 0, b_col = (p.layout & 1) != 0;
    for (int64_t j = threadIdx.x; j < p.N; j += 256) {
        float z = 0.0f;
        for (int64_t k = 0; k < p.K; ++k) {
            const float a = widen_ln<E>(a_col ? A[k * p.lda + i] : A[i * p.lda + k]);
            const float b = widen_ln<E>(b_col ? B[j * p.ldb + k] : B[k * p.ldb + j]);
            z = fmaf(a, b, z);
        }
        Z[i * ldz + j] = z + (p.bias ? p.bias[j] : 0.0f);
    }
}

// (count, mean, sum of squared deviations) of a set of values; merge of two disjoint sets
struct Moments { double n, mean, m2; };
__device__ __forceinline__ Moments merge(const Moments &a, const Moments &b)
{
    if (b.n == 0.0) return a;
    if (a.n == 0.0) return b;
    const double n = a.n + b.n, d = b.mean - a.mean;
    return Moments{n, a.mean + d * (b.n / n), a.m2 + b.m2 + d * d * (a.n * b.n / n)};
}

template <int DT> struct OutType { typedef unsigned short type; };
template <> struct OutType<DT_F32> { typedef float type; };

template <int DT> __device__ __forceinline__ typename OutType<DT>::type round_out(double v)
{
    if constexpr (DT == DT_F32) return (float)v;
    else return to_16<DT>((float)v);
}

// One wave per row (four rows per workgroup).  The row's moments: from the `slices` pairs the
// contraction left (slice q holds columns q * width ..., pairs[q * M + i] = (mean, m2)), lane l
// merging slices l, l + 64, ... in that order, then a butterfly in which both partners merge (lower
// lane's set, higher lane's set) so that every lane ends with the same bits; or, with slices == 0,
// from two passes over z itself (mean first, then squared deviations from it).  Then one pass over
// the row: y = (z - mean) * rstd in fp64, rounded once.  Z and Y may be the same fp32 array.
template <int DT>
__global__ __launch_bounds__(256) void gln_finish_kernel(const float *Z, int64_t ldz, typename OutType<DT>::type *Y, int64_t ldy,
                                                        int64_t M, int64_t N, const ring::floatx2 *pairs, int64_t slices,
                                                        int64_t width, double eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= M) return;
    const float *z = Z + i * ldz;
    Moments mo{0.0, 0.0, 0.0};
    if (slices > 0) {
        for (int64_t q = lane; q < slices; q += 64) {
            const int64_t left = N - q * width;
            const double cnt = (double)(left >= width ? width : left > 0 ? left : 0);
            const ring::floatx2 pr = pairs[q * M + i];
            mo = merge(mo, Moments{cnt, (double)pr[0], (double)pr[1]});
        }
    } else {
        double s = 0.0, cnt = 0.0;
        for (int64_t j = lane; j < N; j += 64) { s += (double)z[j]; cnt += 1.0; }
        const double mean = cnt > 0.0 ? s / cnt : 0.0;
        double q = 0.0;
        for (int64_t j = lane; j < N; j += 64) { const double d = (double)z[j] - mean; q += d * d; }
        mo = Moments{cnt, mean, q};
    }
#pragma unroll
    for (int step = 1; step < 64; step <<= 1) {
        Moments other;
        other.n = __shfl_xor(mo.n, step, 64);
        other.mean = __shfl_xor(mo.mean, step, 64);
        other.m2 = __shfl_xor(mo.m2, step, 64);
        mo = (lane & step) ? merge(other, mo) : merge(mo, other);
    }
    const double mean = mo.mean, rstd = 1.0 / sqrt(mo.m2 / (double)N + eps);
    typename OutType<DT>::type *y = Y + i * ldy;
    const bool vec = (ldz % 4 == 0) && (ldy % 8 == 0) && ((reinterpret_cast<uintptr_t>(Z) & 15) == 0) &&
                     ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
    int64_t j0 = 0;
    if (vec) {
        // four floats per lane and step, 1 KiB of the row per wave and step
        typedef float f4 __attribute__((ext_vector_type(4)));
        for (; j0 + 256 <= N; j0 += 256) {
            const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(z + j0) + lane);
            if constexpr (DT == DT_F32) {
                f4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (float)(((double)v[e] - mean) * rstd);
                __builtin_nontemporal_store(o, reinterpret_cast<f4 *>(y + j0) + lane);
            } else {
                typedef unsigned int u2 __attribute__((ext_vector_type(2)));
                const u2 o = u2{pack2_16<DT>((float)(((double)v[0] - mean) * rstd), (float)(((double)v[1] - mean) * rstd)),
                                pack2_16<DT>((float)(((double)v[2] - mean) * rstd), (float)(((double)v[3] - mean) * rstd))};
                __builtin_nontemporal_store(o, reinterpret_cast<u2 *>(y + j0) + lane);
            }
        }
    }
    for (int64_t j = j0 + lane; j < N; j += 64) y[j] = round_out<DT>(((double)z[j] - mean) * rstd);
}

template <int DT, bool B_KC> using LnCfg = ring::Cfg<4, B_KC, true, 4, DT, 2>;
using LnCfgF32Rr = ringf::Cfg<128, 4, false, 2>;
using LnCfgF32Rc = ringf::Cfg<128, 4, true, 2>;

template <class C>
hipError_t launch_ring_ln(const Problem &p, float *Z, int64_t ldz, float *pairs, hipStream_t stream)
{
    ring::Params q;
    q.M = p.M; q.N = p.N; q.K = p.K; q.batch = 1;
    q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = 0;
    q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = 0;
    q.bias = p.bias; q.strideBias = 0;
    q.C = reinterpret_cast<char *>(Z); q.ldc = ldz; q.strideC = 0;
    if constexpr (!std::is_same<C, LnCfgF32Rr>::value && !std::is_same<C, LnCfgF32Rc>::value) {
        // the 16-bit kernels also take batches (Z slabs p.strideC floats apart): how the k-split partial
        // products of launch_unrounded_products are formed
        q.batch = p.batch; q.strideA = p.strideA; q.strideB = p.strideB; q.strideBias = p.strideBias; q.strideC = p.strideC;
    }
    q.tiles_m = (p.M + C::BM - 1) / C::BM;
    q.tiles_n = (p.N + C::BN - 1) / C::BN;
    q.act = ACT_NONE;
    q.labels = nullptr; q.picked = pairs; q.bias_row = 0;
    if (q.tiles_m * q.tiles_n * q.batch > 0x7fffffffLL) return hipErrorInvalidValue;     // the grid is 32-bit
    if constexpr (std::is_same<C, LnCfgF32Rr>::value || std::is_same<C, LnCfgF32Rc>::value) {
        hipLaunchKernelGGL(ringf::gemm_ring_f32_kernel<C>, dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(C::THREADS), 0, stream, q);
    } else {
        hipLaunchKernelGGL(ring::gemm_ring_kernel<C>, dim3((unsigned)(q.tiles_m * q.tiles_n * q.batch)), dim3(C::THREADS), 0, stream, q);
    }
    return hipGetLastError();
}

bool ring_takes_ln(const Problem &p)
{
    if (p.dtype == DT_BF16) return p.b_col() ? ring::supports<LnCfg<DT_BF16, true>>(p) : ring::supports<LnCfg<DT_BF16, false>>(p);
    if (p.dtype == DT_F16) return p.b_col() ? ring::supports<LnCfg<DT_F16, true>>(p) : ring::supports<LnCfg<DT_F16, false>>(p);
    return p.b_col() ? ringf::supports<LnCfgF32Rc>(p) : ringf::supports<LnCfgF32Rr>(p);
}

size_t align256_ln(size_t x) { return (x + 255) & ~size_t(255); }

}  // namespace

// The unrounded fp32 products A.B (+ bias) of p.batch problems of 16-bit operands, A row-major, that the ring kernel
// takes: slab b of Z (pitch ldz, p.strideC floats apart) = A_b . B_b.  `pairs` receives the row statistics the kernel
// also forms, 2 * 4 * ceil(N / 256) * M floats per batch; a caller that splits a contraction along k ignores them.
bool unrounded_products_supported(const Problem &p)
{
    Problem q = p;
    q.batch = 1; q.strideA = q.strideB = q.strideBias = q.strideC = 0;
    q.C = const_cast<void *>(p.A); q.ldc = 0;
    return (p.dtype == DT_BF16 || p.dtype == DT_F16) && p.K > 0 && !p.a_col() && ring_takes_ln(q);
}

hipError_t launch_unrounded_products(const Problem &p, float *Z, int64_t ldz, float *pairs, hipStream_t stream)
{
    if (p.dtype == DT_BF16)
        return p.b_col() ? launch_ring_ln<LnCfg<DT_BF16, true>>(p, Z, ldz, pairs, stream)
                         : launch_ring_ln<LnCfg<DT_BF16, false>>(p, Z, ldz, pairs, stream);
    return p.b_col() ? launch_ring_ln<LnCfg<DT_F16, true>>(p, Z, ldz, pairs, stream)
                     : launch_ring_ln<LnCfg<DT_F16, false>>(p, Z, ldz, pairs, stream);
}

// 0: a ring kernel with the statistics epilogue, 1: row-per-workgroup fallback.  p.C / p.ldc are Y.
int linear_ln_path(const Problem &p)
{
    Problem q = p;
    q.batch = 1; q.strideC = 0;
    if (p.dtype != DT_F32) {                  // the ring kernel writes fp32 z into the workspace, not into Y
        q.C = const_cast<void *>(p.A);
        q.ldc = 0;
    }
    return p.K > 0 && !p.a_col() && ring_takes_ln(q) ? 0 : 1;
}

hipError_t launch_linear_ln(const Problem &p, double eps, hipStream_t stream)
{
    const int path = linear_ln_path(p);
    const bool f32 = p.dtype == DT_F32;
    const int64_t width = f32 ? 32 : 64;
    const int64_t slices = path != 0 ? 0 : f32 ? ((p.N + 127) / 128) * 4 : ((p.N + 255) / 256) * 4;
    const int64_t ldz = f32 ? p.ldc : (p.N + 3) / 4 * 4;
    const size_t z_bytes = f32 ? 0 : align256_ln(sizeof(float) * (size_t)p.M * (size_t)ldz);
    const size_t pair_bytes = align256_ln(sizeof(float) * 2 * (size_t)slices * (size_t)p.M);
    float *Z = static_cast<float *>(p.C), *pairs = nullptr;
    if (z_bytes + pair_bytes > 0) {
        void *ws = nullptr;
        hipError_t e = workspace(z_bytes + pair_bytes, &ws, stream);
        if (e != hipSuccess) return e;
        if (!f32) Z = static_cast<float *>(ws);
        pairs = reinterpret_cast<float *>(static_cast<char *>(ws) + z_bytes);
    }
    hipError_t e = hipSuccess;
    if (path == 0) {
        if (p.dtype == DT_BF16)
            e = p.b_col() ? launch_ring_ln<LnCfg<DT_BF16, true>>(p, Z, ldz, pairs, stream)
                          : launch_ring_ln<LnCfg<DT_BF16, false>>(p, Z, ldz, pairs, stream);
        else if (p.dtype == DT_F16)
            e = p.b_col() ? launch_ring_ln<LnCfg<DT_F16, true>>(p, Z, ldz, pairs, stream)
                          : launch_ring_ln<LnCfg<DT_F16, false>>(p, Z, ldz, pairs, stream);
        else
            e = p.b_col() ? launch_ring_ln<LnCfgF32Rc>(p, Z, ldz, pairs, stream)
                          : launch_ring_ln<LnCfgF32Rr>(p, Z, ldz, pairs, stream);
    } else {
        if (p.M > 0x7fffffffLL) return hipErrorInvalidValue;
        const dim3 grid((unsigned)p.M);
        if (f32)
            hipLaunchKernelGGL(gln_fallback_kernel<float>, grid, dim3(256), 0, stream, p, Z, ldz);
        else if (p.dtype == DT_F16)
            hipLaunchKernelGGL(gln_fallback_kernel<_Float16>, grid, dim3(256), 0, stream, p, Z, ldz);
        else
            hipLaunchKernelGGL(gln_fallback_kernel<unsigned short>, grid, dim3(256), 0, stream, p, Z, ldz);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    const int64_t blocks = (p.M + 3) / 4;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const ring::floatx2 *pr = reinterpret_cast<const ring::floatx2 *>(pairs);
    if (f32)
        hipLaunchKernelGGL(gln_finish_kernel<DT_F32>, dim3((unsigned)blocks), dim3(256), 0, stream, Z, ldz,
                           static_cast<float *>(p.C), p.ldc, p.M, p.N, pr, slices, width, eps);
    else if (p.dtype == DT_F16)
        hipLaunchKernelGGL(gln_finish_kernel<DT_F16>, dim3((unsigned)blocks), dim3(256), 0, stream, Z, ldz,
                           static_cast<unsigned short *>(p.C), p.ldc, p.M, p.N, pr, slices, width, eps);
    else
        hipLaunchKernelGGL(gln_finish_kernel<DT_BF16>, dim3((unsigned)blocks), dim3(256), 0, stream, Z, ldz,
                           static_cast<unsigned short *>(p.C), p.ldc, p.M, p.N, pr, slices, width, eps);
    return hipGetLastError();
}

}  // namespace optiml

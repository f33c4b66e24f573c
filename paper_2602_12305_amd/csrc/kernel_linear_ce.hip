// The contraction feeding the cross-entropy (paper Table 4, task 2 into task 17) without the
// logits ever reaching memory:
//     loss = (1/M) sum_i [ log sum_j exp(z_ij) - z_{i, y_i} ],   z = A.B + bias  (M rows, N classes)
//
// Fast path (A row-major, shapes the ring kernels take): the bf16 / fp16 or the fp32 ring kernel
// with its log-sum-exp epilogue - every wave reduces the 64 (fp32: 32) columns it holds of each
// of its rows to a (maximum, sum of exponentials) pair, in registers, and the lane that holds the
// label's column hands out that logit.  What reaches memory is 8 bytes per row and 64 (32)
// columns instead of the logits.  Fallback (everything else): one workgroup per row forms the row's
// logits one column per thread in fp32 and reduces them the same way.  Both are followed by
// lce_rows_kernel (16 threads per row merge the row's pairs in fp64 in a fixed order, form the
// row loss, and a workgroup adds its 16 rows in row order) and lce_mean_kernel (adds the workgroups' sums in
// order, divides by M, rounds once to float).
#include "kernel_ring_f32.hpp"

namespace optiml {
namespace {

constexpr int kRowsPerBlock = 16, kGroups = 16;     // rows per workgroup of lce_rows_kernel, threads per row

template <typename E> __device__ __forceinline__ float widen_ce(E v);
template <> __device__ __forceinline__ float widen_ce<float>(float v) { return v; }
template <> __device__ __forceinline__ float widen_ce<unsigned short>(unsigned short v) { return bf16_to_f32(v); }
template <> __device__ __forceinline__ float widen_ce<_Float16>(_Float16 v) { return (float)v; }

// merge of two (maximum, sum of exp(. - maximum)) pairs; an empty side has sum 0
__device__ __forceinline__ void merge_pair(float &m, float &s, float m2, float s2)
{
    if (s2 == 0.0f) return;
    if (s == 0.0f) { m = m2; s = s2; return; }
    const float hi = m > m2 ? m : m2;
    s = s * __builtin_amdgcn_exp2f((m - hi) * 1.44269504088896341f) + s2 * __builtin_amdgcn_exp2f((m2 - hi) * 1.44269504088896341f);
    m = hi;
}

// Fallback: workgroup = row i; thread t forms z_ij for j = t, t + 256, ... (guarded scalar loads,
// any layout and alignment), keeps a running pair, the workgroup merges in a fixed order.
template <typename E>
__global__ __launch_bounds__(256) void lce_fallback_kernel(Problem p, const int *labels, float *part, float *picked)
{
    __shared__ float sm[256], ss[256];
    const int64_t i = blockIdx.x;
    const E *A = static_cast<const E *>(p.A), *B = static_cast<const E *>(p.B);
    const bool a_col = (p.layout & 2) != 0, b_col = (p.layout & 1) != 0;
    const int64_t label = labels[i];
    float m = 0.0f, s = 0.0f;
    for (int64_t j = threadIdx.x; j < p.N; j += 256) {
        float z = p.bias ? p.bias[j] : 0.0f;
        for (int64_t k = 0; k < p.K; ++k) {
            const float a = widen_ce<E>(a_col ? A[k * p.lda + i] : A[i * p.lda + k]);
            const float b = widen_ce<E>(b_col ? B[j * p.ldb + k] : B[k * p.ldb + j]);
            z = fmaf(a, b, z);
        }
        if (j == label) picked[i] = z;
        merge_pair(m, s, z, 1.0f);
    }
    sm[threadIdx.x] = m; ss[threadIdx.x] = s;
    __syncthreads();
    for (int step = 128; step > 0; step >>= 1) {
        if ((int)threadIdx.x < step) {
            merge_pair(m, s, sm[threadIdx.x + step], ss[threadIdx.x + step]);
            sm[threadIdx.x] = m; ss[threadIdx.x] = s;
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) { part[2 * i] = m; part[2 * i + 1] = s; }
}

// A workgroup owns kRowsPerBlock rows; thread (row r, group g) merges slices g, g + kGroups, ... of
// its row in fp64 (pairs are slice-major: row i, slice q at part[2 (q M + i)], so the threads of
// one group read consecutive rows), then the row's groups are merged in group order,
// loss_i = log(S) + (max - z_label) (a label outside [0, N) gives NaN), and the rows are added in
// row order.  row_loss, if given, receives every row's loss rounded once to float.
__global__ __launch_bounds__(kRowsPerBlock * kGroups) void lce_rows_kernel(const float *part, int64_t slices, int64_t M,
                                                                          int64_t N, const int *labels, const float *picked,
                                                                          double *block_sums, float *row_loss)
{
    __shared__ double sh_hi[kGroups][kRowsPerBlock], sh_s[kGroups][kRowsPerBlock], sh_loss[kRowsPerBlock];
    const int r = threadIdx.x % kRowsPerBlock, g = threadIdx.x / kRowsPerBlock;
    const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + r;
    double hi = 0.0, S = 0.0;                       // S == 0: nothing merged yet
    if (i < M)
        for (int64_t q = g; q < slices; q += kGroups) {
            const float2 pr = *reinterpret_cast<const float2 *>(part + 2 * (q * M + i));
            if (pr.y == 0.0f) continue;                                  // a slice wholly past column N
            const double m = (double)pr.x;
            if (S == 0.0) { hi = m; S = (double)pr.y; }
            else if (m > hi) { S = S * exp(hi - m) + (double)pr.y; hi = m; }
            else S += (double)pr.y * exp(m - hi);
        }
    sh_hi[g][r] = hi; sh_s[g][r] = S;
    __syncthreads();
    if (g == 0) {
        for (int k = 1; k < kGroups; ++k) {
            const double m = sh_hi[k][r], s2 = sh_s[k][r];
            if (s2 == 0.0) continue;
            if (S == 0.0) { hi = m; S = s2; }
            else if (m > hi) { S = S * exp(hi - m) + s2; hi = m; }
            else S += s2 * exp(m - hi);
        }
        double loss = 0.0;
        if (i < M) {
            const int label = labels[i];
            loss = (label < 0 || label >= N) ? (double)__builtin_nanf("") : log(S) + (hi - (double)picked[i]);
            if (row_loss) row_loss[i] = (float)loss;
        }
        sh_loss[r] = loss;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int k = 0; k < kRowsPerBlock; ++k) t += sh_loss[k];
        block_sums[blockIdx.x] = t;
    }
}

// lane t adds the workgroup sums t, t + 64, ... in that order, lane 0 the 64 lane sums in lane order
__global__ __launch_bounds__(64) void lce_mean_kernel(const double *block_sums, int64_t blocks, int64_t M, float *loss)
{
    __shared__ double sh[64];
    double t = 0.0;
    for (int64_t b = threadIdx.x; b < blocks; b += 64) t += block_sums[b];
    sh[threadIdx.x] = t;
    __syncthreads();
    if (threadIdx.x != 0) return;
    double total = 0.0;
    for (int k = 0; k < 64; ++k) total += sh[k];
    *loss = (float)(M > 0 ? total / (double)M : 0.0);
}

template <int DT, bool B_KC> using LseCfg = ring::Cfg<4, B_KC, true, 4, DT, 1>;

using LseCfgF32Rr = ringf::Cfg<128, 4, false, 1>;
using LseCfgF32Rc = ringf::Cfg<128, 4, true, 1>;

template <class C>
hipError_t launch_ring_lse(const Problem &p, const int *labels, float *part, float *picked, hipStream_t stream)
{
    ring::Params q;
    q.M = p.M; q.N = p.N; q.K = p.K; q.batch = 1;
    q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = 0;
    q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = 0;
    q.bias = p.bias; q.strideBias = 0;
    q.C = reinterpret_cast<char *>(part); q.ldc = p.N; q.strideC = 0;
    q.tiles_m = (p.M + C::BM - 1) / C::BM;
    q.tiles_n = (p.N + C::BN - 1) / C::BN;
    q.act = ACT_NONE;
    q.labels = labels; q.picked = picked; q.bias_row = 0;
    if (q.tiles_m * q.tiles_n > 0x7fffffffLL) return hipErrorInvalidValue;     // the grid is 32-bit
    if constexpr (std::is_same<C, LseCfgF32Rr>::value || std::is_same<C, LseCfgF32Rc>::value) {
        hipLaunchKernelGGL(ringf::gemm_ring_f32_kernel<C>, dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(C::THREADS), 0, stream, q);
    } else {
        hipLaunchKernelGGL(ring::gemm_ring_kernel<C>, dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(C::THREADS), 0, stream, q);
    }
    return hipGetLastError();
}

// the problem as the ring kernel's support check wants it (C stands for the pair buffer)
bool ring_takes(const Problem &p)
{
    if (p.dtype == DT_BF16) return p.b_col() ? ring::supports<LseCfg<DT_BF16, true>>(p) : ring::supports<LseCfg<DT_BF16, false>>(p);
    if (p.dtype == DT_F16) return p.b_col() ? ring::supports<LseCfg<DT_F16, true>>(p) : ring::supports<LseCfg<DT_F16, false>>(p);
    return p.b_col() ? ringf::supports<LseCfgF32Rc>(p) : ringf::supports<LseCfgF32Rr>(p);
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

}  // namespace

// 0: a ring kernel with the log-sum-exp epilogue, 1: row-per-workgroup fallback
int linear_ce_path(const Problem &p)
{
    Problem q = p;
    q.C = const_cast<void *>(p.A);            // any 16-byte aligned address: C is not written on this path
    q.ldc = 0; q.strideC = 0; q.batch = 1;    // no C row pitch to keep aligned either
    return p.K > 0 && !p.a_col() && ring_takes(q) ? 0 : 1;
}

hipError_t launch_linear_ce(const Problem &p, const int *labels, float *loss, float *row_loss, hipStream_t stream)
{
    const int path = linear_ce_path(p);
    // a pair per row and wave-wide slice of columns: 4 slices per 256-column (fp32: 128-column) tile
    const int64_t slices = path != 0 ? 1 : p.dtype == DT_F32 ? ((p.N + 127) / 128) * 4 : ((p.N + 255) / 256) * 4;
    const int64_t blocks = (p.M + kRowsPerBlock - 1) / kRowsPerBlock;
    const size_t part_bytes = align256(sizeof(float) * 2 * (size_t)slices * p.M);
    const size_t pick_bytes = align256(sizeof(float) * (size_t)p.M);
    void *ws = nullptr;
    hipError_t e = workspace(part_bytes + pick_bytes + sizeof(double) * (size_t)blocks, &ws, stream);
    if (e != hipSuccess) return e;
    float *part = static_cast<float *>(ws);
    float *picked = reinterpret_cast<float *>(static_cast<char *>(ws) + part_bytes);
    double *block_sums = reinterpret_cast<double *>(static_cast<char *>(ws) + part_bytes + pick_bytes);
    if (p.M == 0) {                                   // no rows: the mean of nothing is 0
        if (!loss) return hipSuccess;
        hipLaunchKernelGGL(lce_mean_kernel, dim3(1), dim3(64), 0, stream, block_sums, 0, 0, loss);
        return hipGetLastError();
    }
    if (path == 0) {
        if (p.dtype == DT_BF16)
            e = p.b_col() ? launch_ring_lse<LseCfg<DT_BF16, true>>(p, labels, part, picked, stream)
                          : launch_ring_lse<LseCfg<DT_BF16, false>>(p, labels, part, picked, stream);
        else if (p.dtype == DT_F16)
            e = p.b_col() ? launch_ring_lse<LseCfg<DT_F16, true>>(p, labels, part, picked, stream)
                          : launch_ring_lse<LseCfg<DT_F16, false>>(p, labels, part, picked, stream);
        else
            e = p.b_col() ? launch_ring_lse<LseCfgF32Rc>(p, labels, part, picked, stream)
                          : launch_ring_lse<LseCfgF32Rr>(p, labels, part, picked, stream);
    } else {
        if (p.M > 0x7fffffffLL) return hipErrorInvalidValue;
        const dim3 grid((unsigned)p.M);
        if (p.dtype == DT_F32)
            hipLaunchKernelGGL(lce_fallback_kernel<float>, grid, dim3(256), 0, stream, p, labels, part, picked);
        else if (p.dtype == DT_F16)
            hipLaunchKernelGGL(lce_fallback_kernel<_Float16>, grid, dim3(256), 0, stream, p, labels, part, picked);
        else
            hipLaunchKernelGGL(lce_fallback_kernel<unsigned short>, grid, dim3(256), 0, stream, p, labels, part, picked);
        e = hipGetLastError();
    }
    if (e != hipSuccess) return e;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(lce_rows_kernel, dim3((unsigned)blocks), dim3(kRowsPerBlock * kGroups), 0, stream, part, slices, p.M, p.N, labels,
                       picked, block_sums, row_loss);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (!loss) return hipSuccess;
    hipLaunchKernelGGL(lce_mean_kernel, dim3(1), dim3(64), 0, stream, block_sums, blocks, p.M, loss);
    return hipGetLastError();
}

}  // namespace optiml

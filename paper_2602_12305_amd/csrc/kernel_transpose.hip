// Fast path for a column-major A: the ring kernels want A with k contiguous, so A (stored
// [K][M], M contiguous) is first copied into the library's workspace as [M][K], then the ring
// kernel of the same dtype and B layout runs on the copy.  The copy moves 2 M K elements against
// the contraction's 2 M N K flops: from N of about a thousand on it costs a few per cent of the
// time and the ring kernel is about twice as fast as the staged tile kernel that otherwise
// serves this layout.
//
// transpose_kernel: a workgroup owns a 64 x 64 element tile; 16-byte reads along the source's
// contiguous direction, element-wise writes into a padded LDS tile, 16-byte reads of LDS along
// the other direction, 16-byte writes.  Both extents must be whole 16-byte chunks.
#include "common.hpp"

namespace optiml {
namespace {

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// dst[b][c][r] = src[b][r * ld + c] for r < rows, c < cols; E = element type (2 or 4 bytes)
template <typename E>
__global__ __launch_bounds__(256) void transpose_kernel(const E *__restrict__ src, E *__restrict__ dst, int64_t rows,
                                                        int64_t cols, int64_t ld, int64_t stride_src, int64_t tiles_c,
                                                        int64_t tiles_r)
{
    constexpr int T = 64, CH = 16 / sizeof(E), CPR = T / CH;        // chunks per tile row
    __shared__ E tile[T][T + CH];                                   // [c][r], rows kept 16-byte aligned
    const int64_t b = blockIdx.x / (tiles_c * tiles_r), t = blockIdx.x % (tiles_c * tiles_r);
    const int64_t r0 = (t / tiles_c) * T, c0 = (t % tiles_c) * T;
    const E *s = src + b * stride_src;
    E *d = dst + b * rows * cols;
    for (int id = threadIdx.x; id < T * CPR; id += 256) {
        const int r = id / CPR, ch = id % CPR;
        if (r0 + r < rows && c0 + ch * CH < cols) {
            const uintx4 v = *reinterpret_cast<const uintx4 *>(s + (r0 + r) * ld + c0 + ch * CH);
            E e[CH];
            __builtin_memcpy(e, &v, 16);
#pragma unroll
            for (int i = 0; i < CH; ++i) tile[ch * CH + i][r] = e[i];
        }
    }
    __syncthreads();
    for (int id = threadIdx.x; id < T * CPR; id += 256) {
        const int c = id / CPR, ch = id % CPR;
        if (c0 + c < cols && r0 + ch * CH < rows)
            *reinterpret_cast<uintx4 *>(d + (c0 + c) * rows + r0 + ch * CH) =
                *reinterpret_cast<const uintx4 *>(&tile[c][ch * CH]);
    }
}

// the problem the ring kernel sees: A row-major in the workspace
Problem with_row_major_a(const Problem &p, const void *a)
{
    Problem q = p;
    q.A = a;
    q.lda = p.K;
    q.strideA = p.M * p.K;
    q.layout = p.layout & 1;
    return q;
}

const Variant *ring_for(const Problem &q)
{
    const Variant *t = tile_variants();
    const Variant *first = nullptr;
    for (int i = 0; i < kNumTileVariants; ++i) {
        if (t[i].name[0] != 'r' || !t[i].supports(q)) continue;        // "ring..." / "ringp..."
        if (t[i].prefers && t[i].prefers(q)) return &t[i];
        if (!first) first = &t[i];
    }
    return first;
}

bool xa_supports(const Problem &p)
{
    if (!p.a_col() || p.K < 1 || !vector_friendly(p)) return false;
    const int ch = 16 / p.esize();
    if (p.M % ch != 0 || p.K % ch != 0) return false;
    if (p.batch * ((p.M + 63) / 64) * ((p.K + 63) / 64) > 0x7fffffffLL) return false;
    return ring_for(with_row_major_a(p, reinterpret_cast<const void *>(uintptr_t(256)))) != nullptr;
}

// worth the copy: enough columns to amortise it, and enough work to fill the chip with ring tiles
bool xa_prefers(const Problem &p)
{
    return p.N >= 1024 && p.batch * ((p.M + 127) / 128) * ((p.N + 127) / 128) >= 256;
}

hipError_t xa_launch(const Problem &p, hipStream_t s)
{
    void *ws = nullptr;
    hipError_t e = workspace((size_t)p.batch * p.M * p.K * p.esize(), &ws);
    if (e != hipSuccess) return e;
    const Problem q = with_row_major_a(p, ws);
    const Variant *ring = ring_for(q);
    if (!ring) return hipErrorInvalidValue;
    const int64_t tiles_c = (p.M + 63) / 64, tiles_r = (p.K + 63) / 64;
    const dim3 grid((unsigned)(p.batch * tiles_c * tiles_r));
    if (p.esize() == 4)
        hipLaunchKernelGGL(transpose_kernel<uint32_t>, grid, dim3(256), 0, s, static_cast<const uint32_t *>(p.A),
                           static_cast<uint32_t *>(ws), p.K, p.M, p.lda, p.strideA, tiles_c, tiles_r);
    else
        hipLaunchKernelGGL(transpose_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t *>(p.A),
                           static_cast<uint16_t *>(ws), p.K, p.M, p.lda, p.strideA, tiles_c, tiles_r);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    return ring->launch(q, s);
}

}  // namespace

const Variant *transpose_variants()
{
    static const Variant v[] = {{"xa_ring", xa_supports, xa_launch, 256, 256,
                                 reinterpret_cast<const void *>(&transpose_kernel<uint16_t>), xa_prefers}};
    return v;
}
const int kNumTransposeVariants = 1;

}  // namespace optiml

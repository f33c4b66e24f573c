// Fast path for a column-major A: the ring kernels want A with k contiguous, so A (stored
// [K][M], M contiguous) is first copied into the library's workspace as [M][K], then the ring
// kernel of the same dtype and B layout runs on the copy.  The copy moves 2 M K elements against
// the contraction's 2 M N K flops: from N of about a thousand on it costs a few per cent of the
// time and the ring kernel is about twice as fast as the staged tile kernel that otherwise
// serves this layout.
//
// transpose_kernel: a workgroup owns a tile of 256 bytes x 256 bytes; 16-byte accesses on both
// sides of memory and an XOR-swizzled LDS tile in between.  Both extents must be whole 16-byte
// chunks.
#include "common.hpp"

namespace optiml {
namespace {

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// dst[b][c * ld_dst + r] = src[b][r * ld + c] for r < rows, c < cols (batches of the destination are
// cols * ld_dst apart); E = element type (2 or 4 bytes).  A tile is T x T elements with T = 256
// bytes / element size, so both sides move 256-byte row segments.  The tile sits in LDS
// untransposed, 16 chunks of 16 bytes per row, chunk ch of row r at position ch ^ ((r / CH) % 16):
// the 128-bit writes of a row are a permutation of its chunks, and in the read phase thread
// (c, k) gathers element c of rows CH k .. CH k + CH - 1, which for the 16 values of k lie in 16
// different chunk positions - no bank conflicts on either side.
template <typename E, int SEQ>
__global__ __launch_bounds__(256) void transpose_kernel(const E *__restrict__ src, E *__restrict__ dst, int64_t rows,
                                                        int64_t cols, int64_t ld, int64_t stride_src, int64_t tiles_c,
                                                        int64_t tiles_r, int64_t ld_dst)
{
    constexpr int CH = 16 / sizeof(E), T = 16 * CH;                  // elements per chunk, tile edge
    __shared__ __attribute__((aligned(16))) E tile[T][T];
    // A workgroup takes SEQ tiles side by side (the same rows of the source, consecutive 256-byte
    // pieces of them), one after the other: with two, the second tile's reads continue the DRAM
    // pages the first one opened (measured 399 against 415 us on 16384 x 16384 fp32; longer runs,
    // tiles below one another and register prefetch of the next tile gained nothing more).
    const int64_t groups_c = (tiles_c + SEQ - 1) / SEQ;
    const int64_t b = blockIdx.x / (groups_c * tiles_r), t = blockIdx.x % (groups_c * tiles_r);
    // Diagonal walk: workgroup t takes column group t % groups_c of row band (t / groups_c + that) %
    // tiles_r, so the workgroups that run together read, and write, at different offsets within a
    // row.  With a power-of-two pitch a row-major walk has them all at the same offset, i.e. on
    // the same few memory channels (measured 4.3 against 5.0 TB/s for an odd pitch).
    const int64_t gc = t % groups_c, tr = (t / groups_c + gc) % tiles_r;
    const int64_t r0 = tr * T;
    const E *s = src + b * stride_src;
    E *d = dst + b * cols * ld_dst;
    for (int q = 0; q < SEQ; ++q) {
        const int64_t c0 = (gc * SEQ + q) * T;
        if (c0 >= cols) break;                                       // the same for the whole workgroup
        if (q) __syncthreads();
        for (int id = threadIdx.x; id < T * 16; id += 256) {
            const int r = id >> 4, ch = id & 15;
            if (r0 + r < rows && c0 + ch * CH < cols)
                *reinterpret_cast<uintx4 *>(&tile[r][(ch ^ ((r / CH) & 15)) * CH]) =
                    __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(s + (r0 + r) * ld + c0 + ch * CH));
        }
        __syncthreads();
        for (int id = threadIdx.x; id < T * 16; id += 256) {
            const int c = id >> 4, k = id & 15;
            if (c0 + c < cols && r0 + k * CH < rows) {
                E e[CH];
                const int pos = (((c / CH) ^ k) * CH) + c % CH;
#pragma unroll
                for (int i = 0; i < CH; ++i) e[i] = tile[k * CH + i][pos];
                uintx4 v;
                __builtin_memcpy(&v, e, 16);
                __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(d + (c0 + c) * ld_dst + r0 + k * CH));
            }
        }
    }
}

// Launch of transpose_kernel: pairs of tiles per workgroup once that still leaves every compute
// unit several workgroups.  The caller has checked batch * tiles_c * tiles_r against the grid limit.
template <typename E>
hipError_t launch_transpose(const void *src, void *dst, int64_t batch, int64_t rows, int64_t cols, int64_t ld,
                            int64_t stride_src, int64_t ld_dst, hipStream_t s)
{
    const int64_t T = 256 / (int64_t)sizeof(E);
    const int64_t tiles_c = (cols + T - 1) / T, tiles_r = (rows + T - 1) / T;
    const int64_t pairs = batch * ((tiles_c + 1) / 2) * tiles_r;
    if (pairs >= 2048)
        hipLaunchKernelGGL((transpose_kernel<E, 2>), dim3((unsigned)pairs), dim3(256), 0, s, static_cast<const E *>(src),
                           static_cast<E *>(dst), rows, cols, ld, stride_src, tiles_c, tiles_r, ld_dst);
    else
        hipLaunchKernelGGL((transpose_kernel<E, 1>), dim3((unsigned)(batch * tiles_c * tiles_r)), dim3(256), 0, s,
                           static_cast<const E *>(src), static_cast<E *>(dst), rows, cols, ld, stride_src, tiles_c, tiles_r,
                           ld_dst);
    return hipGetLastError();
}

// Any shape, pitch and alignment: a 64 x 64 tile through a padded LDS tile, one element per access,
// consecutive threads on consecutive addresses on both sides.
template <typename E>
__global__ __launch_bounds__(256) void transpose_any_kernel(const E *__restrict__ src, E *__restrict__ dst, int64_t rows,
                                                            int64_t cols, int64_t ld, int64_t ld_dst, int64_t tiles_c)
{
    constexpr int T = 64;
    __shared__ E tile[T][T + 1];
    const int64_t r0 = (blockIdx.x / tiles_c) * T, c0 = (blockIdx.x % tiles_c) * T;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int r = ty; r < T; r += 4)
        if (r0 + r < rows && c0 + tx < cols) tile[r][tx] = src[(r0 + r) * ld + c0 + tx];
    __syncthreads();
    for (int c = ty; c < T; c += 4)
        if (c0 + c < cols && r0 + tx < rows) dst[(c0 + c) * ld_dst + r0 + tx] = tile[tx][c];
}

// the problem the second kernel sees: A row-major in the workspace
Problem with_row_major_a(const Problem &p, const void *a)
{
    Problem q = p;
    q.A = a;
    q.lda = p.K;
    q.strideA = p.M * p.K;
    q.layout = p.layout & 1;
    return q;
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

// The streaming kernels keep split-k partial sums in the workspace, behind the copy of A: at most
// 64 splits of [batch][blocks of 16 rows][16][N] floats.  Beyond this bound the copy is followed
// by a kernel that needs no scratch.
constexpr size_t kMaxPartialBytes = size_t(1) << 30;
size_t partial_bound(const Problem &p)
{
    return sizeof(float) * 64 * (size_t)p.batch * (size_t)((p.M + 15) / 16) * 16 * (size_t)p.N;
}

// the kernel that follows the copy: the dispatcher's choice for the row-major problem
int second_kernel(const Problem &p, double *us)
{
    const Problem q = with_row_major_a(p, reinterpret_cast<const void *>(uintptr_t(256)));
    const int id = select_variant(q, us, partial_bound(p) <= kMaxPartialBytes);
    const Variant *v = variant_at(id);
    return v && v->name[0] != 'g' ? id : -1;                   // not the guarded fallback: no gain in copying for it
}

bool xa_supports(const Problem &p)
{
    if (!p.a_col() || p.K < 1 || is_8bit(p.dtype) || !vector_friendly(p)) return false;
    const int ch = 16 / p.esize();
    if (p.M % ch != 0 || p.K % ch != 0) return false;
    const int64_t T = 256 / p.esize();
    if (p.batch * ((p.M + T - 1) / T) * ((p.K + T - 1) / T) > 0x7fffffffLL) return false;
    return second_kernel(p, nullptr) >= 0;
}

// the copy (read and write of A at about 5 TB/s, one launch) plus the second kernel
double xa_estimate(const Problem &p)
{
    double us = 1e30;
    if (second_kernel(p, &us) < 0) return 1e30;
    return us + 3.0 + 2.0 * (double)p.batch * (double)p.M * (double)p.K * p.esize() / 5.0e6;
}

hipError_t xa_launch(const Problem &p, hipStream_t s)
{
    const Variant *second = variant_at(second_kernel(p, nullptr));
    if (!second) return hipErrorInvalidValue;
    const size_t copy = align256((size_t)p.batch * p.M * p.K * p.esize());
    const size_t more = second->name[0] == 's' ? partial_bound(p) : 0;        // "skinny...": split-k partials
    void *ws = nullptr;
    hipError_t e = workspace(copy + more, &ws, s);
    if (e != hipSuccess) return e;
    const Problem q = with_row_major_a(p, ws);
    e = p.esize() == 4 ? launch_transpose<uint32_t>(p.A, ws, p.batch, p.K, p.M, p.lda, p.strideA, p.K, s)
                       : launch_transpose<uint16_t>(p.A, ws, p.batch, p.K, p.M, p.lda, p.strideA, p.K, s);
    if (e != hipSuccess) return e;
    const WorkspaceHead keep(copy);          // the second kernel's scratch, if any, goes behind the copy
    return second->launch(q, s);
}

// ---- 8-bit operands: the matrix-pipe kernel wants k contiguous in BOTH operands -----------------
// Whichever operand has k as its slow direction (A column-major: stored [K][M]; B row-major:
// stored [K][N]) is copied into the workspace with k contiguous, then the E4M3 ring kernel runs on
// the copies as an A-row-major, B-column-major problem.

template <typename E>
hipError_t copy_transposed(const void *src, void *dst, int64_t batch, int64_t rows, int64_t cols, int64_t ld, int64_t stride,
                           hipStream_t s)
{
    const int64_t T = 256 / (int64_t)sizeof(E);
    const int64_t tiles_c = (cols + T - 1) / T, tiles_r = (rows + T - 1) / T;
    if (batch * tiles_c * tiles_r > 0x7fffffffLL) return hipErrorInvalidValue;
    return launch_transpose<E>(src, dst, batch, rows, cols, ld, stride, rows, s);
}

Problem with_k_contiguous(const Problem &p, const void *a, const void *b)
{
    Problem q = p;
    if (p.a_col()) { q.A = a; q.lda = p.K; q.strideA = p.M * p.K; }
    if (!p.b_col()) { q.B = b; q.ldb = p.K; q.strideB = p.N * p.K; }
    q.layout = 1;
    return q;
}

// the kernel that follows the copies: the dispatcher's choice for the k-contiguous problem
const Variant *second_kernel_f8(const Problem &p)
{
    const void *fake = reinterpret_cast<const void *>(uintptr_t(256));
    const Variant *v = variant_at(select_variant(with_k_contiguous(p, fake, fake), nullptr, partial_bound(p) <= kMaxPartialBytes));
    return v && v->name[0] != 'g' ? v : nullptr;
}

bool x8_supports(const Problem &p)
{
    if (!is_f8(p.dtype) || (!p.a_col() && p.b_col()) || p.K < 1 || !vector_friendly(p)) return false;
    if (p.K % 16 != 0 || (p.a_col() && p.M % 16 != 0) || (!p.b_col() && p.N % 16 != 0)) return false;
    if (p.batch * ((p.M + 255) / 256 + (p.N + 255) / 256) * ((p.K + 255) / 256) > 0x7fffffffLL) return false;
    return second_kernel_f8(p) != nullptr;
}

// the alternative is the element-wise fallback: worth it as soon as there is a tile's worth of work
bool x8_prefers(const Problem &p) { return p.M * p.N >= 65536 && p.K >= 256; }

hipError_t x8_launch(const Problem &p, hipStream_t s)
{
    const Variant *second = second_kernel_f8(p);
    if (!second) return hipErrorInvalidValue;
    const size_t a_bytes = p.a_col() ? align256((size_t)p.batch * p.M * p.K) : 0;
    const size_t b_bytes = !p.b_col() ? align256((size_t)p.batch * p.N * p.K) : 0;
    const size_t more = second->name[0] == 's' ? partial_bound(p) : 0;        // "skinny...": split-k partials
    void *ws = nullptr;
    hipError_t e = workspace(a_bytes + b_bytes + more, &ws, s);
    if (e != hipSuccess) return e;
    void *wa = ws, *wb = static_cast<char *>(ws) + a_bytes;
    const Problem q = with_k_contiguous(p, wa, wb);
    if (p.a_col()) {
        e = copy_transposed<uint8_t>(p.A, wa, p.batch, p.K, p.M, p.lda, p.strideA, s);
        if (e != hipSuccess) return e;
    }
    if (!p.b_col()) {
        e = copy_transposed<uint8_t>(p.B, wb, p.batch, p.K, p.N, p.ldb, p.strideB, s);
        if (e != hipSuccess) return e;
    }
    const WorkspaceHead keep(a_bytes + b_bytes);     // the second kernel's scratch, if any, goes behind the copies
    return second->launch(q, s);
}

}  // namespace

// Table 4 task 8 as an operation of its own: dst (cols x rows, pitch ld_dst) = transpose of src
// (rows x cols, pitch ld_src), elements of 2 or 4 bytes.  Arguments already validated.
hipError_t launch_transpose(int64_t rows, int64_t cols, const void *src, int64_t ld_src, void *dst, int64_t ld_dst, int esize,
                            hipStream_t s)
{
    if (rows == 0 || cols == 0) return hipSuccess;
    const int64_t ch = 16 / esize;
    auto aligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    const bool fast = aligned(src) && aligned(dst) && rows % ch == 0 && cols % ch == 0 && ld_src % ch == 0 && ld_dst % ch == 0;
    const int64_t T = fast ? 256 / esize : 64;                       // tile edge of the kernel that will run
    const int64_t tiles_c = (cols + T - 1) / T, tiles_r = (rows + T - 1) / T;
    if (tiles_c * tiles_r > 0x7fffffffLL) return hipErrorInvalidValue;
    if (fast)
        return esize == 4 ? launch_transpose<uint32_t>(src, dst, 1, rows, cols, ld_src, 0, ld_dst, s)
                          : launch_transpose<uint16_t>(src, dst, 1, rows, cols, ld_src, 0, ld_dst, s);
    const dim3 grid((unsigned)(tiles_c * tiles_r));
    if (esize == 4)
        hipLaunchKernelGGL(transpose_any_kernel<uint32_t>, grid, dim3(256), 0, s, static_cast<const uint32_t *>(src),
                           static_cast<uint32_t *>(dst), rows, cols, ld_src, ld_dst, tiles_c);
    else
        hipLaunchKernelGGL(transpose_any_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t *>(src),
                           static_cast<uint16_t *>(dst), rows, cols, ld_src, ld_dst, tiles_c);
    return hipGetLastError();
}

const Variant *transpose_variants()
{
    static const Variant v[] = {{"xa_ring", xa_supports, xa_launch, 256, 256,
                                 reinterpret_cast<const void *>(&transpose_kernel<uint16_t, 2>), nullptr, true, xa_estimate},
                                {"xk_ring_f8", x8_supports, x8_launch, 256, 256,
                                 reinterpret_cast<const void *>(&transpose_kernel<uint8_t, 2>), x8_prefers, true}};
    return v;
}
const int kNumTransposeVariants = 2;

}  // namespace optiml

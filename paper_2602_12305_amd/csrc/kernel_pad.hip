// Problems no fast kernel takes as they are - an operand that is not 16-byte aligned, a leading
// dimension or K that is not a whole number of 16-byte chunks, an odd N with a row-major B - used to
// go to the element-wise fallback (about 50 TFLOP/s whatever the storage type).  Here they are
// copied into the workspace in the form every fast kernel likes: A as [M][Kp] and B as [N][Kp], k
// contiguous in both, Kp = K rounded up to a whole chunk with zeros behind K (zeros add nothing to
// a sum), the bias padded likewise; the dispatcher's choice for that problem writes a C with an
// aligned pitch into the workspace, and a last copy puts it where the caller wants it.  Four
// small kernels around the contraction: worth it from a few hundred rows and columns on.
#include "common.hpp"

namespace optiml {
namespace {

// dst[b][r][c] for r < rows, c < cols_dst: the source element (r, c), or zero for c >= cols.
// TRANS: the source is stored [cols][rows] (element (r, c) at src[c * ld_src + r]) and goes through
// a 64 x 64 LDS tile so that both sides are walked along their contiguous direction.
template <typename E, bool TRANS>
__global__ __launch_bounds__(256) void pad_copy_kernel(const E *__restrict__ src, int64_t ld_src, int64_t stride_src,
                                                       E *__restrict__ dst, int64_t ld_dst, int64_t stride_dst, int64_t rows,
                                                       int64_t cols, int64_t cols_dst, int64_t tiles_c)
{
    constexpr int T = 64;
    const int64_t r0 = (blockIdx.x / tiles_c) * T, c0 = (blockIdx.x % tiles_c) * T;
    const E *s = src + (int64_t)blockIdx.y * stride_src;
    E *d = dst + (int64_t)blockIdx.y * stride_dst;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    if (TRANS) {
        __shared__ E tile[T][T + 1];
        for (int cc = ty; cc < T; cc += 4) {
            const int64_t c = c0 + cc, r = r0 + tx;
            tile[cc][tx] = (c < cols && r < rows) ? s[c * ld_src + r] : E(0);
        }
        __syncthreads();
        for (int rr = ty; rr < T; rr += 4) {
            const int64_t r = r0 + rr, c = c0 + tx;
            if (r < rows && c < cols_dst) d[r * ld_dst + c] = tile[tx][rr];
        }
    } else {
        for (int rr = ty; rr < T; rr += 4) {
            const int64_t r = r0 + rr, c = c0 + tx;
            if (r < rows && c < cols_dst) d[r * ld_dst + c] = c < cols ? s[r * ld_src + c] : E(0);
        }
    }
}

template <typename E>
hipError_t pad_copy(const void *src, int64_t ld_src, int64_t stride_src, void *dst, int64_t ld_dst, int64_t stride_dst,
                    int64_t batch, int64_t rows, int64_t cols, int64_t cols_dst, bool trans, hipStream_t s)
{
    const int64_t tiles_c = (cols_dst + 63) / 64, tiles_r = (rows + 63) / 64;
    if (tiles_c * tiles_r > 0x7fffffffLL || batch > 65535) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(tiles_c * tiles_r), (unsigned)batch);
    if (trans)
        hipLaunchKernelGGL((pad_copy_kernel<E, true>), grid, dim3(256), 0, s, static_cast<const E *>(src), ld_src, stride_src,
                           static_cast<E *>(dst), ld_dst, stride_dst, rows, cols, cols_dst, tiles_c);
    else
        hipLaunchKernelGGL((pad_copy_kernel<E, false>), grid, dim3(256), 0, s, static_cast<const E *>(src), ld_src, stride_src,
                           static_cast<E *>(dst), ld_dst, stride_dst, rows, cols, cols_dst, tiles_c);
    return hipGetLastError();
}

hipError_t pad_copy_bytes(int esize, const void *src, int64_t ld_src, int64_t stride_src, void *dst, int64_t ld_dst,
                          int64_t stride_dst, int64_t batch, int64_t rows, int64_t cols, int64_t cols_dst, bool trans,
                          hipStream_t s)
{
    if (esize == 4) return pad_copy<uint32_t>(src, ld_src, stride_src, dst, ld_dst, stride_dst, batch, rows, cols, cols_dst, trans, s);
    if (esize == 2) return pad_copy<uint16_t>(src, ld_src, stride_src, dst, ld_dst, stride_dst, batch, rows, cols, cols_dst, trans, s);
    return pad_copy<uint8_t>(src, ld_src, stride_src, dst, ld_dst, stride_dst, batch, rows, cols, cols_dst, trans, s);
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }
int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

struct Plan {
    int64_t Kp, Np, nbias;                // padded K, pitch of the temporary C, entries of the padded bias
    size_t a_bytes, b_bytes, bias_bytes, c_bytes;
    size_t total() const { return a_bytes + b_bytes + bias_bytes + c_bytes; }
};

Plan plan_for(const Problem &p)
{
    Plan pl;
    pl.Kp = round_up(p.K, 16 / p.esize());
    pl.Np = round_up(p.N, 16 / p.csize());
    pl.nbias = round_up(p.bias_row ? p.M : p.N, 8);
    pl.a_bytes = align256((size_t)p.batch * p.M * pl.Kp * p.esize());
    pl.b_bytes = align256((size_t)p.batch * p.N * pl.Kp * p.esize());
    pl.bias_bytes = p.bias ? align256((size_t)p.batch * pl.nbias * 4) : 0;
    pl.c_bytes = align256((size_t)p.batch * p.M * pl.Np * p.csize());
    return pl;
}

// the problem the second kernel sees: k contiguous in both operands, everything aligned
Problem padded(const Problem &p, const Plan &pl, void *ws)
{
    char *w = static_cast<char *>(ws);
    Problem q = p;
    q.K = pl.Kp;
    q.A = w; q.lda = pl.Kp; q.strideA = p.M * pl.Kp;
    q.B = w + pl.a_bytes; q.ldb = pl.Kp; q.strideB = p.N * pl.Kp;
    q.bias = p.bias ? reinterpret_cast<const float *>(w + pl.a_bytes + pl.b_bytes) : nullptr;
    q.strideBias = pl.nbias;
    q.C = w + pl.a_bytes + pl.b_bytes + pl.bias_bytes; q.ldc = pl.Np; q.strideC = p.M * pl.Np;
    q.layout = 1;
    return q;
}

// split-k partial sums of a streaming second kernel go behind everything else in the workspace
constexpr size_t kMaxPartialBytes = size_t(1) << 30;
size_t partial_bound(const Problem &p)
{
    return sizeof(float) * 64 * (size_t)p.batch * (size_t)((p.M + 15) / 16) * 16 * (size_t)p.N;
}

thread_local bool tls_inside = false;            // the dispatcher asks this variant about the padded problem too

const Variant *second_kernel(const Problem &p, double *us)
{
    const Plan pl = plan_for(p);
    const Problem q = padded(p, pl, reinterpret_cast<void *>(uintptr_t(256)));
    tls_inside = true;
    const Variant *v = variant_at(select_variant(q, us, partial_bound(p) <= kMaxPartialBytes));
    tls_inside = false;
    return v && v->name[0] != 'g' ? v : nullptr;
}

// only problems the fast kernels do not take as they are
bool needs_padding(const Problem &p)
{
    const int64_t ch = 16 / p.esize();
    if (!vector_friendly(p) || p.K % ch != 0) return true;
    if (p.a_col() && p.M % ch != 0) return true;
    if (!p.b_col() && p.N % ch != 0) return true;
    return false;
}

bool pad_supports(const Problem &p)
{
    if (tls_inside || p.K < 1 || p.batch > 65535 || is_f6(p.dtype) || !needs_padding(p)) return false;   // (dense 6-bit codes: not whole bytes)
    return second_kernel(p, nullptr) != nullptr;
}

// five more launches and every operand moved twice more, by kernels that reach about 2 TB/s
double pad_estimate(const Problem &p)
{
    double us = 1e30;
    if (!second_kernel(p, &us)) return 1e30;
    const Plan pl = plan_for(p);
    return us + 15.0 + 2.0 * (double)pl.total() / 2.0e6;
}

hipError_t pad_launch(const Problem &p, hipStream_t s)
{
    const Variant *second = second_kernel(p, nullptr);
    if (!second) return hipErrorInvalidValue;
    const Plan pl = plan_for(p);
    const size_t more = second->name[0] == 's' ? partial_bound(p) : 0;        // "skinny...": split-k partials
    void *ws = nullptr;
    hipError_t e = workspace(pl.total() + more, &ws, s);
    if (e != hipSuccess) return e;
    const Problem q = padded(p, pl, ws);
    const int es = p.esize();
    // A: stored [M][K] or, column-major, [K][M]
    e = pad_copy_bytes(es, p.A, p.lda, p.strideA, const_cast<void *>(q.A), q.lda, q.strideA, p.batch, p.M, p.K, pl.Kp, p.a_col(), s);
    if (e != hipSuccess) return e;
    // B: stored [N][K] when column-major, else [K][N]
    e = pad_copy_bytes(es, p.B, p.ldb, p.strideB, const_cast<void *>(q.B), q.ldb, q.strideB, p.batch, p.N, p.K, pl.Kp, !p.b_col(), s);
    if (e != hipSuccess) return e;
    if (p.bias) {
        const int64_t n = p.bias_row ? p.M : p.N;
        e = pad_copy_bytes(4, p.bias, n, p.strideBias, const_cast<float *>(q.bias), pl.nbias, pl.nbias, p.batch, 1, n, pl.nbias, false, s);
        if (e != hipSuccess) return e;
    }
    {
        const WorkspaceHead keep(pl.total());    // the second kernel's scratch, if any, goes behind the copies
        e = second->launch(q, s);
    }
    if (e != hipSuccess) return e;
    return pad_copy_bytes(p.csize(), q.C, q.ldc, q.strideC, p.C, p.ldc, p.strideC, p.batch, p.M, p.N, p.N, false, s);
}

}  // namespace

const Variant *pad_variants()
{
    static const Variant v[] = {{"xpad", pad_supports, pad_launch, 256, 256,
                                 reinterpret_cast<const void *>(&pad_copy_kernel<uint16_t, false>), nullptr, true, pad_estimate}};
    return v;
}
const int kNumPadVariants = 1;

}  // namespace optiml

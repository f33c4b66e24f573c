// 6-bit operands (OCP E2M3 and E3M2) on the matrix pipe.
//
// The operands arrive densely packed: four elements in three bytes, a row of K elements in 3 K / 4
// bytes.  The 64-deep matrix instruction wants a lane's 32 values of k as 24 contiguous bytes in six
// registers; the ring kernel moves 16-byte chunks and reads 16-byte fragments, and 24 is not a
// multiple of 16.  So both operands are first copied into the workspace in SLOT form - every block of
// 32 elements in a 32-byte slot, the last 8 bytes zero - arranged per k-tile of 64 elements the way
// the 64-deep 8-bit kernel reads its fragments (a lane of half h takes chunks h and 2 + h of the 64
// bytes of its row): chunk 0 = bytes 0-15 of the first block, chunk 1 = bytes 0-15 of the second,
// chunk 2 = bytes 16-23 of the first + zeros, chunk 3 = bytes 16-23 of the second + zeros.  Half 0 of
// the wave then holds the first block of every row, half 1 the second, which is also how the scaled
// form of the instruction pairs lanes with block scales.  The 8-bit ring kernel runs on the copies
// unchanged but for the instruction's format code; K is padded with zero slots to whole k-tiles (and
// to the ring's minimum depth), so any K is served.  The copy reads 0.75 and writes 1 byte per
// element; the contraction then reads 1 byte per element where a kernel on the dense form would read
// 0.75 - at M = N = K = 8192 the copy is about a tenth of the time.
#include "kernel_tile_ring.hpp"

namespace optiml {
namespace {

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

template <int DT> using F6Cfg = ring::Cfg<5, true, false, 4, DT, 0, true>;

// One thread per 16-byte chunk of the copy: chunk c of k-tile t holds bytes off .. off + 15 (c < 2) or off .. off + 7
// and zeros (c >= 2) of the tile's 48 bytes, off = 0, 24, 16, 40, so a wave's stores are 1 KiB in a row and its loads
// cover 768 contiguous bytes.  WIDE: every row starts on a 16-byte boundary (8-byte loads); else byte loads.
// Elements at or beyond K read as zero.
template <bool WIDE>
__global__ __launch_bounds__(256) void f6_slots_kernel(const unsigned char *__restrict__ src, int64_t ld_bytes, int64_t stride_bytes,
                                                       int64_t rows, int64_t K, int64_t tiles, unsigned char *__restrict__ dst)
{
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t t = id >> 2, r = blockIdx.y, b = blockIdx.z;          // k-tile, row, batch
    const int c = (int)(id & 3);
    if (t >= tiles) return;
    const int off = c == 0 ? 0 : c == 1 ? 24 : c == 2 ? 16 : 40, len = c < 2 ? 16 : 8;
    const unsigned char *in = src + b * stride_bytes + r * ld_bytes + t * 48 + off;
    const int64_t left = K - t * 64;                                      // elements of this k-tile inside K
    const int valid = (left >= 64 ? 48 : left <= 0 ? 0 : (int)(left * 3 / 4)) - off;   // bytes of this chunk inside K (K is a multiple of 4)
    typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
    uintx4 v = uintx4{0u, 0u, 0u, 0u};
    if (WIDE && valid >= len) {
        const uintx2 lo = __builtin_nontemporal_load(reinterpret_cast<const uintx2 *>(in));
        v[0] = lo[0]; v[1] = lo[1];
        if (c < 2) {
            const uintx2 hi = __builtin_nontemporal_load(reinterpret_cast<const uintx2 *>(in + 8));
            v[2] = hi[0]; v[3] = hi[1];
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            unsigned int w = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (4 * i + j < len && 4 * i + j < valid) w |= (unsigned int)in[4 * i + j] << (8 * j);
            v[i] = w;
        }
    }
    *reinterpret_cast<uintx4 *>(dst + (((b * rows + r) * tiles + t) * 4 + c) * 16) = v;
}

Problem slot_problem(const Problem &p, const void *a, const void *b)
{
    const int64_t Kp = f6_slot_k(p.K);
    Problem q = p;
    q.K = Kp;
    q.A = a; q.lda = Kp; q.strideA = p.M * Kp;
    q.B = b; q.ldb = Kp; q.strideB = p.N * Kp;
    return q;
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

template <int DT>
bool f6_supports(const Problem &p)
{
    if (p.dtype != DT || p.a_col() || !p.b_col() || p.K < 1 || p.M < 1 || p.N < 1 || p.batch < 1) return false;
    if ((p.K | p.lda | p.ldb | p.strideA | p.strideB) & 3) return false;
    const int64_t Kp = f6_slot_k(p.K);
    if (p.batch > 65535 || Kp / 64 > int64_t(0x7fffffff) * 64) return false;                                            // the copy's grid
    if (p.M > ((int64_t(1) << 40) / Kp) / p.batch || p.N > ((int64_t(1) << 40) / Kp) / p.batch) return false;            // 1 TiB of slots
    const void *ws = reinterpret_cast<const void *>(uintptr_t(256));
    return ring::supports<F6Cfg<DT>>(slot_problem(p, ws, ws));
}

// the copies at 4 TB/s (1.75 bytes per element) and the ring kernel at 11 TFLOP/s per CU, in rounds of tiles
double f6_estimate(const Problem &p)
{
    const double Kp = (double)f6_slot_k(p.K);
    const double copy = (double)p.batch * (double)(p.M + p.N) * Kp * 1.75 / 4.0e6;
    const double tiles = (double)p.batch * (double)((p.M + 255) / 256) * (double)((p.N + 255) / 256);
    const double rounds = std::ceil(tiles / (double)compute_units());
    return 12.0 + copy + rounds * 2.0 * 65536.0 * Kp / 11.0e6;
}

template <int DT>
hipError_t f6_launch(const Problem &p, hipStream_t s)
{
    const int64_t Kp = f6_slot_k(p.K);
    const size_t a_bytes = align256((size_t)p.batch * p.M * Kp), b_bytes = align256((size_t)p.batch * p.N * Kp);
    void *ws = nullptr;
    hipError_t e = workspace(a_bytes + b_bytes, &ws, s);
    if (e != hipSuccess) return e;
    void *wa = ws, *wb = static_cast<char *>(ws) + a_bytes;
    e = launch_f6_slots(p.A, p.lda, p.strideA, p.batch, p.M, p.K, wa, s);
    if (e != hipSuccess) return e;
    e = launch_f6_slots(p.B, p.ldb, p.strideB, p.batch, p.N, p.K, wb, s);
    if (e != hipSuccess) return e;
    return ring::launch<F6Cfg<DT>>(slot_problem(p, wa, wb), s);
}

}  // namespace

// whole k-tiles of 64, at least as many as the ring is deep
int64_t f6_slot_k(int64_t K)
{
    const int64_t Kp = (K + 63) / 64 * 64, least = int64_t(64) * F6Cfg<DT_F6>::NS;
    return Kp < least ? least : Kp;
}

hipError_t launch_f6_slots(const void *src, int64_t ld, int64_t stride, int64_t batch, int64_t rows, int64_t K, void *dst, hipStream_t s)
{
    if (rows <= 0 || batch <= 0) return hipSuccess;
    const int64_t tiles = f6_slot_k(K) / 64, bx = (4 * tiles + 255) / 256;
    if (bx > 0x7fffffffLL || batch > 65535 || ((K | ld | stride) & 3)) return hipErrorInvalidValue;
    const int64_t ld_bytes = ld / 4 * 3, stride_bytes = stride / 4 * 3;
    const bool wide = (reinterpret_cast<uintptr_t>(src) & 15u) == 0 && ld_bytes % 16 == 0 && stride_bytes % 16 == 0;
    const unsigned char *in = static_cast<const unsigned char *>(src);
    unsigned char *out = static_cast<unsigned char *>(dst);
    for (int64_t r0 = 0; r0 < rows; r0 += 65535) {                         // grid.y holds at most 65535 rows
        const int64_t n = rows - r0 < 65535 ? rows - r0 : 65535;
        const dim3 grid((unsigned)bx, (unsigned)n, (unsigned)batch);
        // (the batch stride of the copy is rows * tiles * 64: the kernel is given all `rows`)
        if (wide)
            hipLaunchKernelGGL(f6_slots_kernel<true>, grid, dim3(256), 0, s, in + r0 * ld_bytes, ld_bytes, stride_bytes, rows, K, tiles,
                               out + r0 * tiles * 64);
        else
            hipLaunchKernelGGL(f6_slots_kernel<false>, grid, dim3(256), 0, s, in + r0 * ld_bytes, ld_bytes, stride_bytes, rows, K, tiles,
                               out + r0 * tiles * 64);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

const Variant *f6_variants()
{
    static const Variant v[] = {
        {"xs_ring_f6_rc_256x256_w2x4_ns5_k64", f6_supports<DT_F6>, f6_launch<DT_F6>, 256, 256,
         reinterpret_cast<const void *>(&ring::gemm_ring_kernel<F6Cfg<DT_F6>>), nullptr, true, f6_estimate},
        {"xs_ring_bf6_rc_256x256_w2x4_ns5_k64", f6_supports<DT_BF6>, f6_launch<DT_BF6>, 256, 256,
         reinterpret_cast<const void *>(&ring::gemm_ring_kernel<F6Cfg<DT_BF6>>), nullptr, true, f6_estimate}};
    return v;
}

}  // namespace optiml

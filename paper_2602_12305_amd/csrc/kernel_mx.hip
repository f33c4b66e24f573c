// The contraction on block-scaled ("microscaling") 4-bit, 6-bit or 8-bit operands:
//     C = act((sA * A) . (sB * B) + bias)
// A is M x K and B is N x K (k contiguous in both), elements in OCP E2M1, two to a byte along k, or in OCP E4M3 / E5M2,
// one to a byte; every
// 32 consecutive k of a row of A (of a column of B) share one scale, a power of two stored as an E8M0
// byte: scaleA[i][k / 32], scaleB[j][k / 32], value 2^(byte - 127) (byte 255 is NaN).  C is bf16.
//
// Fast path: the ring-of-stages tile kernel with Cfg::MX (kernel_tile_ring.hpp): the scaled form of the
// 64-deep matrix instruction takes a lane's block scale from a register of that lane, and a lane's
// 16-byte fragment is exactly one block.  The kernel fetches the four scale bytes of a row and k-tile
// (128 k) with one 4-byte load per lane; read from the caller's arrays those loads touch one cache line
// per row (512 lines per k-tile and workgroup, against 256 for the operands: 8192^3 took 0.36 ms), so
// the scales are first copied into the workspace with the rows of one k-tile side by side
// (mx_scale_tiles_kernel: dword [k-tile][row]), from where a wave's 64 loads are 256 contiguous bytes.
// 8-bit elements take the 64-deep kernel of the unscaled 8-bit contraction the same way: a k-tile is 64 k = two
// blocks (two scale bytes in the low half of the dword); lanes 0-31 supply the first block's scale, lanes 32-63 the
// second's.  6-bit elements (E2M3, E3M2; stored densely, four to three bytes) are first copied into the slot form of
// kernel_f6.hip - a lane of the first half then holds a row's first block of the k-tile, a lane of the second half
// its second block - and take the same kernel with the instruction's 6-bit format codes.
// Everything else - k not a whole number of k-tiles, pitches or
// addresses that the 16-byte and 4-byte loads cannot take, small problems - goes to mx_fallback_kernel,
// one thread per entry of C: block sums of the exact products, scaled by 2^(ea + eb - 254), added in
// fp32 in order of k.
#include "kernel_tile_ring.hpp"

namespace optiml {
namespace {

using MxCfg = ring::Cfg<4, true, true, 4, DT_F4, 0, false, 8, 4, 2, true>;
template <int DT> using Mx8Cfg = ring::Cfg<4, true, false, 4, DT, 0, true, 8, 4, 2, true>;

// out[t * rows + r] = the `sb` scale bytes in[r * pitch + sb t .. ] of row r and k-tile t (sb = 4 or 2), packed from
// byte 0 up; 64 x 64 blocks through LDS so that both sides move whole lines.  grid.z: 0 = A's scales, 1 = B's.
struct ScaleCopy { const unsigned char *in; int64_t pitch, rows; unsigned int *out; };
__global__ __launch_bounds__(256) void mx_scale_tiles_kernel(ScaleCopy a, ScaleCopy b, int64_t nk, int sb)
{
    __shared__ unsigned int tile[64][65];
    const ScaleCopy c = blockIdx.z == 0 ? a : b;
    const int64_t r0 = (int64_t)blockIdx.x * 64, t0 = (int64_t)blockIdx.y * 64;
    if (r0 >= c.rows) return;                                       // the grid covers the larger operand
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const bool words = sb == 4 && ((reinterpret_cast<uintptr_t>(c.in) | (uintptr_t)c.pitch) & 3) == 0;
    for (int i = 0; i < 16; ++i) {
        const int64_t r = r0 + 4 * i + grp, t = t0 + lane;
        unsigned int v = 0;
        if (r < c.rows && t < nk) {
            const unsigned char *src = c.in + r * c.pitch + sb * t;
            if (words) v = *reinterpret_cast<const unsigned int *>(src);
            else
                for (int k = 0; k < sb; ++k) v |= (unsigned int)src[k] << (8 * k);
        }
        tile[4 * i + grp][lane] = v;
    }
    __syncthreads();
    for (int i = 0; i < 16; ++i) {
        const int64_t t = t0 + 4 * i + grp, r = r0 + lane;
        if (t < nk && r < c.rows) c.out[t * c.rows + r] = tile[lane][4 * i + grp];
    }
}

template <int DT>
__global__ __launch_bounds__(256) void mx_fallback_kernel(int64_t M, int64_t N, int64_t K, const unsigned char *__restrict__ A, int64_t lda,
                                                          const unsigned char *__restrict__ sA, int64_t lds_a,
                                                          const unsigned char *__restrict__ B, int64_t ldb,
                                                          const unsigned char *__restrict__ sB, int64_t lds_b,
                                                          const float *__restrict__ bias, unsigned short *__restrict__ C, int64_t ldc, int act)
{
    // lda, ldb in bytes here; a block of 32 elements is 16 bytes of E2M1, 24 bytes of E2M3 / E3M2 or 32 bytes of E4M3 / E5M2
    const int64_t col = (int64_t)blockIdx.x * 16 + (threadIdx.x & 15), row = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4);
    if (row >= M || col >= N) return;
    const unsigned char *a = A + row * lda, *b = B + col * ldb;
    float acc = 0.0f;
    for (int64_t blk = 0; blk < K / 32; ++blk) {
        float sum = 0.0f;
        if constexpr (is_f6(DT)) {                          // dense 6-bit codes: a block is 24 bytes
            for (int i = 0; i < 32; ++i) {
                const unsigned x = six_bit_code(a, blk * 32 + i), y = six_bit_code(b, blk * 32 + i);
                sum += DT == DT_F6 ? f6e2m3_to_f32(x) * f6e2m3_to_f32(y) : f6e3m2_to_f32(x) * f6e3m2_to_f32(y);
            }
        } else if constexpr (DT == DT_F4) {
            for (int i = 0; i < 16; ++i) {                  // at most 32 products, each a multiple of 0.25 up to 36: exact
                const unsigned x = a[blk * 16 + i], y = b[blk * 16 + i];
                sum += f4e2m1_to_f32(x & 15u) * f4e2m1_to_f32(y & 15u) + f4e2m1_to_f32(x >> 4) * f4e2m1_to_f32(y >> 4);
            }
        } else {
            for (int i = 0; i < 32; ++i) {                  // exact products, added in fp32 in order of k
                const unsigned char x = a[blk * 32 + i], y = b[blk * 32 + i];
                sum += DT == DT_F8 ? f8e4m3_to_f32(x) * f8e4m3_to_f32(y) : f8e5m2_to_f32(x) * f8e5m2_to_f32(y);
            }
        }
        const int ea = sA[row * lds_a + blk], eb = sB[col * lds_b + blk];
        acc += (ea == 255 || eb == 255) ? __builtin_nanf("") : __builtin_ldexpf(sum, ea + eb - 254);
    }
    C[row * ldc + col] = f32_to_bf16(apply_act(acc + (bias ? bias[col] : 0.0f), act));
}

bool aligned_to(const void *q, uintptr_t a) { return (reinterpret_cast<uintptr_t>(q) & (a - 1)) == 0; }

// the problem in bytes of k, as the ring kernel sees it
Problem byte_problem(int dtype, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias,
                     void *C, int64_t ldc, int act)
{
    const int per_byte = dtype == DT_F4 ? 2 : 1;
    Problem p{};
    p.batch = 1; p.M = M; p.N = N; p.K = K / per_byte;
    p.A = A; p.lda = lda / per_byte; p.strideA = 0;
    p.B = B; p.ldb = ldb / per_byte; p.strideB = 0;
    p.bias = bias; p.strideBias = 0;
    p.C = C; p.ldc = ldc; p.strideC = 0;
    p.layout = 1; p.dtype = dtype; p.act = act;
    return p;
}

template <class Cfg>
hipError_t launch_tiles(const Problem &p, int64_t nk, int sb, const void *scaleA, int64_t lds_a, const void *scaleB, int64_t lds_b,
                        hipStream_t stream)
{
    // the scales of one k-tile side by side: dword [k-tile][row] for A, then for B
    const int64_t M = p.M, N = p.N;
    void *ws = nullptr;
    hipError_t e = workspace((size_t)(M + N) * nk * 4, &ws, stream);
    if (e != hipSuccess) return e;
    unsigned int *tA = static_cast<unsigned int *>(ws), *tB = tA + M * nk;
    const ScaleCopy ca{static_cast<const unsigned char *>(scaleA), lds_a, M, tA}, cb{static_cast<const unsigned char *>(scaleB), lds_b, N, tB};
    const int64_t rows = M > N ? M : N;
    if ((nk + 63) / 64 > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(mx_scale_tiles_kernel, dim3((unsigned)((rows + 63) / 64), (unsigned)((nk + 63) / 64), 2), dim3(256), 0, stream, ca, cb, nk, sb);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    ring::Params q;
    q.M = p.M; q.N = p.N; q.K = p.K; q.batch = 1;
    q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = 0;
    q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = 0;
    q.bias = p.bias; q.strideBias = 0;
    q.C = static_cast<char *>(p.C); q.ldc = p.ldc; q.strideC = 0;
    q.tiles_m = (p.M + Cfg::BM - 1) / Cfg::BM;
    q.tiles_n = (p.N + Cfg::BN - 1) / Cfg::BN;
    q.act = p.act;
    q.labels = nullptr; q.picked = nullptr; q.bias_row = 0;
    q.scaleA = reinterpret_cast<const char *>(tA); q.scaleB = reinterpret_cast<const char *>(tB);
    q.lds_a = 4; q.lds_b = 4; q.sk_a = M * 4; q.sk_b = N * 4;
    hipLaunchKernelGGL(ring::gemm_ring_kernel<Cfg>, dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(Cfg::THREADS), 0, stream, q);
    return hipGetLastError();
}

}  // namespace

// 0: the ring kernel, 1: the fallback
int mx_path(int dtype, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
            int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc)
{
    (void)scaleA; (void)scaleB; (void)lds_a; (void)lds_b;          // the copy takes any scale address and pitch
    const Problem p = byte_problem(dtype, M, N, K, A, lda, B, ldb, bias, C, ldc, 0);
    if (M * N < 65536 || M >= (int64_t(1) << 30) || N >= (int64_t(1) << 30)) return 1;
    if (dtype == DT_F4) return K % 128 == 0 && ring::supports<MxCfg>(p) ? 0 : 1;
    if (K % 64 != 0) return 1;
    if (is_f6(dtype)) {
        // the slot form of both operands in the workspace (kernel_f6.hip), then the 8-bit kernel's geometry
        const int64_t Kp = f6_slot_k(K);                          // the copies' pitch (K itself from five k-tiles on)
        if ((lda | ldb) & 3 || (M + N) > (int64_t(1) << 40) / Kp) return 1;
        const void *ws = reinterpret_cast<const void *>(uintptr_t(256));
        const Problem q = byte_problem(dtype, M, N, K, ws, Kp, ws, Kp, bias, C, ldc, 0);
        return (dtype == DT_F6 ? ring::supports<Mx8Cfg<DT_F6>>(q) : ring::supports<Mx8Cfg<DT_BF6>>(q)) ? 0 : 1;
    }
    return (dtype == DT_F8 ? ring::supports<Mx8Cfg<DT_F8>>(p) : ring::supports<Mx8Cfg<DT_BF8>>(p)) ? 0 : 1;
}

hipError_t launch_mx(int dtype, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a,
                     const void *B, int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc, int act,
                     hipStream_t stream)
{
    if (mx_path(dtype, M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc) == 0) {
        const Problem p = byte_problem(dtype, M, N, K, A, lda, B, ldb, bias, C, ldc, act);
        if (dtype == DT_F4) return launch_tiles<MxCfg>(p, K / 128, 4, scaleA, lds_a, scaleB, lds_b, stream);
        if (dtype == DT_F8) return launch_tiles<Mx8Cfg<DT_F8>>(p, K / 64, 2, scaleA, lds_a, scaleB, lds_b, stream);
        if (dtype == DT_BF8) return launch_tiles<Mx8Cfg<DT_BF8>>(p, K / 64, 2, scaleA, lds_a, scaleB, lds_b, stream);
        // 6-bit elements: slot copies of A and B at the head of the workspace, the scale tiles behind them
        const int64_t Kp = f6_slot_k(K);
        const size_t a_bytes = ((size_t)M * Kp + 255) & ~size_t(255), b_bytes = ((size_t)N * Kp + 255) & ~size_t(255);
        void *ws = nullptr;
        hipError_t e = workspace(a_bytes + b_bytes + (size_t)(M + N) * (K / 64) * 4, &ws, stream);
        if (e != hipSuccess) return e;
        void *wa = ws, *wb = static_cast<char *>(ws) + a_bytes;
        e = launch_f6_slots(A, lda, 0, 1, M, K, wa, stream);
        if (e != hipSuccess) return e;
        e = launch_f6_slots(B, ldb, 0, 1, N, K, wb, stream);
        if (e != hipSuccess) return e;
        const WorkspaceHead keep(a_bytes + b_bytes);
        const Problem q = byte_problem(dtype, M, N, K, wa, Kp, wb, Kp, bias, C, ldc, act);
        if (dtype == DT_F6) return launch_tiles<Mx8Cfg<DT_F6>>(q, K / 64, 2, scaleA, lds_a, scaleB, lds_b, stream);
        return launch_tiles<Mx8Cfg<DT_BF6>>(q, K / 64, 2, scaleA, lds_a, scaleB, lds_b, stream);
    }
    const int64_t bx = (N + 15) / 16, by = (M + 15) / 16;
    if (bx > 0x7fffffffLL || by > 65535) return hipErrorInvalidValue;
    const int per_byte = dtype == DT_F4 ? 2 : 1;
    const dim3 grid((unsigned)bx, (unsigned)by), block(256);
    const unsigned char *a = static_cast<const unsigned char *>(A), *b = static_cast<const unsigned char *>(B);
    const unsigned char *sa = static_cast<const unsigned char *>(scaleA), *sb = static_cast<const unsigned char *>(scaleB);
    unsigned short *c = static_cast<unsigned short *>(C);
    if (dtype == DT_F4)
        hipLaunchKernelGGL(mx_fallback_kernel<DT_F4>, grid, block, 0, stream, M, N, K, a, lda / per_byte, sa, lds_a, b, ldb / per_byte, sb, lds_b, bias, c, ldc, act);
    else if (dtype == DT_F6)
        hipLaunchKernelGGL(mx_fallback_kernel<DT_F6>, grid, block, 0, stream, M, N, K, a, lda / 4 * 3, sa, lds_a, b, ldb / 4 * 3, sb, lds_b, bias, c, ldc, act);
    else if (dtype == DT_BF6)
        hipLaunchKernelGGL(mx_fallback_kernel<DT_BF6>, grid, block, 0, stream, M, N, K, a, lda / 4 * 3, sa, lds_a, b, ldb / 4 * 3, sb, lds_b, bias, c, ldc, act);
    else if (dtype == DT_F8)
        hipLaunchKernelGGL(mx_fallback_kernel<DT_F8>, grid, block, 0, stream, M, N, K, a, lda, sa, lds_a, b, ldb, sb, lds_b, bias, c, ldc, act);
    else
        hipLaunchKernelGGL(mx_fallback_kernel<DT_BF8>, grid, block, 0, stream, M, N, K, a, lda, sa, lds_a, b, ldb, sb, lds_b, bias, c, ldc, act);
    return hipGetLastError();
}

}  // namespace optiml

// The contraction on block-scaled ("microscaling") 4-bit operands:
//     C = act((sA * A) . (sB * B) + bias)
// A is M x K and B is N x K (k contiguous in both), elements in OCP E2M1, two to a byte along k; every
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
// Everything else - k not a whole number of k-tiles, pitches or
// addresses that the 16-byte and 4-byte loads cannot take, small problems - goes to mx_fallback_kernel,
// one thread per entry of C: block sums of the exact products, scaled by 2^(ea + eb - 254), added in
// fp32 in order of k.
#include "kernel_tile_ring.hpp"

namespace optiml {
namespace {

using MxCfg = ring::Cfg<4, true, true, 4, DT_F4, 0, false, 8, 4, 2, true>;

// out[t * rows + r] = the four scale bytes in[r * pitch + 4 t .. + 3] of row r and k-tile t; 64 x 64 blocks
// through LDS so that both sides move whole lines.  grid.z: 0 = A's scales, 1 = B's.
struct ScaleCopy { const unsigned char *in; int64_t pitch, rows; unsigned int *out; };
__global__ __launch_bounds__(256) void mx_scale_tiles_kernel(ScaleCopy a, ScaleCopy b, int64_t nk)
{
    __shared__ unsigned int tile[64][65];
    const ScaleCopy c = blockIdx.z == 0 ? a : b;
    const int64_t r0 = (int64_t)blockIdx.x * 64, t0 = (int64_t)blockIdx.y * 64;
    if (r0 >= c.rows) return;                                       // the grid covers the larger operand
    const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const bool words = ((reinterpret_cast<uintptr_t>(c.in) | (uintptr_t)c.pitch) & 3) == 0;
    for (int i = 0; i < 16; ++i) {
        const int64_t r = r0 + 4 * i + grp, t = t0 + lane;
        unsigned int v = 0;
        if (r < c.rows && t < nk) {
            const unsigned char *src = c.in + r * c.pitch + 4 * t;
            v = words ? *reinterpret_cast<const unsigned int *>(src)
                      : (unsigned int)src[0] | ((unsigned int)src[1] << 8) | ((unsigned int)src[2] << 16) | ((unsigned int)src[3] << 24);
        }
        tile[4 * i + grp][lane] = v;
    }
    __syncthreads();
    for (int i = 0; i < 16; ++i) {
        const int64_t t = t0 + 4 * i + grp, r = r0 + lane;
        if (t < nk && r < c.rows) c.out[t * c.rows + r] = tile[lane][4 * i + grp];
    }
}

__global__ __launch_bounds__(256) void mx_fallback_kernel(int64_t M, int64_t N, int64_t K, const unsigned char *__restrict__ A, int64_t lda,
                                                          const unsigned char *__restrict__ sA, int64_t lds_a,
                                                          const unsigned char *__restrict__ B, int64_t ldb,
                                                          const unsigned char *__restrict__ sB, int64_t lds_b,
                                                          const float *__restrict__ bias, unsigned short *__restrict__ C, int64_t ldc, int act)
{
    // lda, ldb in bytes here; a block of 32 elements is 16 bytes
    const int64_t col = (int64_t)blockIdx.x * 16 + (threadIdx.x & 15), row = (int64_t)blockIdx.y * 16 + (threadIdx.x >> 4);
    if (row >= M || col >= N) return;
    const unsigned char *a = A + row * lda, *b = B + col * ldb;
    float acc = 0.0f;
    for (int64_t blk = 0; blk < K / 32; ++blk) {
        float sum = 0.0f;                                   // at most 32 products, each a multiple of 0.25 up to 36: exact
        for (int i = 0; i < 16; ++i) {
            const unsigned x = a[blk * 16 + i], y = b[blk * 16 + i];
            sum += f4e2m1_to_f32(x & 15u) * f4e2m1_to_f32(y & 15u) + f4e2m1_to_f32(x >> 4) * f4e2m1_to_f32(y >> 4);
        }
        const int ea = sA[row * lds_a + blk], eb = sB[col * lds_b + blk];
        acc += (ea == 255 || eb == 255) ? __builtin_nanf("") : __builtin_ldexpf(sum, ea + eb - 254);
    }
    C[row * ldc + col] = f32_to_bf16(apply_act(acc + (bias ? bias[col] : 0.0f), act));
}

bool aligned_to(const void *q, uintptr_t a) { return (reinterpret_cast<uintptr_t>(q) & (a - 1)) == 0; }

// the problem in bytes of k, as the ring kernel sees it
Problem byte_problem(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias, void *C,
                     int64_t ldc, int act)
{
    Problem p{};
    p.batch = 1; p.M = M; p.N = N; p.K = K / 2;
    p.A = A; p.lda = lda / 2; p.strideA = 0;
    p.B = B; p.ldb = ldb / 2; p.strideB = 0;
    p.bias = bias; p.strideBias = 0;
    p.C = C; p.ldc = ldc; p.strideC = 0;
    p.layout = 1; p.dtype = DT_F4; p.act = act;
    return p;
}

}  // namespace

// 0: the ring kernel, 1: the fallback
int mx_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B, int64_t ldb,
            const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc)
{
    (void)scaleA; (void)scaleB; (void)lds_a; (void)lds_b;          // the copy takes any scale address and pitch
    const Problem p = byte_problem(M, N, K, A, lda, B, ldb, bias, C, ldc, 0);
    return K % 128 == 0 && M * N >= 65536 && M < (int64_t(1) << 30) && N < (int64_t(1) << 30) && ring::supports<MxCfg>(p) ? 0 : 1;
}

hipError_t launch_mx(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
                     int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc, int act, hipStream_t stream)
{
    if (mx_path(M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc) == 0) {
        const Problem p = byte_problem(M, N, K, A, lda, B, ldb, bias, C, ldc, act);
        // the scales of one k-tile side by side: dword [k-tile][row] for A, then for B
        const int64_t nk = K / 128;
        void *ws = nullptr;
        hipError_t e = workspace((size_t)(M + N) * nk * 4, &ws, stream);
        if (e != hipSuccess) return e;
        unsigned int *tA = static_cast<unsigned int *>(ws), *tB = tA + M * nk;
        const ScaleCopy ca{static_cast<const unsigned char *>(scaleA), lds_a, M, tA}, cb{static_cast<const unsigned char *>(scaleB), lds_b, N, tB};
        const int64_t rows = M > N ? M : N;
        if ((nk + 63) / 64 > 65535) return hipErrorInvalidValue;
        hipLaunchKernelGGL(mx_scale_tiles_kernel, dim3((unsigned)((rows + 63) / 64), (unsigned)((nk + 63) / 64), 2), dim3(256), 0, stream, ca, cb, nk);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        ring::Params q;
        q.M = p.M; q.N = p.N; q.K = p.K; q.batch = 1;
        q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = 0;
        q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = 0;
        q.bias = p.bias; q.strideBias = 0;
        q.C = static_cast<char *>(p.C); q.ldc = p.ldc; q.strideC = 0;
        q.tiles_m = (p.M + MxCfg::BM - 1) / MxCfg::BM;
        q.tiles_n = (p.N + MxCfg::BN - 1) / MxCfg::BN;
        q.act = act;
        q.labels = nullptr; q.picked = nullptr; q.bias_row = 0;
        q.scaleA = reinterpret_cast<const char *>(tA); q.scaleB = reinterpret_cast<const char *>(tB);
        q.lds_a = 4; q.lds_b = 4; q.sk_a = M * 4; q.sk_b = N * 4;
        hipLaunchKernelGGL(ring::gemm_ring_kernel<MxCfg>, dim3((unsigned)(q.tiles_m * q.tiles_n)), dim3(MxCfg::THREADS), 0, stream, q);
        return hipGetLastError();
    }
    const int64_t bx = (N + 15) / 16, by = (M + 15) / 16;
    if (bx > 0x7fffffffLL || by > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL(mx_fallback_kernel, dim3((unsigned)bx, (unsigned)by), dim3(256), 0, stream, M, N, K,
                       static_cast<const unsigned char *>(A), lda / 2, static_cast<const unsigned char *>(scaleA), lds_a,
                       static_cast<const unsigned char *>(B), ldb / 2, static_cast<const unsigned char *>(scaleB), lds_b, bias,
                       static_cast<unsigned short *>(C), ldc, act);
    return hipGetLastError();
}

}  // namespace optiml

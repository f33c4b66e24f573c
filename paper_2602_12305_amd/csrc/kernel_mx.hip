// The contraction on block-scaled ("microscaling") 4-bit operands:
//     C = act((sA * A) . (sB * B) + bias)
// A is M x K and B is N x K (k contiguous in both), elements in OCP E2M1, two to a byte along k; every
// 32 consecutive k of a row of A (of a column of B) share one scale, a power of two stored as an E8M0
// byte: scaleA[i][k / 32], scaleB[j][k / 32], value 2^(byte - 127) (byte 255 is NaN).  C is bf16.
//
// Fast path: the ring-of-stages tile kernel with Cfg::MX (kernel_tile_ring.hpp): the scaled form of the
// 64-deep matrix instruction takes a lane's block scale from a register of that lane, and a lane's
// 16-byte fragment is exactly one block.  Everything else - k not a whole number of k-tiles, pitches or
// addresses that the 16-byte and 4-byte loads cannot take, small problems - goes to mx_fallback_kernel,
// one thread per entry of C: block sums of the exact products, scaled by 2^(ea + eb - 254), added in
// fp32 in order of k.
#include "kernel_tile_ring.hpp"

namespace optiml {
namespace {

using MxCfg = ring::Cfg<4, true, false, 4, DT_F4, 0, false, 8, 4, 2, true>;

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
    const Problem p = byte_problem(M, N, K, A, lda, B, ldb, bias, C, ldc, 0);
    const bool scales_ok = aligned_to(scaleA, 4) && aligned_to(scaleB, 4) && lds_a % 4 == 0 && lds_b % 4 == 0 &&
                           M * lds_a < (int64_t(1) << 32) && N * lds_b < (int64_t(1) << 32);
    return K % 128 == 0 && M * N >= 65536 && scales_ok && ring::supports<MxCfg>(p) ? 0 : 1;
}

hipError_t launch_mx(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
                     int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc, int act, hipStream_t stream)
{
    if (mx_path(M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc) == 0) {
        const Problem p = byte_problem(M, N, K, A, lda, B, ldb, bias, C, ldc, act);
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
        q.scaleA = static_cast<const char *>(scaleA); q.scaleB = static_cast<const char *>(scaleB);
        q.lds_a = lds_a; q.lds_b = lds_b;
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

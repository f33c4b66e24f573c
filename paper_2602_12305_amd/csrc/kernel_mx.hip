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
#include <type_traits>

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

// ---- a few rows of block-scaled E2M1: straight from memory into the 128-deep scaled instruction ----
// Up to 128 rows of A over a large B the contraction is bound by reading B (N K / 2 bytes and N K / 32 scale bytes).
// The 128-deep scaled instruction takes from lane l the block k = 32 (l / 16) .. + 31 of row l % 16 of each operand -
// 16 contiguous bytes - and that block's scale from a register of the same lane: one 16-byte load and one byte load
// per lane, operand and k-step, no LDS, no copy of the scales.  A wave owns 16 CG columns of C, the WK waves of a
// workgroup take every WK-th run of U k-steps and add their partial sums through LDS; blockIdx.y is the block of 16
// rows (each block reads B again).  K a multiple of 128, rows on 16-byte boundaries.
typedef unsigned int mx_uintx4 __attribute__((ext_vector_type(4)));
typedef float mx_floatx4 __attribute__((ext_vector_type(4)));
typedef int mx_intx8 __attribute__((ext_vector_type(8)));

template <int CG, int U> struct Mx4Set { mx_uintx4 a[U], b[U][CG]; unsigned int sa[U], sb[U][CG]; };

template <int CG, int WK, int U>
__global__ __launch_bounds__(64 * WK) void mx4_stream_kernel(int64_t M, int64_t N, int64_t K, const unsigned char *__restrict__ A, int64_t lda,
                                                             const unsigned char *__restrict__ sA, int64_t lds_a,
                                                             const unsigned char *__restrict__ B, int64_t ldb,
                                                             const unsigned char *__restrict__ sB, int64_t lds_b,
                                                             const float *__restrict__ bias, unsigned short *__restrict__ C, int64_t ldc, int act)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // lda, ldb in bytes here
    __shared__ float part[WK][CG][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, row = lane & 15, grp = lane >> 4;
    const int64_t m0 = 16 * (int64_t)blockIdx.y, n0 = (int64_t)blockIdx.x * (16 * CG);
    const int64_t m = m0 + row < M ? m0 + row : M - 1;                     // lanes beyond M or N read the last row, store nothing
    const unsigned char *a = A + m * lda + grp * 16, *as = sA + m * lds_a + grp;
    const unsigned char *b[CG], *bs[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) {
        const int64_t n = n0 + 16 * g + row < N ? n0 + 16 * g + row : N - 1;
        b[g] = B + n * ldb + grp * 16;
        bs[g] = sB + n * lds_b + grp;
    }
    const int64_t steps = K / 128;
    mx_floatx4 acc[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[g] = mx_floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    Mx4Set<CG, U> cur, nxt;
    // a k-step beyond the last one: the first step is read again and dropped (zero elements, unit scales)
    auto fetch = [&](int64_t run, Mx4Set<CG, U> &f) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t step = run * U + u;
            const bool inside = step < steps;
            const int64_t s = inside ? step : 0;
            const mx_uintx4 va = *reinterpret_cast<const mx_uintx4 *>(a + s * 64);
            const unsigned int ea = as[s * 4];
            f.a[u] = inside ? va : mx_uintx4{0u, 0u, 0u, 0u};
            f.sa[u] = inside ? ea : 127u;
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                const mx_uintx4 vb = __builtin_nontemporal_load(reinterpret_cast<const mx_uintx4 *>(b[g] + s * 64));
                const unsigned int eb = bs[g][s * 4];
                f.b[u][g] = inside ? vb : mx_uintx4{0u, 0u, 0u, 0u};
                f.sb[u][g] = inside ? eb : 127u;
            }
        }
    };
    auto multiply = [&](const Mx4Set<CG, U> &f) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const mx_intx8 a8 = {(int)f.a[u][0], (int)f.a[u][1], (int)f.a[u][2], (int)f.a[u][3], 0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                const mx_intx8 b8 = {(int)f.b[u][g][0], (int)f.b[u][g][1], (int)f.b[u][g][2], (int)f.b[u][g][3], 0, 0, 0, 0};
                // first operand B: acc[r] of lane l = sum over k of B[n0 + 16 g + 4 (l / 16) + r][k] A[l % 16][k], scaled per block
                acc[g] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b8, a8, acc[g], 4, 4, 0, (int)f.sb[u][g], 0, (int)f.sa[u]);
            }
        }
    };
    const int64_t runs = (steps + U - 1) / U;
    fetch(wave, cur);
    for (int64_t run = wave; run < runs; run += 2 * WK) {
        fetch(run + WK, nxt);
        multiply(cur);
        fetch(run + 2 * WK, cur);
        multiply(nxt);
    }
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[wave][g][r][lane] = acc[g][r];
    __syncthreads();
    for (int idx = wave; idx < CG * 4; idx += WK) {
        const int g = idx >> 2, r = idx & 3;
        float z = 0.0f;
#pragma unroll
        for (int w = 0; w < WK; ++w) z += part[w][g][r][lane];
        const int64_t col = n0 + 16 * g + 4 * grp + r;                      // this lane: row m0 + `row` of C
        if (m0 + row < M && col < N) C[(m0 + row) * ldc + col] = f32_to_bf16(apply_act(z + (bias ? bias[col] : 0.0f), act));
    }
#endif
}

// The same through LDS-DMA (16-byte loads at 64-byte runs per row reach 2.5 TB/s): a stage is four k-steps = 256 bytes of
// each row, 16-byte chunks by consecutive lanes, plus the stage's 16 scale bytes of each row as one more chunk; chunk c
// of row r sits at position c ^ (r % 16) of the row's 16, so that the 16 rows a 16-byte read touches fall on different
// banks.  Private stages per wave, NS - 1 in flight, hand-counted waits as in the other direct-to-LDS kernels; every
// workgroup walks its stages from a start of its own.  Needs K a multiple of 512 and the scale rows on 16-byte
// boundaries as well.
template <int CG, int WK, int NS>
__global__ __launch_bounds__(64 * WK) void mx4_dma_kernel(int64_t M, int64_t N, int64_t K, const unsigned char *__restrict__ A, int64_t lda,
                                                          const unsigned char *__restrict__ sA, int64_t lds_a,
                                                          const unsigned char *__restrict__ B, int64_t ldb,
                                                          const unsigned char *__restrict__ sB, int64_t lds_b,
                                                          const float *__restrict__ bias, unsigned short *__restrict__ C, int64_t ldc, int act)
{
#if defined(__HIP_DEVICE_COMPILE__)
    static_assert(CG == 2 || CG == 4, "the scale chunks of B: half or all of one instruction");
    constexpr int A_DATA = 4096, A_SC = 1024, B_DATA = CG * 4096, B_SC = 1024;
    constexpr int STAGE = A_DATA + A_SC + B_DATA + B_SC, LOADS = 4 + 1 + 4 * CG + 1;
    static_assert((NS - 1) * LOADS < 64, "the counted wait has six bits");
    static_assert(WK * CG * 4 * 64 * 4 <= WK * NS * STAGE, "the reduction buffer reuses the staging area");
    extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
    ring::lds_char *const lds = (ring::lds_char *)lds_raw;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), row = lane & 15, grp = lane >> 4;
    const int64_t m0 = 16 * (int64_t)blockIdx.y, n0 = (int64_t)blockIdx.x * (16 * CG);
    const char *a_base = reinterpret_cast<const char *>(A) + m0 * lda, *as_base = reinterpret_cast<const char *>(sA) + m0 * lds_a;
    const char *b_base = reinterpret_cast<const char *>(B) + n0 * ldb, *bs_base = reinterpret_cast<const char *>(sB) + n0 * lds_b;
    // global side (rows beyond M or N fetch the last row again: their sums are never stored).  Data: slot f = 64 j +
    // lane of an operand holds chunk (f % 16) ^ (row % 16) of row f / 16; scales: slot f holds the chunk of row f
    uint32_t a_off[4], b_off[4 * CG], as_off, bs_off;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int f = 64 * j + lane, r = f >> 4;
        const int64_t rr = m0 + r < M ? r : M - 1 - m0;
        a_off[j] = (uint32_t)(rr * lda + (((f & 15) ^ (r & 15)) << 4));
    }
#pragma unroll
    for (int j = 0; j < 4 * CG; ++j) {
        const int f = 64 * j + lane, r = f >> 4;
        const int64_t rr = n0 + r < N ? r : N - 1 - n0;
        b_off[j] = (uint32_t)(rr * ldb + (((f & 15) ^ (r & 15)) << 4));
    }
    {
        const int r = lane & 15;                                           // (lanes 16-63 fetch these rows again, into unused space)
        as_off = (uint32_t)((m0 + r < M ? r : M - 1 - m0) * lds_a);
        const int rb = lane % (16 * CG);
        bs_off = (uint32_t)((n0 + rb < N ? rb : N - 1 - n0) * lds_b);
    }
    const uint32_t wave_lds = (uint32_t)reinterpret_cast<uintptr_t>(lds) + wave * (NS * STAGE);
    auto issue = [&](int64_t stage, int slot) {
        const char *ga = ring::scalar_ptr(a_base + stage * 256), *gb = ring::scalar_ptr(b_base + stage * 256);
        const char *gas = ring::scalar_ptr(as_base + stage * 16), *gbs = ring::scalar_ptr(bs_base + stage * 16);
        const uint32_t d = __builtin_amdgcn_readfirstlane(wave_lds + slot * STAGE);
#pragma unroll
        for (int j = 0; j < 4; ++j) ring::dma_load16(ga, a_off[j], d + j * 1024);
        ring::dma_load16(gas, as_off, d + A_DATA);
#pragma unroll
        for (int j = 0; j < 4 * CG; ++j) ring::dma_load16_once(gb, b_off[j], d + A_DATA + A_SC + j * 1024);
        ring::dma_load16_once(gbs, bs_off, d + A_DATA + A_SC + B_DATA);
    };
    mx_floatx4 acc[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[g] = mx_floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    const int64_t stages = K / 512;
    const int64_t mine = stages > wave ? (stages - wave + WK - 1) / WK : 0;
    const int64_t rot = mine > 0 ? (int64_t)blockIdx.x % mine : 0;
    auto stage_of = [&](int64_t i) { return wave + ((i + rot) % mine) * WK; };
    if (mine > 0) {
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(stage_of(s < mine ? s : mine - 1), s);
        for (int64_t i = 0; i < mine; ++i) {
            const int slot = (int)(i % NS);
            const int64_t nxt = i + NS - 1;
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0xc07f);                    // lgkmcnt(0): the previous stage's LDS reads have returned
            issue(stage_of(nxt < mine ? nxt : mine - 1), (int)(nxt % NS));
            ring::wait_vmcnt<(NS - 1) * LOADS>();                  // stage i has landed; its LDS reads below are new
            asm volatile("" ::: "memory");
            const ring::lds_char *st = lds + wave * (NS * STAGE) + slot * STAGE;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int pos = (((4 * u + grp) ^ row) << 4) + row * 256;                   // this lane's block of k-step u
                const mx_uintx4 va = *reinterpret_cast<const __attribute__((address_space(3))) mx_uintx4 *>(st + pos);
                const unsigned int ea = *reinterpret_cast<const __attribute__((address_space(3))) unsigned char *>(st + A_DATA + row * 16 + 4 * u + grp);
                const mx_intx8 a8 = {(int)va[0], (int)va[1], (int)va[2], (int)va[3], 0, 0, 0, 0};
#pragma unroll
                for (int g = 0; g < CG; ++g) {
                    const mx_uintx4 vb = *reinterpret_cast<const __attribute__((address_space(3))) mx_uintx4 *>(st + A_DATA + A_SC + g * 4096 + pos);
                    const unsigned int eb =
                        *reinterpret_cast<const __attribute__((address_space(3))) unsigned char *>(st + A_DATA + A_SC + B_DATA + (16 * g + row) * 16 + 4 * u + grp);
                    const mx_intx8 b8 = {(int)vb[0], (int)vb[1], (int)vb[2], (int)vb[3], 0, 0, 0, 0};
                    acc[g] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b8, a8, acc[g], 4, 4, 0, (int)eb, 0, (int)ea);
                }
            }
            asm volatile("" ::: "memory");                          // the reads are done before the slot is refilled
        }
        ring::wait_vmcnt<0>();
    }
    __syncthreads();                                                // the staging area is free now
    __attribute__((address_space(3))) float *part = (__attribute__((address_space(3))) float *)lds;
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[((wave * CG + g) * 4 + r) * 64 + lane] = acc[g][r];
    __syncthreads();
    for (int idx = wave; idx < CG * 4; idx += WK) {
        const int g = idx >> 2, r = idx & 3;
        float z = 0.0f;
#pragma unroll
        for (int w = 0; w < WK; ++w) z += part[((w * CG + g) * 4 + r) * 64 + lane];
        const int64_t col = n0 + 16 * g + 4 * grp + r;
        if (m0 + row < M && col < N) C[(m0 + row) * ldc + col] = f32_to_bf16(apply_act(z + (bias ? bias[col] : 0.0f), act));
    }
#endif
}

// ... and the DMA form's: whole stages of 512 k, scale rows on 16-byte boundaries, 32-bit offsets within a block of rows
bool mx4_dma_streams(int64_t K, const void *sA, int64_t lds_a, const void *sB, int64_t lds_b, int64_t lda, int64_t ldb)
{
    if (K % 512 != 0 || ((lds_a | lds_b) & 15) || lda >= (int64_t(1) << 28) || ldb >= (int64_t(1) << 26)) return false;
    return ((reinterpret_cast<uintptr_t>(sA) | reinterpret_cast<uintptr_t>(sB)) & 15u) == 0 && lds_a < (int64_t(1) << 26) && lds_b < (int64_t(1) << 24);
}

// the streaming kernel's ground: few rows, many columns, whole k-steps, rows the 16-byte loads can take
bool mx4_streams(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb)
{
    if (M < 1 || M > 128 || N < 1024 || K < 128 || K % 128 != 0 || (N + 15) / 16 > 0x7fffffffLL) return false;
    // every block of 16 rows reads B again: beyond three blocks only while B (N K / 2 bytes) stays in the Infinity Cache
    // (64 x 8192 x 8192: 23.7 us against 55.9 us on the tile kernel; 128 x 16384 x 16384: 221 us against 100 us)
    if (M > 48 && (double)N * (double)K > 96e6) return false;
    if ((lda | ldb) & 31) return false;                                     // (elements: 16 bytes)
    return ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15u) == 0;
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

// 0: the ring kernel, 1: the fallback, 2: the streaming kernel for a few rows of E2M1
int mx_path(int dtype, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
            int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc)
{
    (void)scaleA; (void)scaleB; (void)lds_a; (void)lds_b;          // the copy takes any scale address and pitch
    const Problem p = byte_problem(dtype, M, N, K, A, lda, B, ldb, bias, C, ldc, 0);
    if (dtype == DT_F4 && mx4_streams(M, N, K, A, lda, B, ldb)) return 2;
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
    const int path = mx_path(dtype, M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc);
    if (path == 2) {
        const unsigned char *a = static_cast<const unsigned char *>(A), *b = static_cast<const unsigned char *>(B);
        const unsigned char *sa = static_cast<const unsigned char *>(scaleA), *sb = static_cast<const unsigned char *>(scaleB);
        unsigned short *c = static_cast<unsigned short *>(C);
        const unsigned rb = (unsigned)((M + 15) / 16);
        if (mx4_dma_streams(K, scaleA, lds_a, scaleB, lds_b, lda, ldb)) {
            // 64 columns and three waves a workgroup (16 x 16384 x 16384: 28.6 us against 40.6 us for 32 columns and four
            // waves) once that still gives three quarters of the CUs a workgroup
            auto go = [&](auto cg, auto wk) -> hipError_t {
                constexpr int CG = decltype(cg)::value, WK = decltype(wk)::value, NS = 2, LDS_BYTES = WK * NS * (4096 + 1024 + CG * 4096 + 1024);
                static_assert(LDS_BYTES <= 160 * 1024, "LDS");
                static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&mx4_dma_kernel<CG, WK, NS>),
                                                                   hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
                if (attr != hipSuccess) return attr;
                hipLaunchKernelGGL((mx4_dma_kernel<CG, WK, NS>), dim3((unsigned)((N + 16 * CG - 1) / (16 * CG)), rb), dim3(64 * WK), LDS_BYTES, stream,
                                   M, N, K, a, lda / 2, sa, lds_a, b, ldb / 2, sb, lds_b, bias, c, ldc, act);
                return hipGetLastError();
            };
            if ((N + 63) / 64 * (int64_t)rb >= (int64_t)compute_units() * 3 / 4) return go(std::integral_constant<int, 4>{}, std::integral_constant<int, 3>{});
            return go(std::integral_constant<int, 2>{}, std::integral_constant<int, 4>{});
        }
        if (N >= 8192)
            hipLaunchKernelGGL((mx4_stream_kernel<4, 8, 2>), dim3((unsigned)((N + 63) / 64), rb), dim3(512), 0, stream, M, N, K, a, lda / 2, sa, lds_a, b,
                               ldb / 2, sb, lds_b, bias, c, ldc, act);
        else
            hipLaunchKernelGGL((mx4_stream_kernel<1, 4, 4>), dim3((unsigned)((N + 15) / 16), rb), dim3(256), 0, stream, M, N, K, a, lda / 2, sa, lds_a, b,
                               ldb / 2, sb, lds_b, bias, c, ldc, act);
        return hipGetLastError();
    }
    if (path == 0) {
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

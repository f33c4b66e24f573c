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

// ---- a few rows: the dense form straight into registers -------------------------------------------
// C (up to 16 rows per workgroup; up to kF6RowBlocks such blocks, each reading B again) = act(A . B + bias) is bound
// by reading B.  The 128-deep form of the matrix instruction takes from lane l the 32 values k = 32 (l / 16) .. + 31
// of row l % 16 of each operand: 24 contiguous bytes of a dense row, which three 8-byte loads fetch as they lie in
// memory - no copy, no LDS.  A wave owns 16 CG columns of C (16 CG rows of B, stored [N][K]); the WK waves of a
// workgroup take every WK-th run of U k-steps of 128 and add their partial sums through LDS; the loads of the next
// run are issued before the current run is multiplied.  A (16 x K, at most 192 KiB at K = 16384) is re-read by every
// wave from the caches.  Needs rows that start on 8-byte boundaries (pitches multiples of 32 elements = 24 bytes)
// and K a multiple of 32.
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx8 __attribute__((ext_vector_type(8)));

// this lane's block of a k-step: inside K, or zeros (K is a whole number of blocks; a lane whose block lies beyond K
// reads the first block of its row instead and drops it)
template <bool ONCE>
__device__ __forceinline__ void f6_fetch(const unsigned char *row, int64_t step, int grp, int64_t blocks, unsigned int (&f)[6])
{
    const bool inside = step * 4 + grp < blocks;
    const uintx2 *src = reinterpret_cast<const uintx2 *>(row + (inside ? step * 96 : -(int64_t)grp * 24));   // 24 bytes on an 8-byte boundary
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uintx2 v = ONCE ? __builtin_nontemporal_load(src + i) : src[i];
        f[2 * i] = inside ? v[0] : 0u;
        f[2 * i + 1] = inside ? v[1] : 0u;
    }
}

// first operand B: acc[r] of lane l = sum_k B[n0 + 4 (l / 16) + r][k] A[l % 16][k]
template <int DT>
__device__ __forceinline__ floatx4 f6_mma(const unsigned int (&a)[6], const unsigned int (&b)[6], floatx4 acc)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int F = F8F6F4Code<DT>::value;
    const intx8 a8 = {(int)a[0], (int)a[1], (int)a[2], (int)a[3], (int)a[4], (int)a[5], 0, 0};
    const intx8 b8 = {(int)b[0], (int)b[1], (int)b[2], (int)b[3], (int)b[4], (int)b[5], 0, 0};
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b8, a8, acc, F, F, 0, 0, 0, 0);
#else
    return acc;
#endif
}

// blocks of 16 rows the streaming kernels take (each block reads B again, from the caches when it fits)
constexpr int64_t kF6RowBlocks = 8;

// CG groups of 16 columns per wave (an A fragment serves CG matrix instructions), WK waves along k, U k-steps per run
template <int CG, int U> struct F6Set { unsigned int a[U][6], b[U][CG][6]; };

template <int DT, int CG, int WK, int U>
__global__ __launch_bounds__(64 * WK) void f6_stream_kernel(Problem p, int64_t lda_bytes, int64_t ldb_bytes, int64_t sa_bytes, int64_t sb_bytes)
{
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ float part[WK][CG][4][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, row = lane & 15, grp = lane >> 4;
    // blockIdx.y: (batch, block of 16 rows of A and C)
    const int64_t row_blocks = (p.M + 15) / 16, batch = blockIdx.y / row_blocks, m0 = 16 * (blockIdx.y % row_blocks);
    const int64_t n0 = (int64_t)blockIdx.x * (16 * CG);
    const int64_t m = m0 + row < p.M ? m0 + row : p.M - 1;                 // lanes beyond M or N read the last row, store nothing
    const unsigned char *a = static_cast<const unsigned char *>(p.A) + batch * sa_bytes + m * lda_bytes + grp * 24;
    const unsigned char *b[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) {
        const int64_t n = n0 + 16 * g + row < p.N ? n0 + 16 * g + row : p.N - 1;
        b[g] = static_cast<const unsigned char *>(p.B) + batch * sb_bytes + n * ldb_bytes + grp * 24;
    }
    const int64_t steps = (p.K + 127) / 128;                               // k-steps of 128 elements = 96 bytes a row
    const int64_t blocks = p.K / 32;                                       // whole blocks of 32 elements in a row
    floatx4 acc[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[g] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};
    F6Set<CG, U> cur, nxt;
    auto fetch = [&](int64_t run, F6Set<CG, U> &f) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            f6_fetch<false>(a, run * U + u, grp, blocks, f.a[u]);
#pragma unroll
            for (int g = 0; g < CG; ++g) f6_fetch<true>(b[g], run * U + u, grp, blocks, f.b[u][g]);
        }
    };
    auto multiply = [&](const F6Set<CG, U> &f) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int g = 0; g < CG; ++g) acc[g] = f6_mma<DT>(f.a[u], f.b[u][g], acc[g]);
    };
    // runs of U steps, dealt to the waves in turn; a fetch beyond the last step yields zeros without touching memory
    // beyond the rows, so the two halves of the loop need no conditions
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
    unsigned short *C = static_cast<unsigned short *>(p.C) + batch * p.strideC;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    // the WK waves share the CG x 4 values of every lane position
    for (int idx = wave; idx < CG * 4; idx += WK) {
        const int g = idx >> 2, r = idx & 3;
        float z = 0.0f;
#pragma unroll
        for (int w = 0; w < WK; ++w) z += part[w][g][r][lane];
        const int64_t col = n0 + 16 * g + 4 * grp + r;                      // this lane: row `row` of C
        if (m0 + row < p.M && col < p.N) {
            if (bias) z += p.bias_row ? bias[m0 + row] : bias[col];
            C[(m0 + row) * p.ldc + col] = f32_to_bf16(apply_act(z, p.act));
        }
    }
#endif
}

// The same contraction with the rows brought in by LDS-DMA: a lane's three 8-byte loads at a 24-byte stride over 16
// rows make poor use of the memory pipeline (2.4 TB/s at 16 x 16384 x 16384), whereas 16-byte chunks, consecutive lanes
// on consecutive chunks of a row, stream at the rate of the other direct-to-LDS kernels.  Per wave and k-step of 128:
// the 96 bytes of each of A's 16 rows (two instructions, the second half idle: its lanes fetch rows again into unused
// space) and of 16 CG rows of B (3 CG / 2 instructions; chunk f = 64 j + lane of instruction j is chunk f % 6 of row
// f / 6) land in a private stage with rows 96 bytes apart; NS - 1 steps in flight per wave, no barriers until the sum
// over the waves.  A lane then reads its 24 bytes as three 8-byte LDS reads.  K a multiple of 128, rows on 16-byte
// boundaries (pitches multiples of 64 elements).
// SUB k-steps of 128 make one stage (rows 96 SUB bytes apart): with SUB = 2 a wave's runs are 192 bytes on 64-byte
// boundaries, whole memory requests (96-byte runs straddle them: 1.24 x the operand's bytes came from HBM).
template <int DT, int CG, int WK, int NS, int SUB>
__global__ __launch_bounds__(64 * WK) void f6_dma_kernel(Problem p, int64_t lda_bytes, int64_t ldb_bytes, int64_t sa_bytes, int64_t sb_bytes)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int CH = 6 * SUB, PITCH = 16 * CH;                           // 16-byte chunks and bytes of a row in a stage
    constexpr int A_INSTR = (16 * CH + 63) / 64, B_INSTR = 16 * CG * CH / 64, A_AREA = A_INSTR * 1024;
    constexpr int STAGE = A_AREA + B_INSTR * 1024, LOADS = A_INSTR + B_INSTR;
    static_assert((16 * CG * CH) % 64 == 0 && (NS - 1) * LOADS < 64, "whole instructions; the counted wait has six bits");
    static_assert(WK * CG * 4 * 64 * 4 <= WK * NS * STAGE, "the reduction buffer reuses the staging area");
    extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
    ring::lds_char *const lds = (ring::lds_char *)lds_raw;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), row = lane & 15, grp = lane >> 4;
    const int64_t row_blocks = (p.M + 15) / 16, batch = blockIdx.y / row_blocks, m0 = 16 * (blockIdx.y % row_blocks);
    const int64_t n0 = (int64_t)blockIdx.x * (16 * CG);
    const char *a_base = static_cast<const char *>(p.A) + batch * sa_bytes + m0 * lda_bytes;
    const char *b_base = static_cast<const char *>(p.B) + batch * sb_bytes + n0 * ldb_bytes;
    // global side (rows beyond M or N fetch the last row again: their sums are never stored)
    uint32_t a_off[A_INSTR], b_off[B_INSTR];
#pragma unroll
    for (int j = 0; j < A_INSTR; ++j) {
        const int f = (64 * j + lane) % (16 * CH);
        const int64_t r = m0 + f / CH < p.M ? f / CH : p.M - 1 - m0;
        a_off[j] = (uint32_t)(r * lda_bytes + (f % CH) * 16);
    }
#pragma unroll
    for (int j = 0; j < B_INSTR; ++j) {
        const int f = 64 * j + lane;
        const int64_t r = n0 + f / CH < p.N ? f / CH : p.N - 1 - n0;
        b_off[j] = (uint32_t)(r * ldb_bytes + (f % CH) * 16);
    }
    const uint32_t wave_lds = (uint32_t)reinterpret_cast<uintptr_t>(lds) + wave * (NS * STAGE);
    auto issue = [&](int64_t step, int slot) {
        const char *ga = ring::scalar_ptr(a_base + step * PITCH), *gb = ring::scalar_ptr(b_base + step * PITCH);
        const uint32_t d = __builtin_amdgcn_readfirstlane(wave_lds + slot * STAGE);
#pragma unroll
        for (int j = 0; j < A_INSTR; ++j) ring::dma_load16(ga, a_off[j], d + j * 1024);
#pragma unroll
        for (int j = 0; j < B_INSTR; ++j) ring::dma_load16_once(gb, b_off[j], d + A_AREA + j * 1024);
    };
    const int rd = row * PITCH + grp * 24;                                 // this lane's first block within a group of 16 rows
    floatx4 acc[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[g] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    // this wave's steps: wave, wave + WK, ...
    const int64_t steps = p.K / (128 * SUB);
    const int64_t mine = steps > wave ? (steps - wave + WK - 1) / WK : 0;
    // ... walked from a start that differs from workgroup to workgroup and wrapping: with a pitch that is a multiple of a
    // few KiB, workgroups that all start at k = 0 sit on the same memory channels all the way
    const int64_t rot = mine > 0 ? (int64_t)blockIdx.x % mine : 0;
    auto step_of = [&](int64_t i) { return wave + ((i + rot) % mine) * WK; };
    if (mine > 0) {
        // NS - 1 steps in flight (past the end the last step is fetched again, never used, so that the wait counts
        // stay uniform)
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(step_of(s < mine ? s : mine - 1), s);
        for (int64_t i = 0; i < mine; ++i) {
            const int slot = (int)(i % NS);
            const int64_t nxt = i + NS - 1;
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(0xc07f);                    // lgkmcnt(0): the previous step's LDS reads have returned
            issue(step_of(nxt < mine ? nxt : mine - 1), (int)(nxt % NS));
            ring::wait_vmcnt<(NS - 1) * LOADS>();                  // step i has landed; its LDS reads below are new
            asm volatile("" ::: "memory");
            const ring::lds_char *st = lds + wave * (NS * STAGE) + slot * STAGE;
#pragma unroll
            for (int u = 0; u < SUB; ++u) {
                unsigned int a[6], b[CG][6];
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    const uintx2 v = *reinterpret_cast<const __attribute__((address_space(3))) uintx2 *>(st + rd + u * 96 + 8 * t);
                    a[2 * t] = v[0]; a[2 * t + 1] = v[1];
                }
#pragma unroll
                for (int g = 0; g < CG; ++g)
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        const uintx2 v = *reinterpret_cast<const __attribute__((address_space(3))) uintx2 *>(st + A_AREA + g * 16 * PITCH + rd + u * 96 + 8 * t);
                        b[g][2 * t] = v[0]; b[g][2 * t + 1] = v[1];
                    }
#pragma unroll
                for (int g = 0; g < CG; ++g) acc[g] = f6_mma<DT>(a, b[g], acc[g]);
            }
            asm volatile("" ::: "memory");                          // the reads are done before the slot is refilled
        }
        ring::wait_vmcnt<0>();
    }
    // sum the WK waves in wave order (the staging area is free now)
    __syncthreads();
    __attribute__((address_space(3))) float *part = (__attribute__((address_space(3))) float *)lds;
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) part[((wave * CG + g) * 4 + r) * 64 + lane] = acc[g][r];
    __syncthreads();
    unsigned short *C = static_cast<unsigned short *>(p.C) + batch * p.strideC;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    for (int idx = wave; idx < CG * 4; idx += WK) {
        const int g = idx >> 2, r = idx & 3;
        float z = 0.0f;
#pragma unroll
        for (int w = 0; w < WK; ++w) z += part[((w * CG + g) * 4 + r) * 64 + lane];
        const int64_t col = n0 + 16 * g + 4 * grp + r;                      // this lane: row `row` of C
        if (m0 + row < p.M && col < p.N) {
            if (bias) z += p.bias_row ? bias[m0 + row] : bias[col];
            C[(m0 + row) * p.ldc + col] = f32_to_bf16(apply_act(z, p.act));
        }
    }
#endif
}

template <int DT, int CG, int SUB>
bool f6_dma_supports(const Problem &p)
{
    if (p.dtype != DT || p.a_col() || !p.b_col() || p.M < 1 || p.M > 16 * kF6RowBlocks || p.N < 1 || p.K < 128 * SUB || p.K % (128 * SUB) != 0 || p.batch < 1 ||
        p.batch > 65535 / kF6RowBlocks)
        return false;
    // rows of 16-byte chunks; SUB >= 2: runs of 96 SUB bytes on 64-byte boundaries
    constexpr int64_t kPitch = SUB == 1 ? 64 : 256, kBase = SUB == 1 ? 16 : 64;
    if ((p.lda | p.ldb | p.strideA | p.strideB) & (kPitch - 1)) return false;
    if ((reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B)) & (uintptr_t)(kBase - 1)) return false;
    if (p.lda >= (int64_t(1) << 26) || p.ldb >= (int64_t(1) << 24)) return false;          // 32-bit offsets within a block of rows
    return (p.N + 16 * CG - 1) / (16 * CG) <= 0x7fffffffLL;
}

template <int DT, int CG, int WK, int NS, int SUB>
hipError_t f6_dma_launch(const Problem &p, hipStream_t s)
{
    constexpr int LDS_BYTES = WK * NS * ((16 * 6 * SUB + 63) / 64 * 1024 + 16 * CG * 6 * SUB / 64 * 1024);
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    if (!f6_dma_supports<DT, CG, SUB>(p)) return hipErrorInvalidValue;
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&f6_dma_kernel<DT, CG, WK, NS, SUB>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((f6_dma_kernel<DT, CG, WK, NS, SUB>), dim3((unsigned)((p.N + 16 * CG - 1) / (16 * CG)), (unsigned)(p.batch * ((p.M + 15) / 16))),
                       dim3(64 * WK), LDS_BYTES, s, p, p.lda / 4 * 3, p.ldb / 4 * 3, p.strideA / 4 * 3, p.strideB / 4 * 3);
    return hipGetLastError();
}

template <int DT>
bool f6_stream_supports(const Problem &p)
{
    if (p.dtype != DT || p.a_col() || !p.b_col() || p.M < 1 || p.M > 16 * kF6RowBlocks || p.N < 1 || p.K < 32 || p.batch < 1 ||
        p.batch > 65535 / kF6RowBlocks)
        return false;
    if ((p.K | p.lda | p.ldb | p.strideA | p.strideB) & 31) return false;                   // rows of 24-byte blocks on 8-byte boundaries
    if ((reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B)) & 7u) return false;
    return (p.N + 15) / 16 <= 0x7fffffffLL;
}

// B once at RATE GB/s (measured at 16 x 16384 x 16384, every CU with a workgroup), one launch.  Fewer workgroups than
// CUs: the rate falls with the square root of the share (16 x 8192 x 8192 at 64 columns a workgroup: 128 workgroups,
// 18.6 us); more: whole rounds of workgroups (13 x 10016 x 12032 at 32 columns: 313 workgroups take two rounds, 30.9 us
// against 25.4 us for 157 of 64 columns).
// PER_CU: workgroups a CU holds at a time (registers or LDS).
template <int CG, int RATE, int PER_CU>
double f6_stream_estimate(const Problem &p)
{
    const double rb = (double)((p.M + 15) / 16);
    const double wgs = (double)((p.N + 16 * CG - 1) / (16 * CG)) * (double)p.batch * rb, full = (double)compute_units(), cap = full * PER_CU;
    const double bytes = (double)p.batch * (double)p.N * (double)p.K * 0.75 * rb;
    const double slow = wgs >= cap ? std::ceil(wgs / cap) * cap / wgs : wgs >= full ? 1.0 : std::sqrt(full / wgs);
    return 4.0 + bytes / (1e3 * RATE) * slow;
}

template <int DT, int CG, int WK, int U>
hipError_t f6_stream_launch(const Problem &p, hipStream_t s)
{
    if (!f6_stream_supports<DT>(p)) return hipErrorInvalidValue;
    hipLaunchKernelGGL((f6_stream_kernel<DT, CG, WK, U>), dim3((unsigned)((p.N + 16 * CG - 1) / (16 * CG)), (unsigned)(p.batch * ((p.M + 15) / 16))), dim3(64 * WK), 0, s, p,
                       p.lda / 4 * 3, p.ldb / 4 * 3, p.strideA / 4 * 3, p.strideB / 4 * 3);
    return hipGetLastError();
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
         reinterpret_cast<const void *>(&ring::gemm_ring_kernel<F6Cfg<DT_BF6>>), nullptr, true, f6_estimate},
#define F6_STREAM(DT, TAG, CG, WK, U, RATE, PER_CU)                                                                                  \
    {"stream6_" TAG "_rc_cg" #CG "_wk" #WK "_u" #U, f6_stream_supports<DT>, f6_stream_launch<DT, CG, WK, U>, 16, 16 * CG,       \
     reinterpret_cast<const void *>(&f6_stream_kernel<DT, CG, WK, U>), nullptr, true, f6_stream_estimate<CG, RATE, PER_CU>}
        F6_STREAM(DT_F6, "f6", 1, 4, 4, 2000, 4), F6_STREAM(DT_BF6, "bf6", 1, 4, 4, 2000, 4),
        F6_STREAM(DT_F6, "f6", 2, 4, 4, 2300, 3), F6_STREAM(DT_BF6, "bf6", 2, 4, 4, 2300, 3),
        F6_STREAM(DT_F6, "f6", 4, 8, 2, 2600, 1), F6_STREAM(DT_BF6, "bf6", 4, 8, 2, 2600, 1),
#define F6_DMA(DT, TAG, CG, WK, NS, SUB, RATE, PER_CU)                                                                                      \
    {"stream6_" TAG "_rc_dma_cg" #CG "_wk" #WK "_ns" #NS "_sub" #SUB, f6_dma_supports<DT, CG, SUB>, f6_dma_launch<DT, CG, WK, NS, SUB>, 16, \
     16 * CG, reinterpret_cast<const void *>(&f6_dma_kernel<DT, CG, WK, NS, SUB>), nullptr, true, f6_stream_estimate<CG, RATE, PER_CU>}
        F6_DMA(DT_F6, "f6", 2, 4, 4, 1, 4000, 1), F6_DMA(DT_BF6, "bf6", 2, 4, 4, 1, 4000, 1),
        F6_DMA(DT_F6, "f6", 4, 8, 2, 1, 4100, 1), F6_DMA(DT_BF6, "bf6", 4, 8, 2, 1, 4100, 1),
        F6_DMA(DT_F6, "f6", 2, 4, 3, 2, 4400, 1), F6_DMA(DT_BF6, "bf6", 2, 4, 3, 2, 4400, 1),
        F6_DMA(DT_F6, "f6", 4, 4, 2, 2, 4900, 1), F6_DMA(DT_BF6, "bf6", 4, 4, 2, 2, 4900, 1)};
#undef F6_DMA
#undef F6_STREAM
    return v;
}

}  // namespace optiml

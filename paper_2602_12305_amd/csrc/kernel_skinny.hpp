// Streaming kernels for 16 rows of A at a time (fp32, A and B row-major).
//
// With M <= 16 the contraction reads every element of B once and uses it for 16
// multiply-adds: HBM bandwidth is the bound, and the whole design serves one
// goal - keep many 128-bit loads of B in flight on every CU and touch each byte
// of B exactly once.  The paper's own matmul trajectory names the same levers for
// its memory-side bottleneck (appendix "How OptiML-X improves the kernel":
// vectorised loads to cut transactions, reuse from on-chip storage); what is
// specific to gfx950 here is that the 16 multiply-adds per element go to the
// matrix pipe (v_mfma_f32_16x16x4_f32: M = 16 is exactly one MFMA tile), which
// leaves the vector ALUs to address generation.
//
// Work split.  A workgroup is WN x WK waves.  Along n a wave owns CG groups of 64
// columns; along k the WK waves of a workgroup, times SPLIT workgroups (grid.y),
// own contiguous ranges of 16-row "super-steps".  Lane (q = lane/16, c = lane%16)
// loads, per super-step at k0:
//     A[c][k0+4q .. k0+4q+3]                        one 128-bit load (L2 resident)
//     B[k0+4q+t][n0 + 64g + 4c .. +3], t = 0..3     four 128-bit loads per group g
// MFMA number (t, cc) multiplies A-register component t with component cc of B load
// t: lane group q supplies k = k0+4q+t on both sides, and output column j = c stands
// for n = n0 + 64g + 4c + cc.  Accumulator (g, cc) register r of lane (q, c) is then
// Z[4q + r][n0 + 64g + 4c + cc]: four consecutive n per lane, stored as one 128-bit
// vector.
//
// Reduction over k is deterministic: the WK waves of a workgroup leave their
// accumulators in LDS and are summed in wave order; with SPLIT > 1 the per-workgroup
// sums go to a workspace [SPLIT][batch][16][N] and a second kernel adds them in
// split order, then applies bias and activation.  No atomics anywhere.
//
// More than 16 rows.  grid.z also counts blocks of 16 rows of A and C: every block streams B
// again (from L2), which only pays while the whole problem is small - a few hundred rows of a
// B that fits L2 - and the MFMA tile kernels would leave most CUs idle (256^3: 16 workgroups
// of the 64x64 tile kernel take 17 us, this path spreads the same work over 128).
#pragma once
#include "common.hpp"
#include "epilogue.hpp"
#include "kernel_tile_ring.hpp"      // the LDS-DMA load, the hand-counted wait, the scalarised pointer

namespace optiml {
namespace skinny {

typedef float floatx4 __attribute__((ext_vector_type(4)));

struct SkinnyParams {
    int64_t M, N, K;
    const float *A; int64_t lda, strideA;
    const float *B; int64_t ldb, strideB;
    const float *bias; int64_t strideBias;
    int bias_row;          // bias[m] (the row of C) instead of bias[n]
    float *C; int64_t ldc, strideC;
    float *partial;        // [split][batch * row_blocks][16][N] when split > 1
    int64_t batch, row_blocks;
    int split, act;
};

// SS = super-steps (of 16 k) per pipelined batch of loads; two batches are live at a time

template <int CG, int SS>
struct Stage {
    floatx4 a[SS];
    floatx4 b[SS][CG][4];
};

template <int CG, int SS, bool NT>
__device__ __forceinline__ void load_stage(Stage<CG, SS> &st, const float *a_ptr, const float *b_ptr, int64_t ldb,
                                           bool a_valid, const bool (&col_valid)[CG])
{
#pragma unroll
    for (int s = 0; s < SS; ++s) {
        st.a[s] = a_valid ? *reinterpret_cast<const floatx4 *>(a_ptr + 16 * s) : floatx4{0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const floatx4 *src = reinterpret_cast<const floatx4 *>(b_ptr + (16 * s + t) * ldb + 64 * g);
                if (col_valid[g])
                    st.b[s][g][t] = NT ? __builtin_nontemporal_load(src) : *src;
                else
                    st.b[s][g][t] = floatx4{0, 0, 0, 0};
            }
    }
}

template <int CG, int SS>
__device__ __forceinline__ void mma_stage(const Stage<CG, SS> &st, floatx4 (&acc)[CG][4])
{
#pragma unroll
    for (int s = 0; s < SS; ++s)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int g = 0; g < CG; ++g)
#pragma unroll
                for (int cc = 0; cc < 4; ++cc)
                    acc[g][cc] = __builtin_amdgcn_mfma_f32_16x16x4f32(st.a[s][t], st.b[s][g][t][cc], acc[g][cc], 0, 0, 0);
}

// IL: the WK waves of a workgroup take the batches of SS super-steps of the workgroup's k range in
// turn (wave w: batches w, w + WK, ...) instead of one contiguous sub-range each, so that all
// waves of all workgroups of a split read neighbouring rows of B at any moment.
template <int WN, int WK, int CG, bool NT, bool IL = false>
__global__ __launch_bounds__(64 * WN * WK) void skinny_kernel(SkinnyParams p)
{
    // register budget: 128 per lane for 16 waves, 256 up to 8 waves
    constexpr int SS = (WN * WK > 8) ? 1 : (CG > 1 ? 2 : 4);
    constexpr int COLS = 64 * CG * WN;          // columns per workgroup
    constexpr int THREADS = 64 * WN * WK;
    __shared__ floatx4 red[WK > 1 ? WK * 16 * (COLS / 4) : 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % WN, wk = wave / WN;
    const int q = lane >> 4, c = lane & 15;
    const int64_t zb = blockIdx.z, batch = zb / p.row_blocks, rb = zb % p.row_blocks;
    const int64_t rows = p.M - 16 * rb < 16 ? p.M - 16 * rb : 16;       // rows of this block
    const int64_t nblock0 = (int64_t)blockIdx.x * COLS;
    const int64_t n0 = nblock0 + (int64_t)wn * CG * 64 + 4 * c;   // this lane's first column in group 0

    // super-steps of this (split, wk): first full batch (s), distance between batches, number of
    // full batches, and the range [tail, s_end) of left-over steps taken one at a time
    const int64_t steps = (p.K + 15) / 16, full_steps = p.K / 16;   // full: all 16 rows below K
    int64_t s, batch_stride, nbatches, tail, s_end;
    if (IL) {
        const int64_t g0 = steps * blockIdx.y / p.split, g1 = steps * (blockIdx.y + 1) / p.split;
        const int64_t g1f = g1 < full_steps ? g1 : full_steps;
        const int64_t total = g1f > g0 ? (g1f - g0) / SS : 0;   // full batches of the workgroup
        s = g0 + (int64_t)wk * SS;
        batch_stride = (int64_t)SS * WK;
        nbatches = total > wk ? (total - wk + WK - 1) / WK : 0;
        tail = g0 + total * SS;
        s_end = wk == 0 ? g1 : tail;                            // wave 0 takes what the batches leave
    } else {
        const int64_t parts = (int64_t)p.split * WK, part = (int64_t)blockIdx.y * WK + wk;
        s = steps * part / parts;
        s_end = steps * (part + 1) / parts;
        const int64_t s_full_end = s_end < full_steps ? s_end : full_steps;
        batch_stride = SS;
        nbatches = s_full_end > s ? (s_full_end - s) / SS : 0;
        tail = s + nbatches * SS;
    }

    const float *A = p.A + batch * p.strideA + 16 * rb * p.lda;
    const float *B = p.B + batch * p.strideB;
    const bool a_row_valid = c < rows;
    bool col_valid[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) col_valid[g] = n0 + 64 * g < p.N;     // N % 4 == 0: whole vectors

    floatx4 acc[CG][4];
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) acc[g][cc] = floatx4{0, 0, 0, 0};

    // full batches of SS super-steps whose last row is below K
    const float *a_ptr = A + (int64_t)c * p.lda + 16 * s + 4 * q;
    const float *b_ptr = B + (16 * s + 4 * q) * p.ldb + n0;
    if (nbatches > 0) {
        Stage<CG, SS> cur, nxt;
        load_stage<CG, SS, NT>(cur, a_ptr, b_ptr, p.ldb, a_row_valid, col_valid);
        for (int64_t it = 1; it < nbatches; ++it) {
            a_ptr += 16 * batch_stride;
            b_ptr += 16 * batch_stride * p.ldb;
            load_stage<CG, SS, NT>(nxt, a_ptr, b_ptr, p.ldb, a_row_valid, col_valid);
            mma_stage<CG, SS>(cur, acc);
            cur = nxt;
        }
        mma_stage<CG, SS>(cur, acc);
    }
    s = tail;
    a_ptr = A + (int64_t)c * p.lda + 16 * s + 4 * q;
    b_ptr = B + (16 * s + 4 * q) * p.ldb + n0;
    // remaining super-steps one at a time, rows guarded against K (K % 4 == 0: a lane's four
    // rows k0+4q..k0+4q+3 are valid together)
    for (; s < s_end; ++s) {
        const bool k_valid = 16 * s + 4 * q < p.K;
        floatx4 a = floatx4{0, 0, 0, 0};
        if (k_valid && a_row_valid) a = *reinterpret_cast<const floatx4 *>(a_ptr);
#pragma unroll
        for (int g = 0; g < CG; ++g) {
            floatx4 b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                b[t] = floatx4{0, 0, 0, 0};
                if (k_valid && col_valid[g]) b[t] = *reinterpret_cast<const floatx4 *>(b_ptr + t * p.ldb + 64 * g);
            }
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int cc = 0; cc < 4; ++cc)
                    acc[g][cc] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t][cc], acc[g][cc], 0, 0, 0);
        }
        a_ptr += 16;
        b_ptr += 16 * p.ldb;
    }

    // accumulator (g, cc) register r of lane (q, c) is Z[4q + r][n0 + 64 g + cc]
    if (WK > 1) {
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 4 * q + r, col4 = (wn * CG + g) * 16 + c;
                red[(wk * 16 + row) * (COLS / 4) + col4] = floatx4{acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]};
            }
        __syncthreads();
    }

    float *out = p.split > 1 ? p.partial + ((int64_t)blockIdx.y * p.batch * p.row_blocks + zb) * 16 * p.N
                             : p.C + batch * p.strideC + 16 * rb * p.ldc;
    const int64_t out_ld = p.split > 1 ? p.N : p.ldc;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;

    auto finish = [&](int row, int64_t col, floatx4 z) {
        if (row >= rows || col >= p.N) return;
        if (p.split == 1) {
            floatx4 bj = floatx4{0, 0, 0, 0};
            if (bias && p.bias_row) { const float b = bias[16 * rb + row]; bj = floatx4{b, b, b, b}; }
            else if (bias) bj = *reinterpret_cast<const floatx4 *>(bias + col);
#pragma unroll
            for (int e = 0; e < 4; ++e) z[e] = apply_act(z[e] + bj[e], p.act);
        }
        *reinterpret_cast<floatx4 *>(out + (int64_t)row * out_ld + col) = z;
    };

    if (WK > 1) {
        for (int e = tid; e < 16 * (COLS / 4); e += THREADS) {
            const int row = e / (COLS / 4), col4 = e % (COLS / 4);
            floatx4 z = red[row * (COLS / 4) + col4];
#pragma unroll
            for (int w = 1; w < WK; ++w) {
                const floatx4 v = red[(w * 16 + row) * (COLS / 4) + col4];
                z += v;
            }
            finish(row, nblock0 + 4 * col4, z);
        }
    } else {
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                finish(4 * q + r, n0 + 64 * g, floatx4{acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]});
    }
}

// The same walk with B brought to LDS by direct loads instead of through registers (16 x 16384 x
// 16384: 0.159 against 0.168 ms per call).  A workgroup is WK waves deep in k and 64 CG columns
// wide; its waves take the steps of 16 rows of its k range in turn, and every wave stages only
// what it consumes itself, NS - 1 steps ahead: one 1 KiB block of A (16 rows x 16 k) and CG
// 4 KiB blocks of B (16 k-rows x 64 columns, row-major as in memory) per step, no barriers, just
// counted waits (loads complete in issue order).  Lane (q, c) then reads A[c][4q .. 4q+3] and, for
// t = 0..3, B[4q + t][4c .. 4c+3] of every group back as 128-bit vectors and feeds the same
// matrix instructions as skinny_kernel; the accumulators, the sum over the waves in wave order,
// the partial sums of a split along k and the second kernel are the same too.  A's 16-byte chunks
// sit in LDS XORed with bits 2-3 of their row, so that the 16 lanes of a read (64 bytes apart)
// spread over the banks.  NT: B is loaded with the non-temporal hint (read once: a single block of
// rows); without it B stays in the caches for the other blocks of rows.
template <int WK, int CG, int NS, bool NT>
__global__ __launch_bounds__(64 * WK) void skinny_dma_kernel(SkinnyParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int COLS = 64 * CG, THREADS = 64 * WK;
    constexpr int STAGE = 1024 + CG * 4096, LOADS = 1 + 4 * CG;     // bytes and DMA instructions per step
    extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
    ring::lds_char *const lds = (ring::lds_char *)lds_raw;
    static_assert(WK * 16 * COLS * 4 <= WK * NS * STAGE, "the reduction buffer reuses the staging area");
    static_assert((NS - 1) * LOADS < 64, "the counted wait has six bits");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4, c = lane & 15;
    const int64_t zb = blockIdx.z, batch = zb / p.row_blocks, rb = zb % p.row_blocks;
    const int64_t rows = p.M - 16 * rb < 16 ? p.M - 16 * rb : 16;
    const int64_t nblock0 = (int64_t)blockIdx.x * COLS;
    const int64_t n0 = nblock0 + 4 * c;

    const int64_t steps = (p.K + 15) / 16, full_steps = p.K / 16;   // full: all 16 rows below K
    const int64_t g0 = steps * blockIdx.y / p.split, g1 = steps * (blockIdx.y + 1) / p.split;
    const int64_t g1f = g1 < full_steps ? g1 : full_steps;

    const float *A = p.A + batch * p.strideA + 16 * rb * p.lda;
    const float *B = p.B + batch * p.strideB;
    // global side.  A's instruction: lane l fetches the chunk (l % 4) ^ (row / 4 % 4) of row l / 4
    // (rows past the end re-read the last one: their sums are never stored).  Instruction i of B's
    // group g: lane l fetches columns 64 g + 4 (l % 16) .. +3 of row 4 i + l / 16 (columns past N
    // re-read the last four).
    uint32_t a_off, b_off[CG][4];
    {
        const int r = lane >> 2;
        const int64_t row = r < rows ? r : rows - 1;
        a_off = (uint32_t)((row * p.lda + 4 * ((lane & 3) ^ ((r >> 2) & 3))) * 4);
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int64_t col = nblock0 + 64 * g + 4 * (lane & 15);
                col = col < p.N ? col : p.N - 4;
                b_off[g][i] = (uint32_t)(((4 * i + (lane >> 4)) * p.ldb + (col - nblock0)) * 4);
            }
    }
    const char *a_base = reinterpret_cast<const char *>(A), *b_base = reinterpret_cast<const char *>(B + nblock0);
    const uint32_t wave_lds = (uint32_t)reinterpret_cast<uintptr_t>(lds) + wave * (NS * STAGE);
    auto issue = [&](int64_t step, int slot) {
        const char *ga = ring::scalar_ptr(a_base + step * 64), *gb = ring::scalar_ptr(b_base + step * 64 * p.ldb);
        const uint32_t d = __builtin_amdgcn_readfirstlane(wave_lds + slot * STAGE);
        ring::dma_load16(ga, a_off, d);
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (NT) ring::dma_load16_once(gb, b_off[g][i], d + 1024 + g * 4096 + i * 1024);
                else ring::dma_load16(gb, b_off[g][i], d + 1024 + g * 4096 + i * 1024);
            }
    };
    // LDS side of this lane
    const int rd_a = c * 64 + ((q ^ ((c >> 2) & 3)) << 4);
    const int rd_b = 1024 + 4 * q * 256 + c * 16;

    floatx4 acc[CG][4];
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) acc[g][cc] = floatx4{0, 0, 0, 0};

    // this wave's full steps: wave, wave + WK, ... of the workgroup's range
    const int64_t nfull = g1f > g0 ? g1f - g0 : 0;
    const int64_t mine = nfull > wave ? (nfull - wave + WK - 1) / WK : 0;
    auto step_of = [&](int64_t i) { return g0 + wave + i * WK; };
    if (mine > 0) {
        // NS - 1 steps in flight (past the end the last step is fetched again, never used, so that
        // the wait counts stay uniform)
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
            const floatx4 a = *reinterpret_cast<const __attribute__((address_space(3))) floatx4 *>(st + rd_a);
#pragma unroll
            for (int g = 0; g < CG; ++g)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const floatx4 b = *reinterpret_cast<const __attribute__((address_space(3))) floatx4 *>(st + rd_b + g * 4096 + t * 256);
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc)
                        acc[g][cc] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[cc], acc[g][cc], 0, 0, 0);
                }
            asm volatile("" ::: "memory");                          // the reads are done before the slot is refilled
        }
        ring::wait_vmcnt<0>();
    }
    // the ragged last step straight from memory, rows guarded against K (K % 4 == 0: a lane's four
    // rows are valid together), by wave 0 of the split that holds it
    const bool a_row_valid = c < rows;
    if (wave == 0) {
        for (int64_t s = g1f > g0 ? g1f : g0; s < g1; ++s) {
            const bool k_valid = 16 * s + 4 * q < p.K;
            floatx4 a = floatx4{0, 0, 0, 0};
            if (k_valid && a_row_valid) a = *reinterpret_cast<const floatx4 *>(A + (int64_t)c * p.lda + 16 * s + 4 * q);
#pragma unroll
            for (int g = 0; g < CG; ++g)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    floatx4 b = floatx4{0, 0, 0, 0};
                    if (k_valid && n0 + 64 * g < p.N)
                        b = *reinterpret_cast<const floatx4 *>(B + (16 * s + 4 * q + t) * p.ldb + n0 + 64 * g);
#pragma unroll
                    for (int cc = 0; cc < 4; ++cc)
                        acc[g][cc] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[cc], acc[g][cc], 0, 0, 0);
                }
        }
    }

    // sum the WK waves in wave order (the staging area is free now)
    __syncthreads();
    floatx4 *red = reinterpret_cast<floatx4 *>(lds_raw);
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r)
            red[(wave * 16 + 4 * q + r) * (COLS / 4) + g * 16 + c] = floatx4{acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]};
    __syncthreads();

    float *out = p.split > 1 ? p.partial + ((int64_t)blockIdx.y * p.batch * p.row_blocks + zb) * 16 * p.N
                             : p.C + batch * p.strideC + 16 * rb * p.ldc;
    const int64_t out_ld = p.split > 1 ? p.N : p.ldc;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    for (int e = tid; e < 16 * (COLS / 4); e += THREADS) {
        const int row = e / (COLS / 4), col4 = e % (COLS / 4);
        floatx4 z = red[row * (COLS / 4) + col4];
#pragma unroll
        for (int w = 1; w < WK; ++w) {
            const floatx4 v = red[(w * 16 + row) * (COLS / 4) + col4];
            z += v;
        }
        const int64_t col = nblock0 + 4 * col4;
        if (row >= rows || col >= p.N) continue;
        if (p.split == 1) {
            floatx4 bj = floatx4{0, 0, 0, 0};
            if (bias && p.bias_row) { const float b = bias[16 * rb + row]; bj = floatx4{b, b, b, b}; }
            else if (bias) bj = *reinterpret_cast<const floatx4 *>(bias + col);
#pragma unroll
            for (int k = 0; k < 4; ++k) z[k] = apply_act(z[k] + bj[k], p.act);
        }
        *reinterpret_cast<floatx4 *>(out + (int64_t)row * out_ld + col) = z;
    }
#endif
}

// C = act(bias + sum over splits of partial), splits added in ascending order
__global__ __launch_bounds__(256) void skinny_reduce_kernel(SkinnyParams p)
{
    const int64_t n4 = p.N / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t batch = blockIdx.y;
    if (idx >= p.M * n4) return;
    const int64_t row = idx / n4, col = 4 * (idx % n4);
    const int64_t zb = batch * p.row_blocks + row / 16;
    floatx4 z = floatx4{0, 0, 0, 0};
    for (int s = 0; s < p.split; ++s)
        z += *reinterpret_cast<const floatx4 *>(
            p.partial + (((int64_t)s * p.batch * p.row_blocks + zb) * 16 + row % 16) * p.N + col);
    floatx4 bj = floatx4{0, 0, 0, 0};
    if (p.bias && p.bias_row) { const float b = p.bias[batch * p.strideBias + row]; bj = floatx4{b, b, b, b}; }
    else if (p.bias) bj = *reinterpret_cast<const floatx4 *>(p.bias + batch * p.strideBias + col);
#pragma unroll
    for (int e = 0; e < 4; ++e) z[e] = apply_act(z[e] + bj[e], p.act);
    *reinterpret_cast<floatx4 *>(p.C + batch * p.strideC + row * p.ldc + col) = z;
}

inline bool skinny_supports(const Problem &p)
{
    return p.dtype == DT_F32 && p.layout == 0 && p.M >= 1 && p.K >= 4 && p.K % 4 == 0 &&
           p.N % 4 == 0 && p.batch * ((p.M + 15) / 16) <= 65535 && vector_friendly(p);
}

template <int WN, int WK, int CG, bool NT, int SPLIT, bool IL = false>
hipError_t skinny_launch(const Problem &p, hipStream_t stream)
{
    constexpr int COLS = 64 * CG * WN;
    SkinnyParams sp;
    sp.M = p.M; sp.N = p.N; sp.K = p.K;
    sp.A = static_cast<const float *>(p.A); sp.lda = p.lda; sp.strideA = p.strideA;
    sp.B = static_cast<const float *>(p.B); sp.ldb = p.ldb; sp.strideB = p.strideB;
    sp.bias = p.bias; sp.strideBias = p.strideBias; sp.bias_row = p.bias_row ? 1 : 0;
    sp.C = static_cast<float *>(p.C); sp.ldc = p.ldc; sp.strideC = p.strideC;
    sp.batch = p.batch; sp.act = p.act;
    sp.row_blocks = (p.M + 15) / 16;
    // SPLIT == 0: enough workgroups for one per CU when a workgroup has eight or more waves or
    // interleaves its waves in k, else about two per CU, but never ranges shorter than 256 rows
    int split = SPLIT;
    if (SPLIT == 0) {
        const int64_t col_blocks = (p.N + COLS - 1) / COLS * p.batch * sp.row_blocks;
        const int64_t target = (IL || WN * WK >= 8) ? 256 : 512;
        const int64_t by_grid = (target + col_blocks - 1) / col_blocks;
        const int64_t by_k = p.K / (256 * WK) > 0 ? p.K / (256 * WK) : 1;
        split = (int)(by_grid < by_k ? by_grid : by_k);
        if (split < 1) split = 1;
        if (split > 64) split = 64;
    }
    sp.split = split;
    sp.partial = nullptr;
    if (split > 1) {
        void *ws = nullptr;
        hipError_t e = workspace(sizeof(float) * (size_t)split * p.batch * sp.row_blocks * 16 * p.N, &ws, stream);
        if (e != hipSuccess) return e;
        sp.partial = static_cast<float *>(ws);
    }
    dim3 grid((unsigned)((p.N + COLS - 1) / COLS), (unsigned)split, (unsigned)(p.batch * sp.row_blocks));
    hipLaunchKernelGGL((skinny_kernel<WN, WK, CG, NT, IL>), grid, dim3(64 * WN * WK), 0, stream, sp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t vecs = p.M * (p.N / 4);
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3((unsigned)((vecs + 255) / 256), (unsigned)p.batch), dim3(256), 0,
                       stream, sp);
    return hipGetLastError();
}

// 32-bit byte offsets inside a step of 16 rows
inline bool skinny_dma_supports(const Problem &p)
{
    return skinny_supports(p) && p.ldb < (1ll << 24) && p.lda < (1ll << 24);
}

template <int WK, int CG, int NS, bool NT>
hipError_t skinny_dma_launch(const Problem &p, hipStream_t stream)
{
    constexpr int COLS = 64 * CG, LDS_BYTES = WK * NS * (1024 + CG * 4096);
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&skinny_dma_kernel<WK, CG, NS, NT>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    SkinnyParams sp;
    sp.M = p.M; sp.N = p.N; sp.K = p.K;
    sp.A = static_cast<const float *>(p.A); sp.lda = p.lda; sp.strideA = p.strideA;
    sp.B = static_cast<const float *>(p.B); sp.ldb = p.ldb; sp.strideB = p.strideB;
    sp.bias = p.bias; sp.strideBias = p.strideBias; sp.bias_row = p.bias_row ? 1 : 0;
    sp.C = static_cast<float *>(p.C); sp.ldc = p.ldc; sp.strideC = p.strideC;
    sp.batch = p.batch; sp.act = p.act;
    sp.row_blocks = (p.M + 15) / 16;
    // never ranges shorter than 256 rows per wave
    const int64_t col_blocks = (p.N + COLS - 1) / COLS * p.batch * sp.row_blocks;
    const int64_t by_k = p.K / (256 * WK) > 0 ? p.K / (256 * WK) : 1;
    const int64_t split = stream_split(col_blocks, 4.0 * COLS * (double)p.K, by_k, 64.0 * (double)p.N * (double)(p.batch * sp.row_blocks));
    sp.split = (int)split;
    sp.partial = nullptr;
    if (split > 1) {
        void *ws = nullptr;
        hipError_t e = workspace(sizeof(float) * (size_t)split * p.batch * sp.row_blocks * 16 * p.N, &ws, stream);
        if (e != hipSuccess) return e;
        sp.partial = static_cast<float *>(ws);
    }
    if ((p.N + COLS - 1) / COLS > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)((p.N + COLS - 1) / COLS), (unsigned)split, (unsigned)(p.batch * sp.row_blocks));
    hipLaunchKernelGGL((skinny_dma_kernel<WK, CG, NS, NT>), grid, dim3(64 * WK), LDS_BYTES, stream, sp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t vecs = p.M * (p.N / 4);
    hipLaunchKernelGGL(skinny_reduce_kernel, dim3((unsigned)((vecs + 255) / 256), (unsigned)p.batch), dim3(256), 0,
                       stream, sp);
    return hipGetLastError();
}

}  // namespace skinny
}  // namespace optiml

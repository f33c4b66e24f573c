// Streaming kernels for 16 rows of A at a time, 16-bit storage (bf16 or fp16), A and B row-major:
// the 16-bit sibling of kernel_skinny.hpp, same work split, same deterministic reductions.
//
// With M <= 16 every element of B is read once and used for 16 multiply-adds: HBM bandwidth is
// the bound.  The 16 multiply-adds go to the matrix pipe as v_mfma_f32_16x16x16 (bf16 or f16),
// whose B operand wants four consecutive k of ONE column per lane, while a 128-bit load of
// row-major B brings eight consecutive columns of one k.  Lane (q = lane/16, c = lane%16)
// therefore loads, per super-step of 16 k at k0,
//     A[c][k0+4q .. k0+4q+3]                          one 64-bit load (L2 resident)
//     B[k0+4q+t][n0 + 128g + 8c .. +7], t = 0..3      four 128-bit loads per group g of 128 columns
// and builds the operand of MFMA number cc (0..7) from the 16-bit element at position cc of each
// of the four loads (two v_perm_b32 per operand - a few per cent of the vector ALU's time at full
// bandwidth).  Lane group q supplies k = k0+4q..+3 on both sides, output column j = c stands for
// n = n0 + 128g + 8c + cc, and accumulator (g, cc) register r of lane (q, c) is
// Z[4q + r][n0 + 128g + 8c + cc]: eight consecutive n per lane and row, stored as one 128-bit
// vector of 16-bit results.
//
// Reduction over k: the WK waves of a workgroup leave their accumulators in LDS and are summed in
// wave order; with SPLIT > 1 the per-workgroup fp32 sums go to a workspace
// [SPLIT][batch * row blocks][16][N] and a second kernel adds them in split order, then applies
// bias and activation and rounds once.  No atomics.  More than 16 rows: grid.z also counts blocks
// of 16 rows, each streaming B again.
#pragma once
#include "common.hpp"
#include "epilogue.hpp"
#include "kernel_tile_ring.hpp"      // the LDS-DMA load, the hand-counted wait, the scalarised pointer

namespace optiml {
namespace skinny16 {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));

struct Params {
    int64_t M, N, K;
    const unsigned short *A; int64_t lda, strideA;
    const unsigned short *B; int64_t ldb, strideB;
    const float *bias; int64_t strideBias;
    int bias_row;          // bias[m] (the row of C) instead of bias[n]
    unsigned short *C; int64_t ldc, strideC;
    float *partial;        // [split][batch * row_blocks][16][N] when split > 1
    int64_t batch, row_blocks;
    int split, act;
};

// SS = super-steps (of 16 k) per pipelined batch of loads; two batches are live at a time
template <int CG, int SS>
struct Stage {
    uintx2 a[SS];
    uintx4 b[SS][CG][4];
};

template <int CG, int SS, bool NT>
__device__ __forceinline__ void load_stage(Stage<CG, SS> &st, const unsigned short *a_ptr, const unsigned short *b_ptr,
                                           int64_t ldb, bool a_valid, const bool (&col_valid)[CG])
{
#pragma unroll
    for (int s = 0; s < SS; ++s) {
        st.a[s] = a_valid ? *reinterpret_cast<const uintx2 *>(a_ptr + 16 * s) : uintx2{0, 0};
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uintx4 *src = reinterpret_cast<const uintx4 *>(b_ptr + (16 * s + t) * ldb + 128 * g);
                if (col_valid[g])
                    st.b[s][g][t] = NT ? __builtin_nontemporal_load(src) : *src;
                else
                    st.b[s][g][t] = uintx4{0, 0, 0, 0};
            }
    }
}

// the sixteen multiply-adds of one super-step and one group: b[t] holds row k0+4q+t, columns 8c..8c+7
template <int DT>
__device__ __forceinline__ void mma_group(uintx2 a, const uintx4 (&b)[4], floatx4 (&acc)[8])
{
#if defined(__HIP_DEVICE_COMPILE__)
#pragma unroll
    for (int cc = 0; cc < 8; ++cc) {
        const int w = cc >> 1;
        const unsigned sel = (cc & 1) ? 0x07060302u : 0x05040100u;       // the high or the low halves of two dwords
        const uintx2 col = uintx2{__builtin_amdgcn_perm(b[1][w], b[0][w], sel), __builtin_amdgcn_perm(b[3][w], b[2][w], sel)};
        if constexpr (DT == DT_F16)
            acc[cc] = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(halfx4, a), __builtin_bit_cast(halfx4, col),
                                                            acc[cc], 0, 0, 0);
        else
            acc[cc] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, a), __builtin_bit_cast(shortx4, col),
                                                                acc[cc], 0, 0, 0);
    }
#endif
}

template <int DT, int CG, int SS>
__device__ __forceinline__ void mma_stage(const Stage<CG, SS> &st, floatx4 (&acc)[CG][8])
{
#pragma unroll
    for (int s = 0; s < SS; ++s)
#pragma unroll
        for (int g = 0; g < CG; ++g) mma_group<DT>(st.a[s], st.b[s][g], acc[g]);
}

// IL: the WK waves of a workgroup take the batches of SS super-steps of the workgroup's k range in
// turn (wave w: batches w, w + WK, ...) instead of one contiguous sub-range each, so that all
// waves of all workgroups of a split read neighbouring rows of B at any moment.
template <int DT, int WN, int WK, int CG, bool NT, bool IL>
__global__ __launch_bounds__(64 * WN * WK) void skinny16_kernel(Params p)
{
    constexpr int SS = (WN * WK > 8) ? 1 : (CG > 1 ? 2 : 4);
    constexpr int COLS = 128 * CG * WN;         // columns per workgroup
    constexpr int C4 = COLS / 4;                // 4-column vectors per row of the reduction buffer
    constexpr int THREADS = 64 * WN * WK;
    __shared__ floatx4 red[WK > 1 ? WK * 16 * C4 : 1];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % WN, wk = wave / WN;
    const int q = lane >> 4, c = lane & 15;
    const int64_t zb = blockIdx.z, batch = zb / p.row_blocks, rb = zb % p.row_blocks;
    const int64_t rows = p.M - 16 * rb < 16 ? p.M - 16 * rb : 16;       // rows of this block
    const int64_t nblock0 = (int64_t)blockIdx.x * COLS;
    const int64_t n0 = nblock0 + (int64_t)wn * CG * 128 + 8 * c;        // this lane's first column in group 0

    // super-steps of this (split, wk): first full batch (s), distance between batches, number of
    // full batches, and the range [tail, s_end) of left-over steps taken one at a time
    const int64_t steps = (p.K + 15) / 16, full_steps = p.K / 16;       // full: all 16 rows below K
    int64_t s, batch_stride, nbatches, tail, s_end;
    if (IL) {
        const int64_t g0 = steps * blockIdx.y / p.split, g1 = steps * (blockIdx.y + 1) / p.split;
        const int64_t g1f = g1 < full_steps ? g1 : full_steps;
        const int64_t total = g1f > g0 ? (g1f - g0) / SS : 0;           // full batches of the workgroup
        s = g0 + (int64_t)wk * SS;
        batch_stride = (int64_t)SS * WK;
        nbatches = total > wk ? (total - wk + WK - 1) / WK : 0;
        tail = g0 + total * SS;
        s_end = wk == 0 ? g1 : tail;                                    // wave 0 takes what the batches leave
    } else {
        const int64_t parts = (int64_t)p.split * WK, part = (int64_t)blockIdx.y * WK + wk;
        s = steps * part / parts;
        s_end = steps * (part + 1) / parts;
        const int64_t s_full_end = s_end < full_steps ? s_end : full_steps;
        batch_stride = SS;
        nbatches = s_full_end > s ? (s_full_end - s) / SS : 0;
        tail = s + nbatches * SS;
    }

    const unsigned short *A = p.A + batch * p.strideA + 16 * rb * p.lda;
    const unsigned short *B = p.B + batch * p.strideB;
    const bool a_row_valid = c < rows;
    bool col_valid[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) col_valid[g] = n0 + 128 * g < p.N;     // N % 8 == 0: whole vectors

    floatx4 acc[CG][8];
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) acc[g][cc] = floatx4{0, 0, 0, 0};

    // full batches of SS super-steps whose last row is below K
    const unsigned short *a_ptr = A + (int64_t)c * p.lda + 16 * s + 4 * q;
    const unsigned short *b_ptr = B + (16 * s + 4 * q) * p.ldb + n0;
    if (nbatches > 0) {
        Stage<CG, SS> cur, nxt;
        load_stage<CG, SS, NT>(cur, a_ptr, b_ptr, p.ldb, a_row_valid, col_valid);
        for (int64_t it = 1; it < nbatches; ++it) {
            a_ptr += 16 * batch_stride;
            b_ptr += 16 * batch_stride * p.ldb;
            load_stage<CG, SS, NT>(nxt, a_ptr, b_ptr, p.ldb, a_row_valid, col_valid);
            mma_stage<DT, CG, SS>(cur, acc);
            cur = nxt;
        }
        mma_stage<DT, CG, SS>(cur, acc);
    }
    s = tail;
    a_ptr = A + (int64_t)c * p.lda + 16 * s + 4 * q;
    b_ptr = B + (16 * s + 4 * q) * p.ldb + n0;
    // remaining super-steps one at a time, rows guarded against K (K % 4 == 0: a lane's four rows
    // k0+4q..k0+4q+3 are valid together)
    for (; s < s_end; ++s) {
        const bool k_valid = 16 * s + 4 * q < p.K;
        uintx2 a = uintx2{0, 0};
        if (k_valid && a_row_valid) a = *reinterpret_cast<const uintx2 *>(a_ptr);
#pragma unroll
        for (int g = 0; g < CG; ++g) {
            uintx4 b[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                b[t] = uintx4{0, 0, 0, 0};
                if (k_valid && col_valid[g]) b[t] = *reinterpret_cast<const uintx4 *>(b_ptr + t * p.ldb + 128 * g);
            }
            mma_group<DT>(a, b, acc[g]);
        }
        a_ptr += 16;
        b_ptr += 16 * p.ldb;
    }

    // accumulator (g, cc) register r of lane (q, c) is Z[4q + r][n0 + 128 g + cc]
    if (WK > 1) {
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int row = 4 * q + r, col4 = (wn * CG + g) * 32 + 2 * c;
                red[(wk * 16 + row) * C4 + col4] = floatx4{acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]};
                red[(wk * 16 + row) * C4 + col4 + 1] = floatx4{acc[g][4][r], acc[g][5][r], acc[g][6][r], acc[g][7][r]};
            }
        __syncthreads();
    }

    float *part = p.split > 1 ? p.partial + ((int64_t)blockIdx.y * p.batch * p.row_blocks + zb) * 16 * p.N : nullptr;
    unsigned short *out = p.C + batch * p.strideC + 16 * rb * p.ldc;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;

    // eight consecutive columns of one row: fp32 partial sums to the workspace, or the finished 16-bit results
    auto finish = [&](int row, int64_t col, floatx4 lo, floatx4 hi) {
        if (row >= rows || col >= p.N) return;
        if (p.split > 1) {
            *reinterpret_cast<floatx4 *>(part + (int64_t)row * p.N + col) = lo;
            *reinterpret_cast<floatx4 *>(part + (int64_t)row * p.N + col + 4) = hi;
            return;
        }
        if (bias && p.bias_row) {
            const float b = bias[16 * rb + row];
            lo += floatx4{b, b, b, b};
            hi += floatx4{b, b, b, b};
        } else if (bias) {
            lo += *reinterpret_cast<const floatx4 *>(bias + col);
            hi += *reinterpret_cast<const floatx4 *>(bias + col + 4);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) { lo[e] = apply_act(lo[e], p.act); hi[e] = apply_act(hi[e], p.act); }
        *reinterpret_cast<uintx4 *>(out + (int64_t)row * p.ldc + col) =
            uintx4{pack2_16<DT>(lo[0], lo[1]), pack2_16<DT>(lo[2], lo[3]), pack2_16<DT>(hi[0], hi[1]), pack2_16<DT>(hi[2], hi[3])};
    };

    if (WK > 1) {
        for (int e = tid; e < 16 * (COLS / 8); e += THREADS) {
            const int row = e / (COLS / 8), col8 = e % (COLS / 8);
            floatx4 lo = red[row * C4 + 2 * col8], hi = red[row * C4 + 2 * col8 + 1];
#pragma unroll
            for (int w = 1; w < WK; ++w) {
                lo += red[(w * 16 + row) * C4 + 2 * col8];
                hi += red[(w * 16 + row) * C4 + 2 * col8 + 1];
            }
            finish(row, nblock0 + 8 * col8, lo, hi);
        }
    } else {
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                finish(4 * q + r, n0 + 128 * g, floatx4{acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]},
                       floatx4{acc[g][4][r], acc[g][5][r], acc[g][6][r], acc[g][7][r]});
    }
}

// The same walk with B brought to LDS by direct loads instead of through registers, as
// skinny_dma_kernel does for fp32 (in bytes the two are alike: a row of a B block is 256 bytes,
// here 128 columns).  A workgroup is WK waves deep in k and 128 CG columns wide; its waves take
// the steps of 16 rows of its k range in turn, and every wave stages only what it consumes
// itself, NS - 1 steps ahead: 1 KiB for A (16 rows x 16 k = 512 bytes, fetched twice so that all
// 64 lanes of the instruction are in use) and CG 4 KiB blocks of B per step; counted waits, no
// barriers.  Lane (q, c) reads A[c][4q .. 4q+3] and B[4q + t][8c .. 8c+7] back and goes on as
// skinny16_kernel does.
template <int DT, int WK, int CG, int NS, bool NT>
__global__ __launch_bounds__(64 * WK) void skinny16_dma_kernel(Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int COLS = 128 * CG, C4 = COLS / 4, THREADS = 64 * WK;
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
    const int64_t n0 = nblock0 + 8 * c;

    const int64_t steps = (p.K + 15) / 16, full_steps = p.K / 16;   // full: all 16 rows below K
    const int64_t g0 = steps * blockIdx.y / p.split, g1 = steps * (blockIdx.y + 1) / p.split;
    const int64_t g1f = g1 < full_steps ? g1 : full_steps;

    const unsigned short *A = p.A + batch * p.strideA + 16 * rb * p.lda;
    const unsigned short *B = p.B + batch * p.strideB;
    // global side (byte offsets).  A's instruction: lane l fetches the 16-byte half l % 2 of row
    // l / 2 % 16 (rows past the end re-read the last one: their sums are never stored).  Instruction
    // i of B's group g: lane l fetches columns 128 g + 8 (l % 16) .. +7 of row 4 i + l / 16 (columns
    // past N re-read the last eight).
    uint32_t a_off, b_off[CG][4];
    {
        const int r = (lane >> 1) & 15;
        const int64_t row = r < rows ? r : rows - 1;
        a_off = (uint32_t)((row * p.lda + 8 * (lane & 1)) * 2);
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int64_t col = nblock0 + 128 * g + 8 * (lane & 15);
                col = col < p.N ? col : p.N - 8;
                b_off[g][i] = (uint32_t)(((4 * i + (lane >> 4)) * p.ldb + (col - nblock0)) * 2);
            }
    }
    const char *a_base = reinterpret_cast<const char *>(A), *b_base = reinterpret_cast<const char *>(B + nblock0);
    const uint32_t wave_lds = (uint32_t)reinterpret_cast<uintptr_t>(lds) + wave * (NS * STAGE);
    auto issue = [&](int64_t step, int slot) {
        const char *ga = ring::scalar_ptr(a_base + step * 32), *gb = ring::scalar_ptr(b_base + step * 32 * p.ldb);
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
    const int rd_a = c * 32 + q * 8;
    const int rd_b = 1024 + 4 * q * 256 + c * 16;

    floatx4 acc[CG][8];
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) acc[g][cc] = floatx4{0, 0, 0, 0};

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
            const uintx2 a = *reinterpret_cast<const __attribute__((address_space(3))) uintx2 *>(st + rd_a);
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                uintx4 b[4];
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    b[t] = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(st + rd_b + g * 4096 + t * 256);
                mma_group<DT>(a, b, acc[g]);
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
            uintx2 a = uintx2{0, 0};
            if (k_valid && a_row_valid) a = *reinterpret_cast<const uintx2 *>(A + (int64_t)c * p.lda + 16 * s + 4 * q);
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                uintx4 b[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    b[t] = uintx4{0, 0, 0, 0};
                    if (k_valid && n0 + 128 * g < p.N)
                        b[t] = *reinterpret_cast<const uintx4 *>(B + (16 * s + 4 * q + t) * p.ldb + n0 + 128 * g);
                }
                mma_group<DT>(a, b, acc[g]);
            }
        }
    }

    // sum the WK waves in wave order (the staging area is free now)
    __syncthreads();
    floatx4 *red = reinterpret_cast<floatx4 *>(lds_raw);
#pragma unroll
    for (int g = 0; g < CG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * q + r, col4 = g * 32 + 2 * c;
            red[(wave * 16 + row) * C4 + col4] = floatx4{acc[g][0][r], acc[g][1][r], acc[g][2][r], acc[g][3][r]};
            red[(wave * 16 + row) * C4 + col4 + 1] = floatx4{acc[g][4][r], acc[g][5][r], acc[g][6][r], acc[g][7][r]};
        }
    __syncthreads();

    float *part = p.split > 1 ? p.partial + ((int64_t)blockIdx.y * p.batch * p.row_blocks + zb) * 16 * p.N : nullptr;
    unsigned short *out = p.C + batch * p.strideC + 16 * rb * p.ldc;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    for (int e = tid; e < 16 * (COLS / 8); e += THREADS) {
        const int row = e / (COLS / 8), col8 = e % (COLS / 8);
        floatx4 lo = red[row * C4 + 2 * col8], hi = red[row * C4 + 2 * col8 + 1];
#pragma unroll
        for (int w = 1; w < WK; ++w) {
            lo += red[(w * 16 + row) * C4 + 2 * col8];
            hi += red[(w * 16 + row) * C4 + 2 * col8 + 1];
        }
        const int64_t col = nblock0 + 8 * col8;
        if (row >= rows || col >= p.N) continue;
        if (p.split > 1) {
            *reinterpret_cast<floatx4 *>(part + (int64_t)row * p.N + col) = lo;
            *reinterpret_cast<floatx4 *>(part + (int64_t)row * p.N + col + 4) = hi;
            continue;
        }
        if (bias && p.bias_row) {
            const float b = bias[16 * rb + row];
            lo += floatx4{b, b, b, b};
            hi += floatx4{b, b, b, b};
        } else if (bias) {
            lo += *reinterpret_cast<const floatx4 *>(bias + col);
            hi += *reinterpret_cast<const floatx4 *>(bias + col + 4);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) { lo[k] = apply_act(lo[k], p.act); hi[k] = apply_act(hi[k], p.act); }
        *reinterpret_cast<uintx4 *>(out + (int64_t)row * p.ldc + col) =
            uintx4{pack2_16<DT>(lo[0], lo[1]), pack2_16<DT>(lo[2], lo[3]), pack2_16<DT>(hi[0], hi[1]), pack2_16<DT>(hi[2], hi[3])};
    }
#endif
}

// C = act(bias + sum over splits of partial), splits added in ascending order, one rounding
template <int DT>
__global__ __launch_bounds__(256) void skinny16_reduce_kernel(Params p)
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
    *reinterpret_cast<uintx2 *>(p.C + batch * p.strideC + row * p.ldc + col) =
        uintx2{pack2_16<DT>(z[0], z[1]), pack2_16<DT>(z[2], z[3])};
}

template <int DT>
bool supports(const Problem &p)
{
    return p.dtype == DT && p.layout == 0 && p.M >= 1 && p.K >= 4 && p.K % 4 == 0 && p.N % 8 == 0 &&
           p.batch * ((p.M + 15) / 16) <= 65535 && vector_friendly(p);
}

template <int DT, int WN, int WK, int CG, bool NT, int SPLIT, bool IL>
hipError_t launch(const Problem &p, hipStream_t stream)
{
    constexpr int COLS = 128 * CG * WN;
    Params sp;
    sp.M = p.M; sp.N = p.N; sp.K = p.K;
    sp.A = static_cast<const unsigned short *>(p.A); sp.lda = p.lda; sp.strideA = p.strideA;
    sp.B = static_cast<const unsigned short *>(p.B); sp.ldb = p.ldb; sp.strideB = p.strideB;
    sp.bias = p.bias; sp.strideBias = p.strideBias; sp.bias_row = p.bias_row ? 1 : 0;
    sp.C = static_cast<unsigned short *>(p.C); sp.ldc = p.ldc; sp.strideC = p.strideC;
    sp.batch = p.batch; sp.act = p.act;
    sp.row_blocks = (p.M + 15) / 16;
    // SPLIT == 0: enough workgroups for one per CU when a workgroup has eight or more waves or
    // interleaves its waves in k, else about two per CU, but never ranges shorter than 256 rows
    int split = SPLIT;
    if (SPLIT == 0) {
        const int64_t col_blocks = (p.N + COLS - 1) / COLS * p.batch * sp.row_blocks;
        const int64_t target = (IL || WN * WK >= 8) ? 256 : 512;
        const int64_t by_grid = target / col_blocks;              // whole rounds: 125 column blocks take 2 parts, not 3
        const int64_t by_k = p.K / (256 * WK) > 0 ? p.K / (256 * WK) : 1;
        split = (int)(by_grid < by_k ? by_grid : by_k);
        if (split < 1) split = 1;
        if (split > 64) split = 64;
        // one workgroup per CU: by the estimate of the time
        if (target == 256)
            split = (int)stream_split(col_blocks, 2.0 * COLS * (double)p.K, by_k, 64.0 * (double)p.N * (double)(p.batch * sp.row_blocks));
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
    hipLaunchKernelGGL((skinny16_kernel<DT, WN, WK, CG, NT, IL>), grid, dim3(64 * WN * WK), 0, stream, sp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t vecs = p.M * (p.N / 4);
    hipLaunchKernelGGL(skinny16_reduce_kernel<DT>, dim3((unsigned)((vecs + 255) / 256), (unsigned)p.batch), dim3(256), 0,
                       stream, sp);
    return hipGetLastError();
}

// 32-bit byte offsets inside a step of 16 rows
template <int DT>
bool dma_supports(const Problem &p)
{
    return supports<DT>(p) && p.ldb < (1ll << 24) && p.lda < (1ll << 24);
}

template <int DT, int WK, int CG, int NS, bool NT>
hipError_t dma_launch(const Problem &p, hipStream_t stream)
{
    constexpr int COLS = 128 * CG, LDS_BYTES = WK * NS * (1024 + CG * 4096);
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&skinny16_dma_kernel<DT, WK, CG, NS, NT>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    Params sp;
    sp.M = p.M; sp.N = p.N; sp.K = p.K;
    sp.A = static_cast<const unsigned short *>(p.A); sp.lda = p.lda; sp.strideA = p.strideA;
    sp.B = static_cast<const unsigned short *>(p.B); sp.ldb = p.ldb; sp.strideB = p.strideB;
    sp.bias = p.bias; sp.strideBias = p.strideBias; sp.bias_row = p.bias_row ? 1 : 0;
    sp.C = static_cast<unsigned short *>(p.C); sp.ldc = p.ldc; sp.strideC = p.strideC;
    sp.batch = p.batch; sp.act = p.act;
    sp.row_blocks = (p.M + 15) / 16;
    // never ranges shorter than 256 rows per wave
    const int64_t col_blocks = (p.N + COLS - 1) / COLS * p.batch * sp.row_blocks;
    const int64_t by_k = p.K / (256 * WK) > 0 ? p.K / (256 * WK) : 1;
    const int64_t split = stream_split(col_blocks, 2.0 * COLS * (double)p.K, by_k, 64.0 * (double)p.N * (double)(p.batch * sp.row_blocks));
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
    hipLaunchKernelGGL((skinny16_dma_kernel<DT, WK, CG, NS, NT>), grid, dim3(64 * WK), LDS_BYTES, stream, sp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t vecs = p.M * (p.N / 4);
    hipLaunchKernelGGL(skinny16_reduce_kernel<DT>, dim3((unsigned)((vecs + 255) / 256), (unsigned)p.batch), dim3(256), 0,
                       stream, sp);
    return hipGetLastError();
}

}  // namespace skinny16
}  // namespace optiml

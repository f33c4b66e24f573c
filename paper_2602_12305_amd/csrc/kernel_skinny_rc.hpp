// Streaming kernels for 16 rows of A at a time when B is column-major (stored [N][K]: every column
// of B, i.e. every output feature, is one contiguous K-vector - the usual layout of weights), for
// all four storage types: fp32, bf16, fp16 and 8-bit E4M3 (bf16 result).
//
// As in kernel_skinny.hpp the bound is HBM: every byte of B is read once and used for 16
// multiply-adds on the matrix pipe.  With k contiguous in B nothing has to be rearranged: a lane's
// 128-bit load IS a run of consecutive k of one column, which is what the 16x16 matrix
// instructions want per lane.  Lane (q = lane/16, c = lane%16) of a wave, per step of 64 T bytes
// of k and per group g of 16 columns, loads
//     B[n0 + 16g + c][kb + 64t + 16q .. +15]   and   A[c][kb + 64t + 16q .. +15]   (bytes), t = 0..T-1
// and feeds each 16-byte pair to the matrix pipe in operand-sized pieces: E4M3 two
// v_mfma_f32_16x16x32_fp8_fp8 (8 bytes = 8 k per lane), bf16 / fp16 two v_mfma_f32_16x16x16 (4 k),
// fp32 four v_mfma_f32_16x16x4_f32 (1 k).  Which k a lane's piece stands for only has to agree
// between the two operands.  Accumulator g register r of lane (q, c) is Z[4q + r][n0 + 16g + c].
//
// Memory walk: a workgroup owns COLS = 16 CG WN consecutive columns = one contiguous block of B,
// and its WK waves take the steps of k in turn, so the workgroup streams its block front
// to back (starting at a per-workgroup offset and wrapping).  With N / COLS >= the number of CUs no split of k over workgroups is needed; smaller N
// splits k over grid.y with fp32 partial sums in the workspace, added in split order by a second
// kernel.  The WK waves' sums are added in wave order through LDS.  No atomics; repeatable.
#pragma once
#include "kernel_tile_ring.hpp"      // the LDS-DMA load, the hand-counted wait, the scalarised pointer

namespace optiml {
namespace skinny_rc {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));

struct Params {
    int64_t M, N, K;
    const char *A; int64_t lda, strideA;       // leading dimensions and strides in elements
    const char *B; int64_t ldb, strideB;
    const float *bias; int64_t strideBias;
    int bias_row;          // bias[m] (the row of C) instead of bias[n]
    char *C; int64_t ldc, strideC;
    float *partial;        // [split][batch * row_blocks][16][N] when split > 1
    int64_t batch, row_blocks;
    int split, act;
};

template <int DT> struct Type {
    static constexpr int ES = DT == DT_F32 ? 4 : is_8bit(DT) ? 1 : 2;     // bytes per element of A and B (E2M1: per pair)
    static constexpr int CS = DT == DT_F32 ? 4 : 2;                       // ... of C
    static constexpr int ODT = is_8bit(DT) ? DT_BF16 : DT;                // storage type of a 16-bit C
};

// the multiply-adds of one 16-byte piece of k: a from A's row c, b from B's column c
template <int DT>
__device__ __forceinline__ floatx4 mma16(uintx4 a, uintx4 b, floatx4 acc)
{
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (DT == DT_F32) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a[i]), __uint_as_float(b[i]), acc, 0, 0, 0);
    } else if constexpr (DT == DT_F4) {
        // 16 bytes = 32 E2M1 values: this lane's quarter of one 128-deep scaled instruction, both scales 2^0
        typedef int intx8_ __attribute__((ext_vector_type(8)));
        const intx8_ a8 = {(int)a[0], (int)a[1], (int)a[2], (int)a[3], 0, 0, 0, 0}, b8 = {(int)b[0], (int)b[1], (int)b[2], (int)b[3], 0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, acc, 4, 4, 0, 0x7f7f7f7f, 0, 0x7f7f7f7f);
    } else if constexpr (DT == DT_F8) {
        typedef long longx2_ __attribute__((ext_vector_type(2)));
        const longx2_ a2 = __builtin_bit_cast(longx2_, a), b2 = __builtin_bit_cast(longx2_, b);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a2[0], b2[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a2[1], b2[1], acc, 0, 0, 0);
    } else if constexpr (DT == DT_BF8) {
        typedef long longx2_ __attribute__((ext_vector_type(2)));
        const longx2_ a2 = __builtin_bit_cast(longx2_, a), b2 = __builtin_bit_cast(longx2_, b);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(a2[0], b2[0], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf8_bf8(a2[1], b2[1], acc, 0, 0, 0);
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const uintx2 ai = uintx2{a[2 * i], a[2 * i + 1]}, bi = uintx2{b[2 * i], b[2 * i + 1]};
            if constexpr (DT == DT_F16)
                acc = __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(halfx4, ai), __builtin_bit_cast(halfx4, bi), acc, 0, 0, 0);
            else
                acc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(shortx4, ai), __builtin_bit_cast(shortx4, bi), acc, 0, 0, 0);
        }
    }
#endif
    return acc;
}

// T = 16-byte vectors per lane, column group and step: a step covers 64 T bytes of k
template <int CG, int T>
struct Stage {
    uintx4 a[T];
    uintx4 b[CG][T];
};

// one whole step (256 bytes of k below the end): a_ptr / b_ptr point at this lane's first vector
template <int CG, int T>
__device__ __forceinline__ void load_stage(Stage<CG, T> &st, const char *a_ptr, const char *const (&b_ptr)[CG], int64_t off,
                                           bool a_valid, const bool (&col_valid)[CG])
{
#pragma unroll
    for (int t = 0; t < T; ++t) {
        st.a[t] = a_valid ? *reinterpret_cast<const uintx4 *>(a_ptr + off + 64 * t) : uintx4{0, 0, 0, 0};
#pragma unroll
        for (int g = 0; g < CG; ++g)
            st.b[g][t] = col_valid[g] ? __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(b_ptr[g] + off + 64 * t))
                                      : uintx4{0, 0, 0, 0};
    }
}

template <int DT, int CG, int T>
__device__ __forceinline__ void mma_stage(const Stage<CG, T> &st, floatx4 (&acc)[CG])
{
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int g = 0; g < CG; ++g) acc[g] = mma16<DT>(st.a[t], st.b[g][t], acc[g]);
}

template <int DT, int WN, int WK, int CG, int T>
__global__ __launch_bounds__(64 * WN * WK) void skinny_rc_kernel(Params p)
{
    constexpr int ES = Type<DT>::ES, CS = Type<DT>::CS;
    constexpr int STEP = 64 * T;                                   // bytes of k per step
    constexpr int COLS = 16 * CG * WN;
    constexpr int THREADS = 64 * WN * WK;
    __shared__ floatx4 red[WK > 1 ? WK * 4 * COLS : 1];          // [wk][row group q][column]: rows 4q..4q+3

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave % WN, wk = wave / WN;
    const int q = lane >> 4, c = lane & 15;
    const int64_t zb = blockIdx.z, batch = zb / p.row_blocks, rb = zb % p.row_blocks;
    const int64_t rows = p.M - 16 * rb < 16 ? p.M - 16 * rb : 16;
    const int64_t nblock0 = (int64_t)blockIdx.x * COLS;
    const int64_t n0 = nblock0 + (int64_t)wn * CG * 16 + c;       // this lane's column in group 0

    // steps of 256 bytes of k: this workgroup's range [g0, g1) of the grid split, its waves in turn
    const int64_t kbytes = p.K * ES, steps = (kbytes + STEP - 1) / STEP, full_steps = kbytes / STEP;
    const int64_t g0 = steps * blockIdx.y / p.split, g1 = steps * (blockIdx.y + 1) / p.split;
    const int64_t g1f = g1 < full_steps ? g1 : full_steps;

    const bool a_valid = c < rows;
    const char *a_ptr = p.A + (batch * p.strideA + (16 * rb + (a_valid ? c : 0)) * p.lda) * ES + 16 * q;
    bool col_valid[CG];
    const char *b_ptr[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) {
        col_valid[g] = n0 + 16 * g < p.N;
        b_ptr[g] = p.B + (batch * p.strideB + (col_valid[g] ? n0 + 16 * g : 0) * p.ldb) * ES + 16 * q;
    }

    floatx4 acc[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[g] = floatx4{0, 0, 0, 0};

    // whole steps, two register stages.  The workgroups do not all start at the front of their
    // columns: workgroup x starts 17 x steps in and wraps around, so that the workgroups in flight
    // sit at different offsets within their columns.  With a power-of-two column pitch a common
    // offset means a common set of memory channels (the transpose kernel's finding).
    const int64_t nfull = g1f - g0;
    if (wk < nfull) {
        const int64_t rot = ((int64_t)blockIdx.x * 17) % nfull;
        auto step_of = [&](int64_t j) { const int64_t u = j + rot; return g0 + (u < nfull ? u : u - nfull); };
        Stage<CG, T> cur, nxt;
        int64_t j = wk;
        load_stage<CG, T>(cur, a_ptr, b_ptr, step_of(j) * STEP, a_valid, col_valid);
        for (j += WK; j < nfull; j += WK) {
            load_stage<CG, T>(nxt, a_ptr, b_ptr, step_of(j) * STEP, a_valid, col_valid);
            mma_stage<DT, CG, T>(cur, acc);
            cur = nxt;
        }
        mma_stage<DT, CG, T>(cur, acc);
    }
    // the ragged last step (K * ES is a multiple of 16: whole vectors), taken by wave 0 of the last split
    if (wk == 0 && g1 > g1f) {
        const int64_t kb = full_steps * STEP;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const bool k_valid = kb + 64 * t + 16 * q + 16 <= kbytes;
            const uintx4 a = (k_valid && a_valid) ? *reinterpret_cast<const uintx4 *>(a_ptr + kb + 64 * t) : uintx4{0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                const uintx4 b = (k_valid && col_valid[g]) ? *reinterpret_cast<const uintx4 *>(b_ptr[g] + kb + 64 * t)
                                                           : uintx4{0, 0, 0, 0};
                acc[g] = mma16<DT>(a, b, acc[g]);
            }
        }
    }

    // sum the WK waves in wave order
    if (WK > 1) {
#pragma unroll
        for (int g = 0; g < CG; ++g) red[(wk * 4 + q) * COLS + (wn * CG + g) * 16 + c] = acc[g];
        __syncthreads();
    }
    float *part = p.split > 1 ? p.partial + ((int64_t)blockIdx.y * p.batch * p.row_blocks + zb) * 16 * p.N : nullptr;
    char *out = p.C + (batch * p.strideC + 16 * rb * p.ldc) * CS;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;

    // four rows (4 qq .. 4 qq + 3) of one column
    auto finish = [&](int qq, int64_t col, floatx4 z) {
        if (col >= p.N) return;
        const float bj = (bias && p.split == 1 && !p.bias_row) ? bias[col] : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * qq + r;
            if (row >= rows) continue;
            if (p.split > 1) { part[(int64_t)row * p.N + col] = z[r]; continue; }
            const float y = apply_act(z[r] + (bias && p.bias_row ? bias[16 * rb + row] : bj), p.act);
            if constexpr (DT == DT_F32) reinterpret_cast<float *>(out)[(int64_t)row * p.ldc + col] = y;
            else reinterpret_cast<unsigned short *>(out)[(int64_t)row * p.ldc + col] = to_16<Type<DT>::ODT>(y);
        }
    };
    if (WK > 1) {
        for (int e = tid; e < 4 * COLS; e += THREADS) {
            const int qq = e / COLS, col = e % COLS;
            floatx4 z = red[qq * COLS + col];
#pragma unroll
            for (int w = 1; w < WK; ++w) z += red[(w * 4 + qq) * COLS + col];
            finish(qq, nblock0 + col, z);
        }
    } else {
#pragma unroll
        for (int g = 0; g < CG; ++g) finish(q, n0 + 16 * g, acc[g]);
    }
}

// ---- the same kernel with B and A staged through LDS by DMA -------------------------------------
// In the kernel above adjacent lanes hold different columns (the matrix instruction fixes
// lane % 16 = column), so every lane's 16 bytes is an address segment of its own.  An LDS-DMA
// load writes lane l's 16 bytes to base + 16 l whatever address the lane reads, so here the global
// side is laid out for the memory system - 16 lanes read the 256 contiguous bytes of one column's
// step, an instruction covers four columns - and the matrix-instruction layout is recovered by
// the LDS read.  A 16-column group of a step is a 16 x 256-byte block in LDS; slot s of column c
// holds the step's chunk s ^ c (the XOR is applied to the global address, still inside the same
// 256 bytes), so lane (q, c)'s read of chunk 4t + q sits at slot (4t + q) ^ c and the 64 lanes of
// a read spread evenly over the banks.  A's 16 rows are one more such block.  Every wave stages
// only what it consumes itself: no barriers, just counted waits (loads complete in issue order).
template <int DT, int WK, int CG, int NS>
__global__ __launch_bounds__(64 * WK) void skinny_rc_dma_kernel(Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int ES = Type<DT>::ES, CS = Type<DT>::CS;
    constexpr int COLS = 16 * CG, THREADS = 64 * WK;
    constexpr int BLOCK = 4096, STAGE = (CG + 1) * BLOCK;           // bytes: one 16 x 256 block; A's block + CG of B
    constexpr int LOADS = (CG + 1) * 4;                             // DMA instructions per stage
    extern __shared__ __attribute__((aligned(1024))) char lds_raw[];
    ring::lds_char *const lds = (ring::lds_char *)lds_raw;
    static_assert(WK * 4 * COLS * 16 <= WK * NS * STAGE, "the reduction buffer reuses the staging area");

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4, c = lane & 15;
    const int64_t zb = blockIdx.z, batch = zb / p.row_blocks, rb = zb % p.row_blocks;
    const int64_t rows = p.M - 16 * rb < 16 ? p.M - 16 * rb : 16;
    const int64_t nblock0 = (int64_t)blockIdx.x * COLS;

    const int64_t kbytes = p.K * ES, steps = (kbytes + 255) / 256, full_steps = kbytes / 256;
    const int64_t g0 = steps * blockIdx.y / p.split, g1 = steps * (blockIdx.y + 1) / p.split;
    const int64_t g1f = g1 < full_steps ? g1 : full_steps;

    // global side of the loads: instruction i of a block covers its rows / columns 4i .. 4i+3, lane l
    // the chunk (l % 16) ^ (4i + l / 16) of row / column 4i + l / 16; rows and columns past the
    // end re-read the last valid one (their results are never stored)
    const char *a_base = p.A + (batch * p.strideA + 16 * rb * p.lda) * ES;
    const char *b_base = p.B + (batch * p.strideB + nblock0 * p.ldb) * ES;
    uint32_t a_off[4], b_off[CG][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = 4 * i + (lane >> 4), chunk = (lane & 15) ^ r;
        const int64_t row = r < rows ? r : rows - 1;
        a_off[i] = (uint32_t)(row * p.lda * ES + chunk * 16);
#pragma unroll
        for (int g = 0; g < CG; ++g) {
            int64_t col = nblock0 + 16 * g + r;
            col = col < p.N ? col : p.N - 1;
            b_off[g][i] = (uint32_t)((col - nblock0) * p.ldb * ES + chunk * 16);
        }
    }
    const uint32_t wave_lds = (uint32_t)reinterpret_cast<uintptr_t>(lds) + wave * (NS * STAGE);
    auto issue = [&](int64_t step, int slot) {
        const char *ga = ring::scalar_ptr(a_base + step * 256), *gb = ring::scalar_ptr(b_base + step * 256);
        const uint32_t d = __builtin_amdgcn_readfirstlane(wave_lds + slot * STAGE);
#pragma unroll
        for (int i = 0; i < 4; ++i) ring::dma_load16(ga, a_off[i], d + i * 1024);
#pragma unroll
        for (int g = 0; g < CG; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) ring::dma_load16_once(gb, b_off[g][i], d + (g + 1) * BLOCK + i * 1024);   // B: read once
    };
    // LDS side: this lane's reads of a block: chunk 4t + q of row / column c
    int rd[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) rd[t] = c * 256 + (((4 * t + q) ^ c) << 4);

    floatx4 acc[CG];
#pragma unroll
    for (int g = 0; g < CG; ++g) acc[g] = floatx4{0, 0, 0, 0};

    // this wave's whole steps: local indices wave, wave + WK, ... of the rotated range (see above)
    const int64_t nfull = g1f - g0;
    const int64_t mine = nfull > wave ? (nfull - wave + WK - 1) / WK : 0;
    const int64_t rot = nfull > 0 ? ((int64_t)blockIdx.x * 17) % nfull : 0;
    auto step_of = [&](int64_t i) { const int64_t u = wave + i * WK + rot; return g0 + (u < nfull ? u : u - nfull); };
    // prologue: NS - 1 stages in flight (past the end the last step is fetched again, never used,
    // so that the wait counts stay uniform)
    if (mine > 0) {
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
            for (int t = 0; t < 4; ++t) {
                const uintx4 a = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(st + rd[t]);
#pragma unroll
                for (int g = 0; g < CG; ++g) {
                    const uintx4 b = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(st + (g + 1) * BLOCK + rd[t]);
                    acc[g] = mma16<DT>(a, b, acc[g]);
                }
            }
            asm volatile("" ::: "memory");                          // the reads are done before the slot is refilled
        }
        ring::wait_vmcnt<0>();
    }
    // rows past the block's end were fed the last valid row: harmless, they are not stored
    const bool a_valid = c < rows;
    // the ragged last step, straight from memory, by wave 0 of the last split
    if (wave == 0 && g1 > g1f) {
        const int64_t kb = full_steps * 256;
        const char *a_ptr = a_base + (a_valid ? c : 0) * p.lda * ES + 16 * q;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const bool k_valid = kb + 64 * t + 16 * q + 16 <= kbytes;
            const uintx4 a = (k_valid && a_valid) ? *reinterpret_cast<const uintx4 *>(a_ptr + kb + 64 * t) : uintx4{0, 0, 0, 0};
#pragma unroll
            for (int g = 0; g < CG; ++g) {
                int64_t col = nblock0 + 16 * g + c;
                const bool cv = col < p.N;
                col = cv ? col : p.N - 1;
                const uintx4 b = (k_valid && cv) ? *reinterpret_cast<const uintx4 *>(b_base + (col - nblock0) * p.ldb * ES + 16 * q + kb + 64 * t)
                                                 : uintx4{0, 0, 0, 0};
                acc[g] = mma16<DT>(a, b, acc[g]);
            }
        }
    }

    // sum the WK waves in wave order (the staging area is free now)
    __syncthreads();
    floatx4 *red = reinterpret_cast<floatx4 *>(lds_raw);
    if (WK > 1) {
#pragma unroll
        for (int g = 0; g < CG; ++g) red[(wave * 4 + q) * COLS + g * 16 + c] = acc[g];
        __syncthreads();
    }
    float *part = p.split > 1 ? p.partial + ((int64_t)blockIdx.y * p.batch * p.row_blocks + zb) * 16 * p.N : nullptr;
    char *out = p.C + (batch * p.strideC + 16 * rb * p.ldc) * CS;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    auto finish = [&](int qq, int64_t col, floatx4 z) {
        if (col >= p.N) return;
        const float bj = (bias && p.split == 1 && !p.bias_row) ? bias[col] : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int row = 4 * qq + r;
            if (row >= rows) continue;
            if (p.split > 1) { part[(int64_t)row * p.N + col] = z[r]; continue; }
            const float y = apply_act(z[r] + (bias && p.bias_row ? bias[16 * rb + row] : bj), p.act);
            if constexpr (DT == DT_F32) reinterpret_cast<float *>(out)[(int64_t)row * p.ldc + col] = y;
            else reinterpret_cast<unsigned short *>(out)[(int64_t)row * p.ldc + col] = to_16<Type<DT>::ODT>(y);
        }
    };
    if (WK > 1) {
        for (int e = tid; e < 4 * COLS; e += THREADS) {
            const int qq = e / COLS, col = e % COLS;
            floatx4 z = red[qq * COLS + col];
#pragma unroll
            for (int w = 1; w < WK; ++w) z += red[(w * 4 + qq) * COLS + col];
            finish(qq, nblock0 + col, z);
        }
    } else {
#pragma unroll
        for (int g = 0; g < CG; ++g) finish(q, nblock0 + 16 * g + c, acc[g]);
    }
#endif
}

// C = act(bias + sum over splits of partial), splits added in ascending order, one rounding
template <int DT>
__global__ __launch_bounds__(256) void skinny_rc_reduce_kernel(Params p)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t batch = blockIdx.y;
    if (idx >= p.M * p.N) return;
    const int64_t row = idx / p.N, col = idx % p.N;
    const int64_t zb = batch * p.row_blocks + row / 16;
    float z = 0.0f;
    for (int s = 0; s < p.split; ++s) z += p.partial[(((int64_t)s * p.batch * p.row_blocks + zb) * 16 + row % 16) * p.N + col];
    const float y = apply_act(z + (p.bias ? p.bias[batch * p.strideBias + (p.bias_row ? row : col)] : 0.0f), p.act);
    char *out = p.C + (batch * p.strideC + row * p.ldc + col) * Type<DT>::CS;
    if constexpr (DT == DT_F32) *reinterpret_cast<float *>(out) = y;
    else *reinterpret_cast<unsigned short *>(out) = to_16<Type<DT>::ODT>(y);
}

template <int DT>
bool supports(const Problem &p)
{
    // A row-major, B column-major; whole 16-byte vectors of k; 32-bit friendly sizes
    return p.dtype == DT && p.layout == 1 && p.M >= 1 && p.K >= 1 && (p.K * Type<DT>::ES) % 16 == 0 &&
           p.batch * ((p.M + 15) / 16) <= 65535 && vector_friendly(p);
}

template <int DT, int WN, int WK, int CG, int T>
hipError_t launch(const Problem &p, hipStream_t stream)
{
    constexpr int COLS = 16 * CG * WN;
    Params sp;
    sp.M = p.M; sp.N = p.N; sp.K = p.K;
    sp.A = static_cast<const char *>(p.A); sp.lda = p.lda; sp.strideA = p.strideA;
    sp.B = static_cast<const char *>(p.B); sp.ldb = p.ldb; sp.strideB = p.strideB;
    sp.bias = p.bias; sp.strideBias = p.strideBias; sp.bias_row = p.bias_row ? 1 : 0;
    sp.C = static_cast<char *>(p.C); sp.ldc = p.ldc; sp.strideC = p.strideC;
    sp.batch = p.batch; sp.act = p.act;
    sp.row_blocks = (p.M + 15) / 16;
    // split k over the grid only as far as needed for one workgroup per CU, and never into ranges
    // shorter than WK * 8 steps (2 KiB of k per wave)
    const int64_t col_blocks = (p.N + COLS - 1) / COLS * p.batch * sp.row_blocks;
    const int64_t steps = (p.K * Type<DT>::ES + 64 * T - 1) / (64 * T);
    int64_t split = compute_units() / col_blocks;                 // whole rounds
    const int64_t by_k = steps * T / (WK * 32) > 0 ? steps * T / (WK * 32) : 1;
    if (split > by_k) split = by_k;
    if (split < 1) split = 1;
    if (split > 64) split = 64;
    sp.split = (int)split;
    sp.partial = nullptr;
    if (split > 1) {
        void *ws = nullptr;
        hipError_t e = workspace(sizeof(float) * (size_t)split * p.batch * sp.row_blocks * 16 * p.N, &ws, stream);
        if (e != hipSuccess) return e;
        sp.partial = static_cast<float *>(ws);
    }
    const int64_t gx = (p.N + COLS - 1) / COLS;
    if (gx > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)gx, (unsigned)split, (unsigned)(p.batch * sp.row_blocks));
    hipLaunchKernelGGL((skinny_rc_kernel<DT, WN, WK, CG, T>), grid, dim3(64 * WN * WK), 0, stream, sp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t elems = p.M * p.N;
    hipLaunchKernelGGL(skinny_rc_reduce_kernel<DT>, dim3((unsigned)((elems + 255) / 256), (unsigned)p.batch), dim3(256), 0, stream, sp);
    return hipGetLastError();
}

template <int DT>
bool supports_dma(const Problem &p)
{
    // lane offsets are 32-bit: the 16 rows of A and the workgroup's columns of B must span less than 4 GiB
    return supports<DT>(p) && 16 * p.lda * Type<DT>::ES < (int64_t(1) << 31) && 64 * p.ldb * Type<DT>::ES < (int64_t(1) << 31);
}

template <int DT, int WK, int CG, int NS>
hipError_t launch_dma(const Problem &p, hipStream_t stream)
{
    constexpr int COLS = 16 * CG, LDS_BYTES = WK * NS * (CG + 1) * 4096;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(&skinny_rc_dma_kernel<DT, WK, CG, NS>),
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (attr != hipSuccess) return attr;
    Params sp;
    sp.M = p.M; sp.N = p.N; sp.K = p.K;
    sp.A = static_cast<const char *>(p.A); sp.lda = p.lda; sp.strideA = p.strideA;
    sp.B = static_cast<const char *>(p.B); sp.ldb = p.ldb; sp.strideB = p.strideB;
    sp.bias = p.bias; sp.strideBias = p.strideBias; sp.bias_row = p.bias_row ? 1 : 0;
    sp.C = static_cast<char *>(p.C); sp.ldc = p.ldc; sp.strideC = p.strideC;
    sp.batch = p.batch; sp.act = p.act;
    sp.row_blocks = (p.M + 15) / 16;
    const int64_t col_blocks = (p.N + COLS - 1) / COLS * p.batch * sp.row_blocks;
    const int64_t steps = (p.K * Type<DT>::ES + 255) / 256;
    int64_t split = compute_units() / col_blocks;                 // whole rounds
    const int64_t by_k = steps / (WK * 8) > 0 ? steps / (WK * 8) : 1;
    if (split > by_k) split = by_k;
    if (split < 1) split = 1;
    if (split > 64) split = 64;
    sp.split = (int)split;
    sp.partial = nullptr;
    if (split > 1) {
        void *ws = nullptr;
        hipError_t e = workspace(sizeof(float) * (size_t)split * p.batch * sp.row_blocks * 16 * p.N, &ws, stream);
        if (e != hipSuccess) return e;
        sp.partial = static_cast<float *>(ws);
    }
    const int64_t gx = (p.N + COLS - 1) / COLS;
    if (gx > 0x7fffffffLL) return hipErrorInvalidValue;
    dim3 grid((unsigned)gx, (unsigned)split, (unsigned)(p.batch * sp.row_blocks));
    hipLaunchKernelGGL((skinny_rc_dma_kernel<DT, WK, CG, NS>), grid, dim3(64 * WK), LDS_BYTES, stream, sp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || split == 1) return e;
    const int64_t elems = p.M * p.N;
    hipLaunchKernelGGL(skinny_rc_reduce_kernel<DT>, dim3((unsigned)((elems + 255) / 256), (unsigned)p.batch), dim3(256), 0, stream, sp);
    return hipGetLastError();
}

}  // namespace skinny_rc
}  // namespace optiml

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

}  // namespace skinny16
}  // namespace optiml

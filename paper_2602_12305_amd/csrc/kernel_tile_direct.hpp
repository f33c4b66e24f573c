// bf16 MFMA tile kernel with direct global->LDS loads (no register staging), for A
// row-major and B row- or column-major, K a multiple of 64.
//
// What gfx950 offers beyond the staged kernel of kernel_tile.hpp:
//   * global_load_lds_dwordx4: a wave copies 64 x 16 bytes from arbitrary per-lane global
//     addresses into one contiguous KiB of LDS (lane l lands at base + 16 l, measured).
//     The tile never passes through VGPRs, nobody issues ds_write, and the swizzle is applied
//     by choosing WHICH global chunk a lane fetches for its fixed LDS slot.
//   * ds_read_b64_tr_b16: a 16-lane group reads a 4(k) x 16(n) block of 16-bit elements
//     stored n-contiguous and receives it transposed - lane i gets column i, four
//     consecutive k (measured: source lane j supplies row j/4, columns 4(j%4)..+3).  Two of
//     them build the 8-element MFMA operand of a row-major B without any transposition pass.
//
// LDS formats.  A (k contiguous) and column-major B: ROWS x 128 bytes, chunk c of row r at
// r*128 + ((c ^ ((r >> 1) & 7)) << 4), read with ds_read_b128 (same format as kernel_tile.hpp).
// Row-major B: 64 k-rows of BN elements (BN*2 bytes), 16-byte chunk c of row k at
// k*BN*2 + ((c ^ (2 (k & 3))) << 4): the four rows a transpose read touches fall in four
// different 32-byte bank groups of the 64-bank LDS.
//
// Pipeline: two LDS stages; the loads of k-tile t+1 are issued before the MFMAs of tile t
// and waited for (vmcnt) just before the one barrier per k-tile.  With 8 waves per
// workgroup two waves share a SIMD, so one wave's MFMAs cover the other's LDS latency.
#pragma once
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace direct {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) char lds_char;

struct Params {
    int64_t M, N, K, batch;
    const char *A; int64_t lda, strideA;
    const char *B; int64_t ldb, strideB;
    const float *bias; int64_t strideBias;
    char *C; int64_t ldc, strideC;
    int64_t tiles_m, tiles_n;
    int act;
};

template <int BM_, int BN_, int WM_, int WN_, bool B_KC_, int DT_ = DT_BF16>
struct Cfg {
    static constexpr int DT = DT_;       // DT_BF16 or DT_F16: another matrix instruction and rounding, nothing else
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_, BK = 64;
    static constexpr bool B_KC = B_KC_;
    static constexpr int NW = WM * WN, THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN;
    static constexpr int TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES, LDS_BYTES = 2 * STAGE_BYTES;
    static constexpr int A_INSTR = A_BYTES / 1024 / NW;      // wave-wide 1 KiB loads per wave per k-tile
    static constexpr int B_INSTR = B_BYTES / 1024 / NW;
    static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile must divide over waves");
    static_assert(BN >= 64, "row-major B swizzle needs at least 8 chunks per row");
};

__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }   // vmcnt(0)

// A wave-uniform pointer pinned into scalar registers, so that the loads below take the
// "scalar base + 32-bit lane offset" address form instead of a 64-bit address per lane.
__device__ __forceinline__ const char *scalar_ptr(const char *q)
{
    const uint64_t v = reinterpret_cast<uint64_t>(q);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}


// The helpers below take LDS-address-space pointers, which only the device pass understands;
// the host pass needs nothing but the kernel's symbol.
#if defined(__HIP_DEVICE_COMPILE__)
template <class C>
struct StepCtx {
    uint32_t a_off[C::A_INSTR], b_off[C::B_INSTR];
    int a_frag[4], tr_cb[C::TN];
    int wave, a_wave, b_wave_kc, tr_row;
};

// Wave-wide 1 KiB loads of one k-tile of A and B into the LDS stage at `dst`.
template <class C>
__device__ __forceinline__ void issue_tile(const StepCtx<C> &c, const char *__restrict__ ga, const char *__restrict__ gb,
                                           lds_char *__restrict__ dst)
{
    ga = scalar_ptr(ga);
    gb = scalar_ptr(gb);
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i)
        __builtin_amdgcn_global_load_lds(ga + c.a_off[i], dst + (c.wave + i * C::NW) * 1024, 16, 0, 0);
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i)
        __builtin_amdgcn_global_load_lds(gb + c.b_off[i], dst + C::A_BYTES + (c.wave + i * C::NW) * 1024, 16, 0, 0);
}

template <class C>
__device__ __forceinline__ void multiply_tile(const StepCtx<C> &c, const lds_char *__restrict__ rd,
                                              floatx16 (&acc)[C::TN][C::TM]);

// One k-tile: start the loads of the next tile into `dma`, multiply the tile held in
// `rd`, then wait for the loads and meet the other waves.  `dma` and `rd` are the two LDS
// stages; restrict tells the compiler that the in-flight DMA cannot touch what is being read,
// so it does not wait for the DMA before the fragment loads.
template <class C>
__device__ __forceinline__ void tile_step(const StepCtx<C> &c, const char *__restrict__ ga, const char *__restrict__ gb,
                                          lds_char *__restrict__ dma, const lds_char *__restrict__ rd,
                                          floatx16 (&acc)[C::TN][C::TM])
{
    issue_tile<C>(c, ga, gb, dma);
    __builtin_amdgcn_sched_barrier(0);      // the loads must be in flight while the tile is multiplied
    multiply_tile<C>(c, rd, acc);
    wait_vmem();
    __syncthreads();
}

// acc += the k-tile (64 values of k) held in stage `rd`
template <class C>
__device__ __forceinline__ void multiply_tile(const StepCtx<C> &c, const lds_char *__restrict__ rd,
                                              floatx16 (&acc)[C::TN][C::TM])
{
    constexpr int TM = C::TM, TN = C::TN;
    const lds_char *sa = rd + c.a_wave;
    const lds_char *sb = rd + C::A_BYTES;
    uintx4 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int s, int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[buf][i] = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(sa + i * 32 * 128 + c.a_frag[s]);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (C::B_KC) {
                fb[buf][j] = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(
                    sb + c.b_wave_kc + j * 32 * 128 + c.a_frag[s]);
            } else {
                const lds_char *q0 = sb + (16 * s + c.tr_row) * (C::BN * 2) + c.tr_cb[j];
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4 *)(q0));
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) shortx4 *)(q0 + 4 * (C::BN * 2)));
                const uintx2 l2 = __builtin_bit_cast(uintx2, lo), h2 = __builtin_bit_cast(uintx2, hi);
                fb[buf][j] = uintx4{l2[0], l2[1], h2[0], h2[1]};
            }
        }
    };

    load_frags(0, 0);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        if (s < 3) load_frags(s + 1, (s + 1) & 1);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int i = 0; i < TM; ++i)
                acc[j][i] = mfma_32x32x16<C::DT>(fb[s & 1][j], fa[s & 1][i], acc[j][i]);
    }
}
#endif

template <class C>
__global__ __launch_bounds__(C::THREADS) void gemm_direct_kernel(Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    constexpr int TM = C::TM, TN = C::TN, NW = C::NW;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % C::WM, wn = wave / C::WM;

    // workgroup -> tile: undo the round-robin over 8 XCDs, then bands of 8 tile rows
    int64_t tile_id;
    {
        const int64_t total = p.tiles_m * p.tiles_n * p.batch;
        const int64_t bid = blockIdx.x, x = bid & 7, loc = bid >> 3;
        const int64_t q8 = total >> 3, r8 = total & 7;
        tile_id = x * q8 + (x < r8 ? x : r8) + loc;
    }
    const int64_t per_batch = p.tiles_m * p.tiles_n;
    const int64_t batch = tile_id / per_batch;
    int64_t t = tile_id % per_batch;
    constexpr int BAND = 8;
    const int64_t band = t / (BAND * p.tiles_n), first = band * BAND;
    const int64_t rows_in_band = p.tiles_m - first < BAND ? p.tiles_m - first : BAND;
    t -= band * BAND * p.tiles_n;
    const int64_t tile_m = first + t % rows_in_band, tile_n = t / rows_in_band;
    const int64_t m0 = tile_m * C::BM, n0 = tile_n * C::BN;

    const char *A = p.A + batch * p.strideA * 2;
    const char *B = p.B + batch * p.strideB * 2;

    // ---- per-lane source offsets (bytes from A / B at k = 0), one per wave-wide load ----
    // A and column-major B: load q covers LDS rows 8q..8q+7; lane l fills row 8q + l/8, slot l%8
    uint32_t a_off[C::A_INSTR], b_off[C::B_INSTR];
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i) {
        const int q = wave + i * NW, r = 8 * q + (lane >> 3);
        const int c = (lane & 7) ^ ((r >> 1) & 7);
        int64_t row = m0 + r;
        row = row < p.M ? row : p.M - 1;
        a_off[i] = (uint32_t)(row * p.lda * 2 + c * 16);
    }
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i) {
        const int q = wave + i * NW;
        if constexpr (C::B_KC) {
            const int r = 8 * q + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            int64_t row = n0 + r;
            row = row < p.N ? row : p.N - 1;
            b_off[i] = (uint32_t)(row * p.ldb * 2 + c * 16);
        } else {
            constexpr int CR = C::BN / 8;                 // chunks per k-row
            const int pidx = q * 64 + lane, k = pidx / CR;
            const int c = (pidx % CR) ^ (2 * (k & 3));
            int64_t col = n0 + c * 8;
            col = col + 8 <= p.N ? col : p.N - 8;          // N % 8 == 0, N >= 8
            b_off[i] = (uint32_t)((k * p.ldb + col) * 2);
        }
    }
    const int64_t b_step = C::B_KC ? 128 : 64 * p.ldb * 2;   // bytes per k-tile

    floatx16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.0f;

    // ---- per-lane fragment addresses ----
    const int frag_row = lane & 31, half = lane >> 5;
    int a_frag[4];                                           // k-step s: row frag_row, chunk (2s+half)^key
#pragma unroll
    for (int s = 0; s < 4; ++s) a_frag[s] = frag_row * 128 + (((2 * s + half) ^ ((frag_row >> 1) & 7)) << 4);
    const int a_wave = wm * C::WTM * 128;
    const int b_wave_kc = wn * C::WTN * 128;
    // row-major B through transpose reads: lane (g = lane/16, jj = lane%16) supplies row
    // 16s + 8(g/2) + 4h + jj/4, columns wn*WTN + 32j + 16(g%2) + 4(jj%4) .. +3
    const int g = lane >> 4, jj = lane & 15;
    const int tr_row = 8 * (g >> 1) + (jj >> 2);             // + 16 s + 4 h
    const int tr_col = wn * C::WTN + 16 * (g & 1) + 4 * (jj & 3);   // + 32 j
    const int tr_key = 2 * (jj >> 2);                        // 2 * (row & 3)
    int tr_cb[TN];                                           // byte offset inside a k-row
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = tr_col + 32 * j;
        tr_cb[j] = (((col >> 3) ^ tr_key) << 4) + ((col & 7) << 1);
    }

    const int64_t nk = p.K / 64;
    StepCtx<C> ctx;
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i) ctx.a_off[i] = a_off[i];
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i) ctx.b_off[i] = b_off[i];
#pragma unroll
    for (int s = 0; s < 4; ++s) ctx.a_frag[s] = a_frag[s];
#pragma unroll
    for (int j = 0; j < TN; ++j) ctx.tr_cb[j] = tr_cb[j];
    ctx.wave = wave; ctx.a_wave = a_wave; ctx.b_wave_kc = b_wave_kc; ctx.tr_row = tr_row;

    lds_char *stage0 = (lds_char *)lds, *stage1 = (lds_char *)lds + C::STAGE_BYTES;
    issue_tile<C>(ctx, A, B, stage0);
    wait_vmem();
    __syncthreads();
    // Two k-tiles per trip, so that each call sees its read stage and its DMA stage as distinct
    // restrict-qualified pointers.  The step that multiplies the last tile has nothing left to
    // prefetch; it re-fetches that same tile into the idle stage (in bounds, never read), which
    // keeps the loop body free of branches.
    const int64_t last = nk - 1;
    int64_t kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        const int64_t n2 = kt + 2 < nk ? kt + 2 : last;
        tile_step<C>(ctx, A + (kt + 1) * 128, B + (kt + 1) * b_step, stage1, stage0, acc);
        tile_step<C>(ctx, A + n2 * 128, B + n2 * b_step, stage0, stage1, acc);
    }
    if (kt < nk) tile_step<C>(ctx, A + last * 128, B + last * b_step, stage1, stage0, acc);

    // A K that ends inside a k-tile: the partial last k-tile goes through stage 0 by ordinary loads,
    // 16-byte chunks at or beyond K written as zeros (K is a whole number of chunks), in the places
    // the DMA loads of a full tile would have filled.  Every step above ended with a barrier, so
    // both stages are free.
    if (p.K % 64 != 0) {
        const int64_t k0 = nk * 64;
#pragma unroll
        for (int i = 0; i < C::A_INSTR; ++i) {
            const int q = wave + i * NW, r = 8 * q + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            uintx4 v = uintx4{0, 0, 0, 0};
            if (k0 + c * 8 < p.K) v = *reinterpret_cast<const uintx4 *>(A + a_off[i] + k0 * 2);
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(stage0 + q * 1024 + lane * 16) = v;
        }
#pragma unroll
        for (int i = 0; i < C::B_INSTR; ++i) {
            const int q = wave + i * NW;
            uintx4 v = uintx4{0, 0, 0, 0};
            if constexpr (C::B_KC) {
                const int r = 8 * q + (lane >> 3);
                const int c = (lane & 7) ^ ((r >> 1) & 7);
                if (k0 + c * 8 < p.K) v = *reinterpret_cast<const uintx4 *>(B + b_off[i] + k0 * 2);
            } else {
                constexpr int CR = C::BN / 8;
                const int k = (q * 64 + lane) / CR;
                if (k0 + k < p.K) v = *reinterpret_cast<const uintx4 *>(B + b_off[i] + k0 * p.ldb * 2);
            }
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(stage0 + C::A_BYTES + q * 1024 + lane * 16) = v;
        }
        __syncthreads();
        multiply_tile<C>(ctx, stage0, acc);
        __syncthreads();                     // the epilogue's slabs reuse the stages
    }

    // Epilogue.  Register r of acc[j][i] is Z[m][n] with m = mw + 32 i + lane%32 and
    // n = nw + 32 j + 8 (r/4) + 4 (lane/32) + r%4: a lane owns short runs of one row, which
    // would make 8-byte stores scattered over 32 rows.  Each wave therefore passes its tile
    // through a private LDS slab, 32 rows at a time (bias, activation and the rounding to bf16
    // happen in registers first), and reads it back with 16 bytes per lane along the rows, so
    // that every global store instruction writes whole 128-byte lines.  The slab rows are
    // padded by 16 bytes to spread the 32 row-strided writes over the banks.  All waves have
    // passed the k loop's last barrier, so the operand stages are free to reuse.
    const int64_t mw = m0 + wm * C::WTM, nw = n0 + wn * C::WTN;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    char *Cb = p.C + batch * p.strideC * 2;
    constexpr int PITCH = C::WTN * 2 + 16;                       // bytes per slab row
    constexpr int CPR = C::WTN / 8;                              // 16-byte chunks per row
    constexpr int READS = 32 * CPR / 64;                         // wave-wide 1 KiB reads per slab
    lds_char *slab = (lds_char *)lds + wave * (32 * PITCH);
    float bj[TN][4][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int64_t n = nw + 32 * j + 8 * gq + 4 * half;
            if (bias && n + 3 < p.N) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(bias + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) bj[j][gq][e] = v[e];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) bj[j][gq][e] = (bias && n + e < p.N) ? bias[n + e] : 0.0f;
            }
        }
    dispatch_act(p.act, [&](auto act_tag) {
    constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = apply_act_bf16out(acc[j][i][4 * gq + e] + bj[j][gq][e], ACT);
                *reinterpret_cast<__attribute__((address_space(3))) uintx2 *>(
                    slab + frag_row * PITCH + (32 * j + 8 * gq + 4 * half) * 2) =
                    uintx2{pack2_16<C::DT>(y[0], y[1]), pack2_16<C::DT>(y[2], y[3])};
            }
#pragma unroll
        for (int q = 0; q < READS; ++q) {
            const int id = q * 64 + lane, row = id / CPR, chunk = id % CPR;
            const uintx4 v = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(slab + row * PITCH + chunk * 16);
            const int64_t m = mw + 32 * i + row, n = nw + chunk * 8;
            if (m < p.M && n < p.N) {
                char *dst = Cb + (m * p.ldc + n) * 2;
                if (n + 8 <= p.N) {
                    *reinterpret_cast<uintx4 *>(dst) = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < p.N)
                            reinterpret_cast<unsigned short *>(dst)[e] = (unsigned short)(v[e >> 1] >> ((e & 1) * 16));
                }
            }
        }
    }
    });
#endif
}

template <class C>
bool supports(const Problem &p)
{
    if (p.dtype != C::DT || p.a_col() || p.b_col() != C::B_KC) return false;
    if (p.K < 64 || p.K % 8 != 0 || !vector_friendly(p)) return false;
    if (!C::B_KC && (p.N % 8 != 0)) return false;
    // per-lane source offsets are 32-bit
    const int64_t a_span = p.M * p.lda * 2, b_span = (C::B_KC ? p.N : 64) * p.ldb * 2 + p.N * 2;
    if (a_span >= (int64_t(1) << 31) || b_span >= (int64_t(1) << 31)) return false;
    const int64_t tiles = ((p.M + C::BM - 1) / C::BM) * ((p.N + C::BN - 1) / C::BN);
    if (tiles <= 0 || p.batch > 0x7fffffffLL / tiles) return false;
    return true;
}

template <class C>
hipError_t launch(const Problem &p, hipStream_t stream)
{
    static bool configured[64] = {};
    auto kernel = gemm_direct_kernel<C>;
    if (C::LDS_BYTES > 64 * 1024) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64 && !configured[dev]) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
            if (e != hipSuccess) return e;
            configured[dev] = true;
        }
    }
    Params q;
    q.M = p.M; q.N = p.N; q.K = p.K; q.batch = p.batch;
    q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = p.strideA;
    q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = p.strideB;
    q.bias = p.bias; q.strideBias = p.strideBias;
    q.C = static_cast<char *>(p.C); q.ldc = p.ldc; q.strideC = p.strideC;
    q.tiles_m = (p.M + C::BM - 1) / C::BM;
    q.tiles_n = (p.N + C::BN - 1) / C::BN;
    q.act = p.act;
    const int64_t total = q.tiles_m * q.tiles_n * p.batch;
    hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(C::THREADS), C::LDS_BYTES, stream, q);
    return hipGetLastError();
}

}  // namespace direct
}  // namespace optiml

// fp32 MFMA tile kernel with a ring of LDS stages fed by direct global->LDS loads, for A
// row-major and B row- or column-major, K a multiple of 16.
//
// The fp32 matrix rate of a CU is 256 flop per clock, one sixteenth of the bf16 rate, so one
// 16-deep k-tile of a BM x 128 block keeps the matrix pipe busy for thousands of cycles while it
// needs only 16 - 24 KiB from L2: the memory side is never the limit.  What costs time in the
// staged kernel of kernel_tile.hpp is everything a wave does between MFMAs when it is alone on
// its SIMD (LDS stores of the next tile, the barrier, the first fragment reads, the additions
// of blocked summation).  Here the loads bypass the registers (no LDS stores), eight waves
// share the four SIMDs so that one wave's MFMAs cover the other's gaps, and the wave tile is
// 128 x 32 or 64 x 32 so that two accumulator sets fit the 256 registers a lane then has.
//
// Ring, wait counts, barrier and the assembly-issued loads are those of kernel_tile_ring.hpp
// (whose helpers are used); the order per k-tile t is: wait until tile t has landed, barrier,
// start the loads of tile t+NS-1 into the stage of tile t-1, read fragments, multiply.
//
// LDS formats.  A and column-major B: ROWS x 64 bytes (16 k), chunk c of row r at
// r*64 + ((c ^ ((r >> 2) & 3)) << 4); a lane reads chunk 2s + lane/32 of row lane%32, whose four
// floats are the operands of four 32x32x2 MFMAs: MFMA (s, t) multiplies k = 8s + t (lanes
// 0-31) and k = 8s + 4 + t (lanes 32-63).  Row-major B: 16 k-rows x 512 bytes, chunk c of row
// k at k*512 + ((c ^ 8((k >> 2) & 1)) << 4); MFMA (s, t) reads one float per lane from row
// 8s + t (lanes 0-31) or 8s + 4 + t (lanes 32-63), and the key puts the two half-waves into
// different halves of the 64 banks.
//
// Summation.  Every FLUSH_ROUNDS ring rounds (128 k) the block sums are added to the running
// sums on the vector ALU and cleared, which keeps the rounding error of a long k loop near
// sqrt(128 K) * 2^-24 of the terms' size instead of K * 2^-24.
#pragma once
#include "kernel_tile_ring.hpp"

namespace optiml {
namespace ringf {

using ring::floatx16;
using ring::floatx4;
using ring::lds_char;
using ring::Params;
using ring::uintx4;

template <int BM_, int NS_, bool B_KC_, int EPI_ = 0>
struct Cfg {
    // 0: C = act(A.B + bias).  1: C is not written; each wave reduces its 32 columns of A.B + bias
    // to a (maximum, sum of exponentials) pair per row and hands out the label's logit (see the
    // same switch of the 16-bit ring kernel).
    static constexpr int EPI = EPI_;
    static constexpr int NS = NS_;
    static constexpr bool B_KC = B_KC_;
    static constexpr int BM = BM_, BN = 128, BK = 16, WM = 2, WN = 4, NW = WM * WN, THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * 64, B_BYTES = BN * 64, STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int A_INSTR = A_BYTES / 1024 / NW, B_INSTR = B_BYTES / 1024 / NW;
    static constexpr int LOADS = A_INSTR + B_INSTR;            // per wave per stage
    static constexpr int FLUSH_ROUNDS = 8 / NS_ > 0 ? 8 / NS_ : 1;   // ring rounds per summation block
    static constexpr int SLAB_BYTES = NW * 32 * WTN * 4;       // epilogue staging, one 32-row slab per wave
    static constexpr int LDS_BYTES = NS * STAGE_BYTES > SLAB_BYTES ? NS * STAGE_BYTES : SLAB_BYTES;
    static_assert(NS >= 3 && NS <= 6, "ring depth");
    static_assert(TN == 1 && (BM == 256 || BM == 128), "wave tile is (BM/2) x 32");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

#if defined(__HIP_DEVICE_COMPILE__)

template <class C>
struct Ctx {
    uint32_t a_off[C::A_INSTR], b_off[C::B_INSTR];
    int a_frag[2];
    int wave, a_wave, b_base;
};

template <class C>
__device__ __forceinline__ void issue_stage(const Ctx<C> &c, const char *ga, const char *gb, lds_char *dst)
{
    ga = ring::scalar_ptr(ga);
    gb = ring::scalar_ptr(gb);
    const uint32_t d = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(dst) + c.wave * 1024);
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i) ring::dma_load16(ga, c.a_off[i], d + i * C::NW * 1024);
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i) ring::dma_load16(gb, c.b_off[i], d + C::A_BYTES + i * C::NW * 1024);
}

// One k-tile of 16 held in stage `rd`, added into the block sums.
template <class C>
__device__ __forceinline__ void multiply_stage(const Ctx<C> &c, const lds_char *rd, floatx16 (&part)[C::TM]);

template <class C>
__device__ __forceinline__ void ring_step(const Ctx<C> &c, const char *ga, const char *gb, lds_char *dma,
                                          const lds_char *rd, floatx16 (&part)[C::TM])
{
    ring::wait_vmcnt<(C::NS - 2) * C::LOADS>();
    ring::block_barrier();
    issue_stage<C>(c, ga, gb, dma);
    __builtin_amdgcn_sched_barrier(0);      // the loads go out before the tile is multiplied
    multiply_stage<C>(c, rd, part);
}

// part += the k-tile held in stage `rd`
template <class C>
__device__ __forceinline__ void multiply_stage(const Ctx<C> &c, const lds_char *rd, floatx16 (&part)[C::TM])
{
    const lds_char *sa = rd + c.a_wave;
    const lds_char *sb = rd + C::A_BYTES + c.b_base;
    uintx4 fa[2][C::TM];
    float fb[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
            fa[s][i] = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(sa + i * 32 * 64 + c.a_frag[s]);
        if constexpr (C::B_KC) {
            const floatx4 v = *reinterpret_cast<const __attribute__((address_space(3))) floatx4 *>(sb + c.a_frag[s]);
#pragma unroll
            for (int t = 0; t < 4; ++t) fb[s][t] = v[t];
        } else {
#pragma unroll
            for (int t = 0; t < 4; ++t)
                fb[s][t] = *reinterpret_cast<const __attribute__((address_space(3))) float *>(sb + (8 * s + t) * 512);
        }
    }
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < C::TM; ++i)
                part[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(fb[s][t], __uint_as_float(fa[s][i][t]), part[i], 0, 0, 0);
}
#endif

template <class C>
__global__ __launch_bounds__(C::THREADS) void gemm_ring_f32_kernel(Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    __shared__ __attribute__((aligned(1024))) char lds[C::LDS_BYTES];
    constexpr int TM = C::TM, NW = C::NW, NS = C::NS;

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar
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

    const char *A = p.A + batch * p.strideA * 4;
    const char *B = p.B + batch * p.strideB * 4;

    Ctx<C> ctx;
    ctx.wave = wave;
    // A and column-major B: load q covers LDS rows 16q..16q+15; lane l fills row 16q + l/4, slot l%4
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i) {
        const int q = wave + i * NW, r = 16 * q + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        int64_t row = m0 + r;
        row = row < p.M ? row : p.M - 1;
        ctx.a_off[i] = (uint32_t)(row * p.lda * 4 + c * 16);
    }
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i) {
        const int q = wave + i * NW;
        if constexpr (C::B_KC) {
            const int r = 16 * q + (lane >> 2);
            const int c = (lane & 3) ^ ((r >> 2) & 3);
            int64_t row = n0 + r;
            row = row < p.N ? row : p.N - 1;
            ctx.b_off[i] = (uint32_t)(row * p.ldb * 4 + c * 16);
        } else {
            const int pidx = q * 64 + lane, k = pidx >> 5;          // 32 chunks per k-row
            const int c = (pidx & 31) ^ (8 * ((k >> 2) & 1));
            int64_t col = n0 + c * 4;
            col = col + 4 <= p.N ? col : p.N - 4;
            ctx.b_off[i] = (uint32_t)((k * p.ldb + col) * 4);
        }
    }
    const int64_t b_step = C::B_KC ? 64 : 16 * p.ldb * 4;           // bytes per k-tile

    const int frag_row = lane & 31, half = lane >> 5;
#pragma unroll
    for (int s = 0; s < 2; ++s) ctx.a_frag[s] = frag_row * 64 + (((2 * s + half) ^ ((frag_row >> 2) & 3)) << 4);
    ctx.a_wave = wm * C::WTM * 64;
    if constexpr (C::B_KC) {
        ctx.b_base = wn * C::WTN * 64;
    } else {
        const int col = wn * C::WTN + frag_row;
        ctx.b_base = 4 * half * 512 + (((col >> 2) ^ (8 * half)) << 4) + (col & 3) * 4;
    }

    floatx16 acc[TM], part[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;

    lds_char *const base = (lds_char *)lds;
    const int64_t nk = p.K / 16, last = nk - 1;            // nk >= NS
    auto ga = [&](int64_t kt) { return A + (kt < last ? kt : last) * 64; };
    auto gb = [&](int64_t kt) { return B + (kt < last ? kt : last) * b_step; };

    // prologue: tiles 0 .. NS-2
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_stage<C>(ctx, ga(s), gb(s), base + s * C::STAGE_BYTES);

    int64_t kt = 0;
    while (kt + NS <= nk) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) part[i][r] = 0.0f;
        int64_t end = kt + C::FLUSH_ROUNDS * NS;
        end = end < nk ? end : nk;
        for (; kt + NS <= end; kt += NS) {
#pragma unroll
            for (int s = 0; s < NS; ++s)
                ring_step<C>(ctx, ga(kt + s + NS - 1), gb(kt + s + NS - 1),
                             base + ((s + NS - 1) % NS) * C::STAGE_BYTES, base + s * C::STAGE_BYTES, part);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[i] += part[i];
    }
    // the last nk % NS tiles, same stage order
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[i][r] = 0.0f;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (kt + s < nk)
            ring_step<C>(ctx, ga(kt + s + NS - 1), gb(kt + s + NS - 1), base + ((s + NS - 1) % NS) * C::STAGE_BYTES,
                         base + s * C::STAGE_BYTES, part);
#pragma unroll
    for (int i = 0; i < TM; ++i) acc[i] += part[i];
    ring::wait_vmcnt<0>();
    __syncthreads();                         // every load has landed, every wave is done with the stages

    // A K that ends inside a k-tile: the last, partial k-tile goes through stage 0 by ordinary
    // loads, 16-byte chunks at or beyond K written as zeros (K is a whole number of chunks), in
    // the places the DMA loads of a full tile would have filled.
    if (p.K % 16 != 0) {
        const int64_t k0 = nk * 16;
#pragma unroll
        for (int i = 0; i < C::A_INSTR; ++i) {
            const int q = wave + i * NW, r = 16 * q + (lane >> 2);
            const int c = (lane & 3) ^ ((r >> 2) & 3);
            uintx4 v = uintx4{0, 0, 0, 0};
            if (k0 + c * 4 < p.K) v = *reinterpret_cast<const uintx4 *>(A + ctx.a_off[i] + k0 * 4);
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(base + q * 1024 + lane * 16) = v;
        }
#pragma unroll
        for (int i = 0; i < C::B_INSTR; ++i) {
            const int q = wave + i * NW;
            uintx4 v = uintx4{0, 0, 0, 0};
            if constexpr (C::B_KC) {
                const int r = 16 * q + (lane >> 2);
                const int c = (lane & 3) ^ ((r >> 2) & 3);
                if (k0 + c * 4 < p.K) v = *reinterpret_cast<const uintx4 *>(B + ctx.b_off[i] + k0 * 4);
            } else {
                const int k = (q * 64 + lane) >> 5;
                if (k0 + k < p.K) v = *reinterpret_cast<const uintx4 *>(B + ctx.b_off[i] + k0 * p.ldb * 4);
            }
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(base + C::A_BYTES + q * 1024 + lane * 16) = v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) part[i][r] = 0.0f;
        multiply_stage<C>(ctx, base, part);
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[i] += part[i];
        __syncthreads();                     // stage 0 is the epilogue's slab next
    }

    // Epilogue: bias and activation in registers; then each wave passes 32 rows at a time through
    // a private slab (32 rows x 128 bytes, 16-byte chunks XOR-swizzled by the row pair) and
    // stores whole 128-byte lines.  Register r of acc[i] is Z[m][n] with m = mw + 32 i + lane%32,
    // n = nw + 8 (r/4) + 4 (lane/32) + r%4.
    const int64_t mw = m0 + wm * C::WTM, nw = n0 + wn * C::WTN;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    char *Cb = p.C + batch * p.strideC * 4;
    lds_char *slab = base + wave * (32 * 128);
    float bj[4][4];
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
        const int64_t n = nw + 8 * gq + 4 * half;
        if (bias && !(C::EPI == 0 && p.bias_row) && n + 3 < p.N) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(bias + n);
#pragma unroll
            for (int e = 0; e < 4; ++e) bj[gq][e] = v[e];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) bj[gq][e] = (bias && !(C::EPI == 0 && p.bias_row) && n + e < p.N) ? bias[n + e] : 0.0f;
        }
    }
    if constexpr (C::EPI == 1) {
        float *pairs = reinterpret_cast<float *>(p.C);
        const int64_t slice = tile_n * C::WN + wn;
        const bool ragged = nw + C::WTN > p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = mw + 32 * i + frag_row;
            const bool live = m < p.M;
            // this lane holds columns nw + 8 gq + 4 half + e of row m; `want` is the label's offset
            // in those terms without the 4 half (or a value no offset takes)
            const int64_t d = live ? (int64_t)p.labels[m] - nw : -1;
            const int want = d >= 0 && d < C::WTN ? (int)d - 4 * half : -1000;
            float mx = -__builtin_inff(), pick = 0.0f;
            bool hit = false;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int cofs = 8 * gq + e;
                    float v = acc[i][4 * gq + e] + bj[gq][e];
                    if (ragged && nw + cofs + 4 * half >= p.N) v = -__builtin_inff();
                    acc[i][4 * gq + e] = v;
                    mx = __builtin_fmaxf(mx, v);
                    if (want == cofs) { pick = v; hit = true; }
                }
            mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float ref = mx == -__builtin_inff() ? 0.0f : mx;       // a slice wholly past column N
            float sum = 0.0f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f((acc[i][r] - ref) * 1.44269504088896341f);
            sum += __shfl_xor(sum, 32, 64);
            if (live && half == 0)
                *reinterpret_cast<ring::floatx2 *>(pairs + 2 * (slice * p.M + m)) = ring::floatx2{mx, sum};
            if (live && hit) p.picked[m] = pick;
        }
        return;
    }
    if constexpr (C::EPI == 2) {
        // Z = A.B + bias stays where C is (fp32 already); each wave leaves the mean of its 32 columns
        // of every row and the sum of squared deviations from it (see ring::Cfg::EPI)
        float *Z = reinterpret_cast<float *>(p.C);
        ring::floatx2 *pairs = reinterpret_cast<ring::floatx2 *>(p.picked);
        const int64_t slice = tile_n * C::WN + wn;
        const int64_t left = p.N - nw;
        const float count = (float)(left >= C::WTN ? C::WTN : left > 0 ? left : 0);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = mw + 32 * i + frag_row;
            const bool live = m < p.M;
            float sum = 0.0f;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float v = acc[i][4 * gq + e] + bj[gq][e];
                    acc[i][4 * gq + e] = v;
                    sum += (8 * gq + 4 * half + e < left) ? v : 0.0f;
                }
            sum += __shfl_xor(sum, 32, 64);
            const float mean = count > 0.0f ? sum / count : 0.0f;
            float dev = 0.0f;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float d = (8 * gq + 4 * half + e < left) ? acc[i][4 * gq + e] - mean : 0.0f;
                    dev += d * d;
                }
            dev += __shfl_xor(dev, 32, 64);
            if (live && half == 0) pairs[slice * p.M + m] = ring::floatx2{mean, dev};
            if (!live) continue;
            float *zr = Z + m * p.ldc + nw;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int c0 = 8 * gq + 4 * half;
                if (c0 + 4 <= left) {
                    *reinterpret_cast<floatx4 *>(zr + c0) = floatx4{acc[i][4 * gq], acc[i][4 * gq + 1], acc[i][4 * gq + 2], acc[i][4 * gq + 3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c0 + e < left) zr[c0 + e] = acc[i][4 * gq + e];
                }
            }
        }
        return;
    }
    const int wkey = (frag_row >> 1) & 7;
    dispatch_act(p.act, [&](auto act_tag) {
    constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // a bias that runs down the rows: this lane's row of the 32-row group
        const int64_t mb = mw + 32 * i + frag_row;
        const float bi = (bias && p.bias_row && mb < p.M) ? bias[mb] : 0.0f;
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            floatx4 y;
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = apply_act(acc[i][4 * gq + e] + (bj[gq][e] + bi), ACT);
            *reinterpret_cast<__attribute__((address_space(3))) floatx4 *>(
                slab + frag_row * 128 + (((2 * gq + half) ^ wkey) << 4)) = y;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int id = q * 64 + lane, row = id >> 3, chunk = id & 7;
            const floatx4 v = *reinterpret_cast<const __attribute__((address_space(3))) floatx4 *>(
                slab + row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
            const int64_t m = mw + 32 * i + row, n = nw + chunk * 4;
            if (m < p.M && n < p.N) {
                float *dst = reinterpret_cast<float *>(Cb) + m * p.ldc + n;
                if (n + 4 <= p.N) {
                    __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(dst));
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < p.N) dst[e] = v[e];
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
    if (p.dtype != DT_F32 || p.a_col() || p.b_col() != C::B_KC) return false;
    if (p.K < 16 * C::NS || p.K % 4 != 0 || !vector_friendly(p)) return false;
    if (!C::B_KC && (p.N % 4 != 0)) return false;
    // lane offsets are 32-bit byte offsets from the tile's first k
    const int64_t a_span = p.M * p.lda * 4, b_span = (C::B_KC ? p.N : 16) * p.ldb * 4 + p.N * 4;
    if (a_span >= (int64_t(1) << 31) || b_span >= (int64_t(1) << 31)) return false;
    const int64_t tiles = ((p.M + C::BM - 1) / C::BM) * ((p.N + C::BN - 1) / C::BN);
    if (tiles <= 0 || p.batch > 0x7fffffffLL / tiles) return false;
    return true;
}

template <class C>
hipError_t launch(const Problem &p, hipStream_t stream)
{
    Params q;
    q.M = p.M; q.N = p.N; q.K = p.K; q.batch = p.batch;
    q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = p.strideA;
    q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = p.strideB;
    q.bias = p.bias; q.strideBias = p.strideBias;
    q.C = static_cast<char *>(p.C); q.ldc = p.ldc; q.strideC = p.strideC;
    q.tiles_m = (p.M + C::BM - 1) / C::BM;
    q.tiles_n = (p.N + C::BN - 1) / C::BN;
    q.act = p.act;
    q.labels = nullptr; q.picked = nullptr; q.bias_row = p.bias_row ? 1 : 0;
    const int64_t total = q.tiles_m * q.tiles_n * p.batch;
    hipLaunchKernelGGL(gemm_ring_f32_kernel<C>, dim3((unsigned)total), dim3(C::THREADS), 0, stream, q);
    return hipGetLastError();
}

}  // namespace ringf
}  // namespace optiml

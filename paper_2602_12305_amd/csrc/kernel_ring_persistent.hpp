// Persistent form of the bf16 ring kernel of kernel_tile_ring.hpp: one workgroup per CU walks
// a list of 256x256 C tiles, and the ring of LDS stages never drains between tiles.
//
// Why.  A 256x256 workgroup fills a CU (128 KiB of LDS, 512 accumulator registers per SIMD
// lane pair), so in the one-tile-per-workgroup kernel nothing runs on the CU while a tile's
// first loads are in flight or while its results are converted and stored: about 8 us per
// tile, which is 40 % of the time when K = 512.  Here the last NS-1 steps of a tile already
// issue the first NS-1 k-tiles of the next one, the epilogue runs while those loads are in
// flight, and the stores of C drain while the next tile is multiplied.
//
// Wait counts.  A wave's vector-memory operations complete in issue order, and the ring's
// loads are counted by hand (see kernel_tile_ring.hpp).  The epilogue of a whole tile issues a
// fixed number of stores per wave (TM * READS); the first AHEAD+1 steps of the next tile wait
// for loads that are older than those, so they allow that many more operations to be
// outstanding (ring_step<C, EXTRA>).  A tile that
// touches the edge of C stores a data-dependent number of times: after it the wave simply
// waits for everything (s_waitcnt vmcnt(0)) and the next tile starts with the plain counts.
//
// Bias.  The accumulators of a tile start from its bias values instead of zero, which takes the
// addition (a quarter of the vector instructions of a ReLU epilogue) out of the part of the tile
// during which the matrix pipe idles.  The 256 values come by LDS-DMA too (no compiler-tracked
// load sits between the hand-counted ones), into one of two KiB slices per wave, requested
// before the first k-tiles of the tile they belong to: a load older than the ones a step waits
// for can only make that wait stricter.
//
// LDS: NS ring stages, then the bias slices.  The epilogue's staging slabs live in the stage of
// the k-tile multiplied last, the only one no load in flight is aimed at.
#pragma once
#include <type_traits>

#include "kernel_tile_ring.hpp"

namespace optiml {
namespace ringp {

using ring::floatx16;
using ring::floatx4;
using ring::lds_char;
using ring::Params;
using ring::uintx2;
using ring::uintx4;

template <class C>
struct PCfg {
    static constexpr int CPR = C::WTN / 8, PITCH = C::WTN * 2;      // 16-byte chunks and bytes per slab row
    static constexpr int READS = 32 * CPR / 64;                      // 16-byte stores per lane per 32 rows
    static constexpr int STORES = C::TM * READS;                     // per wave per whole tile
    static constexpr int EXTRA = STORES;
    static constexpr int HEAD = C::AHEAD + 1;                        // steps that may still see them
    static constexpr int MIN_NK = HEAD + C::NS - 1;
    static constexpr int BIAS_BYTES = 2 * C::NW * 1024;              // per wave: this tile's slice and the next one's
    static constexpr int LDS_BYTES = C::NS * C::STAGE_BYTES + BIAS_BYTES;
    static_assert(C::NW * 32 * PITCH <= C::STAGE_BYTES, "slabs fit one stage");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

template <class C>
__global__ __launch_bounds__(C::THREADS) void gemm_ring_persistent_kernel(Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    using P = PCfg<C>;
    __shared__ __attribute__((aligned(1024))) char lds[P::LDS_BYTES];
    constexpr int TM = C::TM, TN = C::TN, NW = C::NW, NS = C::NS, STAGE = C::STAGE_BYTES;

    // the wave index as a scalar: everything derived from it (tile corner of the wave, slab and
    // store bases) then lives in scalar registers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % C::WM, wn = wave / C::WM;
    lds_char *const base = (lds_char *)lds;
    // bias slice `slot` (0 or 1) of this wave
    auto bias_slice = [&](int slot) { return base + NS * STAGE + (slot * NW + wave) * 1024; };

    // Tile list of this workgroup.  Workgroup ids go round-robin over the 8 XCDs; XCD x owns a
    // contiguous range of tiles (in band order, see below) and its workgroups take them in turn,
    // so that the tiles in flight on an XCD at any time are neighbours sharing panels in its L2.
    const int64_t total = p.tiles_m * p.tiles_n * p.batch;
    const int64_t G = gridDim.x, x = blockIdx.x & 7, loc = blockIdx.x >> 3;
    const int64_t q8 = total >> 3, r8 = total & 7;
    const int64_t start = x * q8 + (x < r8 ? x : r8), count = q8 + (x < r8 ? 1 : 0);
    const int64_t nwg = (G >> 3) + (x < (G & 7) ? 1 : 0);

    struct Tile { int64_t m0, n0, batch; };
    auto decode = [&](int64_t tile_id) {
        const int64_t per_batch = p.tiles_m * p.tiles_n;
        Tile r;
        r.batch = tile_id / per_batch;
        int64_t t = tile_id % per_batch;
        constexpr int BAND = 8;       // bands of 8 tile rows, walked column by column
        const int64_t band = t / (BAND * p.tiles_n), first = band * BAND;
        const int64_t rows_in_band = p.tiles_m - first < BAND ? p.tiles_m - first : BAND;
        t -= band * BAND * p.tiles_n;
        r.m0 = (first + t % rows_in_band) * C::BM;
        r.n0 = (t / rows_in_band) * C::BN;
        return r;
    };

    ring::Ctx<C> ctx;
    ctx.wave = wave;
    auto set_offsets = [&](const Tile &t) {
#pragma unroll
        for (int i = 0; i < C::A_INSTR; ++i) {
            const int q = wave + i * NW, r = 16 * q + (lane >> 2);
            const int c = (lane & 3) ^ ((r >> 2) & 3);
            int64_t row = t.m0 + r;
            row = row < p.M ? row : p.M - 1;
            ctx.a_off[i] = (uint32_t)row * (uint32_t)p.lda * 2u + c * 16;    // < 2^31, see supports()
        }
#pragma unroll
        for (int i = 0; i < C::B_INSTR; ++i) {
            const int q = wave + i * NW;
            if constexpr (C::B_KC) {
                const int r = 16 * q + (lane >> 2);
                const int c = (lane & 3) ^ ((r >> 2) & 3);
                int64_t row = t.n0 + r;
                row = row < p.N ? row : p.N - 1;
                ctx.b_off[i] = (uint32_t)row * (uint32_t)p.ldb * 2u + c * 16;
            } else {
                const int pidx = q * 64 + lane, k = pidx >> 5;
                const int c = (pidx & 31) ^ (4 * (k & 3));
                int64_t col = t.n0 + c * 8;
                col = col + 8 <= p.N ? col : p.N - 8;
                ctx.b_off[i] = ((uint32_t)k * (uint32_t)p.ldb + (uint32_t)col) * 2u;
            }
        }
    };
    const int64_t b_step = C::B_KC ? 64 : 32 * p.ldb * 2;           // bytes per k-tile

    const int frag_row = lane & 31, half = lane >> 5;
#pragma unroll
    for (int s = 0; s < 2; ++s) ctx.a_frag[s] = frag_row * 64 + (((2 * s + half) ^ ((frag_row >> 2) & 3)) << 4);
    ctx.a_wave = wm * C::WTM * 64;
    ctx.b_wave_kc = wn * C::WTN * 64;
    {
        const int g = lane >> 4, jj = lane & 15;
        ctx.tr_row = 8 * (g >> 1) + (jj >> 2);
        const int tr_col = wn * C::WTN + 16 * (g & 1) + 4 * (jj & 3);
        const int tr_key = 4 * (jj >> 2);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = tr_col + 32 * j;
            ctx.tr_cb[j] = (((col >> 3) ^ tr_key) << 4) + ((col & 7) << 1);
        }
    }

    // One wave-wide load of a tile's bias slice (lane l: four values from column n0 + 4l, clamped
    // at the edge) into slice `slot` of this wave.  The accumulators of the tile start from these
    // values, so the epilogue has no bias to add.
    const bool has_bias = p.bias != nullptr;
    auto issue_bias = [&](const Tile &t, int slot) {
        const char *src = reinterpret_cast<const char *>(p.bias + t.batch * p.strideBias + t.n0);
        const int64_t col = t.n0 + 4 * lane;
        const uint32_t off = (uint32_t)(((col + 4 <= p.N ? col : p.N - 4) - t.n0) * 4);
        ring::dma_load16(ring::scalar_ptr(src), off,
                         __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(bias_slice(slot))));
    };

    const int64_t nk = p.K / 32;                   // >= MIN_NK
    floatx16 acc[TN][TM];
    ring::Frags<C> f0;
    unsigned st = 0;                               // ring stage of the k-tile multiplied next
    auto step = [&](auto extra, const char *ga, const char *gb) {
        lds_char *rd = base + st * STAGE;
        lds_char *dma = base + ((st + NS - 1) % NS) * STAGE;
        lds_char *nx = base + ((st + 1) % NS) * STAGE;
        ring::ring_step<C, decltype(extra)::value>(ctx, ga, gb, dma, rd, nx, f0, acc);
        st = (st + 1) % NS;
    };
    using Plain = std::integral_constant<int, 0>;
    using AfterStores = std::integral_constant<int, P::EXTRA>;

    int64_t j = loc;
    Tile cur = decode(start + j);
    set_offsets(cur);
    const char *ldA = p.A + cur.batch * p.strideA * 2, *ldB = p.B + cur.batch * p.strideB * 2;
    int slot = 0;                                  // bias slice of the current tile
    if (has_bias) issue_bias(cur, slot);
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) ring::issue_stage<C>(ctx, ldA + s * 64, ldB + s * b_step, base + s * STAGE);
    if constexpr (C::PF) {
        ring::wait_vmcnt<(NS - 2) * C::LOADS>();   // k-tile 0 has landed
        ring::block_barrier();
        ring::load_frags<C>(ctx, base, 0, f0);
    }

    bool pending = false;                          // stores of the previous tile may be outstanding
    for (;;) {
        if (has_bias) {
            // The slice was requested before the NS-1 k-tiles in flight (and before the previous
            // tile's stores): once at most those are outstanding it has landed.  It is this
            // wave's own, so no barrier.
            if (pending) ring::wait_vmcnt<(NS - 1) * C::LOADS + P::STORES>();
            else ring::wait_vmcnt<(NS - 1) * C::LOADS>();
            asm volatile("" ::: "memory");
            const lds_char *const bias_rd = bias_slice(slot);
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const floatx4 bv = *reinterpret_cast<const __attribute__((address_space(3))) floatx4 *>(
                        bias_rd + (wn * C::WTN + 32 * jn + 8 * gq + 4 * half) * 4);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[jn][i][4 * gq + e] = bv[e];
                }
        } else {
#pragma unroll
            for (int jn = 0; jn < TN; ++jn)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[jn][i][r] = 0.0f;
        }

        const int64_t jnext = j + nwg;
        const bool has_next = jnext < count;
        Tile nxt = cur;
        // The last NS-1 steps fetch the first k-tiles of the next tile (or, after the last tile,
        // re-fetch those of this one: in bounds, never read).
        auto turn_to_next = [&]() {
            if (has_next) {
                nxt = decode(start + jnext);
                set_offsets(nxt);
                ldA = p.A + nxt.batch * p.strideA * 2;
                ldB = p.B + nxt.batch * p.strideB * 2;
                if (has_bias) issue_bias(nxt, slot ^ 1);
            }
        };
        if (pending) {
            for (int kt = 0; kt < P::HEAD; ++kt) step(AfterStores{}, ldA + (kt + NS - 1) * 64, ldB + (kt + NS - 1) * b_step);
        } else {
            for (int kt = 0; kt < P::HEAD; ++kt) step(Plain{}, ldA + (kt + NS - 1) * 64, ldB + (kt + NS - 1) * b_step);
        }
        for (int64_t kt = P::HEAD; kt + NS <= nk; ++kt) step(Plain{}, ldA + (kt + NS - 1) * 64, ldB + (kt + NS - 1) * b_step);
        turn_to_next();
        for (int s = 0; s < NS - 1; ++s) step(Plain{}, ldA + s * 64, ldB + s * b_step);

        // ---- epilogue of `cur`: bias, activation, bf16 conversion in registers; 32 rows at a time
        // through this wave's slab (swizzled 16-byte chunks) so that every store is a whole line
        ring::wait_vmcnt<63>();                    // this wave's LDS reads of the last k-tile have returned
        ring::block_barrier();                     // ... and everybody's: its stage is free
        {
            const int64_t mw = cur.m0 + wm * C::WTM, nw = cur.n0 + wn * C::WTN;
            // wave-uniform address of the wave's corner of C; lanes add a 32-bit offset
            char *const Cw = p.C + (cur.batch * p.strideC + mw * p.ldc + nw) * 2;
            constexpr int CPR = P::CPR, PITCH = P::PITCH, READS = P::READS;
            lds_char *slab = base + ((st + NS - 1) % NS) * STAGE + wave * (32 * PITCH);
            const bool whole = cur.m0 + C::BM <= p.M && cur.n0 + C::BN <= p.N;
            auto slab_key = [](int row) { return CPR == 8 ? (row >> 1) & 7 : row & 15; };
            const int wkey = slab_key(frag_row);
            auto rows32 = [&](int i, auto whole_tag, auto act_tag) {
                constexpr bool WHOLE = decltype(whole_tag)::value;
                constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
                for (int jn = 0; jn < TN; ++jn)
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        float y[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) y[e] = apply_act_bf16out(acc[jn][i][4 * gq + e], ACT);
                        *reinterpret_cast<__attribute__((address_space(3))) uintx2 *>(
                            slab + frag_row * PITCH + (((4 * jn + gq) ^ wkey) << 4) + 8 * half) =
                            uintx2{pack2_16<C::DT>(y[0], y[1]), pack2_16<C::DT>(y[2], y[3])};
                    }
#pragma unroll
                for (int q = 0; q < READS; ++q) {
                    const int id = q * 64 + lane, row = id / CPR, chunk = id % CPR;
                    const uintx4 v = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(
                        slab + row * PITCH + ((chunk ^ slab_key(row)) << 4));
                    const int64_t m = mw + 32 * i + row, n = nw + chunk * 8;
                    char *dst = Cw + (int64_t)(32 * i) * p.ldc * 2 + ((uint32_t)row * (uint32_t)p.ldc + chunk * 8) * 2u;
                    if constexpr (WHOLE) {
                        __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(dst));
                    } else if (m < p.M && n < p.N) {
                        if (n + 8 <= p.N) {
                            __builtin_nontemporal_store(v, reinterpret_cast<uintx4 *>(dst));
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (n + e < p.N)
                                    reinterpret_cast<unsigned short *>(dst)[e] = (unsigned short)(v[e >> 1] >> ((e & 1) * 16));
                        }
                    }
                }
            };
            dispatch_act(p.act, [&](auto act_tag) {
                if (whole) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) rows32(i, std::true_type{}, act_tag);
                } else {
#pragma unroll
                    for (int i = 0; i < TM; ++i) rows32(i, std::false_type{}, act_tag);
                }
            });
            if (!has_next) break;
            slot ^= 1;
            if (!whole) ring::wait_vmcnt<0>();     // unknown number of stores: start the next tile drained
            pending = whole;
        }
        cur = nxt;
        j = jnext;
    }
    ring::wait_vmcnt<0>();                         // no load may land in LDS after the workgroup has gone
#endif
}

template <class C>
bool supports(const Problem &p)
{
    if (!ring::supports<C>(p)) return false;
    if (p.K % 32 != 0 || p.K / 32 < PCfg<C>::MIN_NK || p.N % 4 != 0) return false;     // whole k-tiles only
    if (p.ldc >= (int64_t(1) << 22)) return false;      // 32 rows of C within a 32-bit byte offset
    return true;
}

// Measured on the batched 2048 x 2048 case: ahead of the one-tile kernels up to K = 1024 (0.096
// against 0.116 ms at K = 192, 0.169 against 0.181 ms at K = 512), level at 2048, behind at 8192
// where the fixed cost per tile no longer matters and the unrolled ring is faster.
template <class C>
bool prefers(const Problem &p)
{
    const int64_t tiles = ((p.M + C::BM - 1) / C::BM) * ((p.N + C::BN - 1) / C::BN) * p.batch;
    return p.K <= 1024 && tiles > compute_units();
}

template <class C>
hipError_t launch(const Problem &p, hipStream_t stream)
{
    const int64_t cus = compute_units();
    Params q;
    q.M = p.M; q.N = p.N; q.K = p.K; q.batch = p.batch;
    q.A = static_cast<const char *>(p.A); q.lda = p.lda; q.strideA = p.strideA;
    q.B = static_cast<const char *>(p.B); q.ldb = p.ldb; q.strideB = p.strideB;
    q.bias = p.bias; q.strideBias = p.strideBias;
    q.C = static_cast<char *>(p.C); q.ldc = p.ldc; q.strideC = p.strideC;
    q.tiles_m = (p.M + C::BM - 1) / C::BM;
    q.tiles_n = (p.N + C::BN - 1) / C::BN;
    q.act = p.act;
    q.labels = nullptr; q.picked = nullptr; q.bias_row = 0;
    const int64_t total = q.tiles_m * q.tiles_n * p.batch;
    const int64_t grid = total < cus ? total : cus;
    hipLaunchKernelGGL(gemm_ring_persistent_kernel<C>, dim3((unsigned)grid), dim3(C::THREADS), 0, stream, q);
    return hipGetLastError();
}

}  // namespace ringp
}  // namespace optiml

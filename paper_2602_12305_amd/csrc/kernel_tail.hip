// The partly filled last round of a tiled contraction, split along k (the stream-K idea in two
// deterministic steps).
//
// A 256 x 256-tile kernel on a problem of T tiles runs ceil(T / CUs) rounds; with T a little over a
// multiple of the CU count (17 x 17 tiles on 256 CUs) the last round keeps a few CUs busy for a whole
// tile's time.  This variant cuts such a problem into
//   * a main block of whole tile rows and columns whose tile count fills its rounds, given to the
//     dispatcher's choice for that block, and
//   * one or two strips (the tile rows below it, the tile columns to its right), whose tiles are too
//     few for a round of their own.  A strip is split along k into S parts so that strip tiles x S is
//     about one workgroup per CU: the ring kernel with the unrounded-product epilogue computes the S
//     partial products as S batches of one launch into fp32 slabs in the workspace, and
//     tail_reduce_kernel adds the slabs in order, adds the bias, applies the activation and rounds.
// Nothing waits for anything inside a kernel and the order of every sum is fixed: bitwise repeatable.
// The variant brings its own time estimate; the dispatcher takes it where that is the smallest.
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

constexpr int64_t kTile = 256;
thread_local bool tl_inside = false;        // the pieces are dispatched through select_variant: not to this variant again

struct Strip {
    int64_t row0, col0, M, N;               // the strip's place in C
    int64_t S, Kc, Krem;                    // S parts of Kc along k, then one of Krem (0: none)
    int64_t ldz, slab, pair_floats;         // fp32 slabs: pitch, floats per slab, statistics floats per part
};
struct Plan {
    bool ok = false;
    int64_t Mm = 0, Nm = 0;                 // the main block: rows [0, Mm), columns [0, Nm)
    int nstrips = 0;
    Strip strip[2];
    double us = 1e30;
};

// time of one 256 x 256 tile over k elements of depth on a full chip, microseconds (the dispatcher's figures
// for the 16-bit ring kernel: 8 us outside the k loop, 4.9 TFLOP/s per workgroup, 7 % less from K = 1024)
double tile_us(int64_t k) { return 8.0 + 2.0 * kTile * kTile * (double)k / (4.9e6 * (k >= 1024 ? 0.93 : 1.0)); }

bool eligible(const Problem &p)
{
    return (p.dtype == DT_BF16 || p.dtype == DT_F16) && !p.a_col() && p.batch == 1 && p.K >= 2048 && p.K % 8 == 0 &&
           (p.b_col() || p.N % 8 == 0) && vector_friendly(p);
}

Problem sub_problem(const Problem &p, int64_t row0, int64_t col0, int64_t M, int64_t N)
{
    Problem q = p;
    const int64_t es = p.esize();
    q.M = M; q.N = N;
    q.A = static_cast<const char *>(p.A) + row0 * p.lda * es;
    q.B = static_cast<const char *>(p.B) + (p.b_col() ? col0 * p.ldb : col0) * es;
    q.C = static_cast<char *>(p.C) + (row0 * p.ldc + col0) * p.csize();
    if (p.bias) q.bias = p.bias + (p.bias_row ? row0 : col0);
    return q;
}

// the strip's split: tiles x S about one workgroup per CU, parts of whole k-tiles, a last part of at least 128
bool split_strip(const Problem &p, Strip &s)
{
    const int64_t tiles = ((s.M + kTile - 1) / kTile) * ((s.N + kTile - 1) / kTile);
    const int64_t cus = compute_units();
    int64_t S = cus / tiles;
    const int64_t by_k = p.K / 512;                                   // parts of 512 or more along k
    S = S < by_k ? S : by_k;
    if (S < 2) return false;
    int64_t Kc = p.K / S / 64 * 64;
    int64_t rem = p.K - S * Kc;
    if (rem > 0 && rem < 128) { Kc = (p.K - 128) / S / 64 * 64; rem = p.K - S * Kc; }
    if (Kc < 256) return false;
    s.S = S; s.Kc = Kc; s.Krem = rem;
    s.ldz = (s.N + 3) / 4 * 4;
    s.slab = s.M * s.ldz;
    s.pair_floats = 2 * 4 * ((s.N + kTile - 1) / kTile) * s.M;
    return true;
}

Problem part_problem(const Problem &p, const Strip &s, int64_t k0, int64_t K, int64_t batch)
{
    Problem q = sub_problem(p, s.row0, s.col0, s.M, s.N);
    const int64_t es = p.esize();
    q.A = static_cast<const char *>(q.A) + k0 * es;
    q.B = static_cast<const char *>(q.B) + (p.b_col() ? k0 : k0 * p.ldb) * es;
    q.K = K; q.batch = batch;
    q.strideA = s.Kc; q.strideB = p.b_col() ? s.Kc : s.Kc * p.ldb;
    q.bias = nullptr; q.strideBias = 0; q.bias_row = false;
    q.act = ACT_NONE;
    q.strideC = s.slab;
    return q;
}

// One or two launches of at most a round of part-tiles, the slabs written and read back (mostly through the caches),
// the reduction.  Calibrated on 4352^2 x 4352 .. 16384 and 4104^3: two strips cost 75 us at K = 4352, 70 us at 16384.
double strip_us(const Problem &p, const Strip &s)
{
    auto part_us = [](int64_t k) { return 3.0 + 2.0 * kTile * kTile * (double)k / 4.9e6; };
    const double parts = (double)(s.S + (s.Krem > 0 ? 1 : 0));
    return part_us(s.Kc) + (s.Krem > 0 ? part_us(s.Krem) : 0.0) + 4.0 + 2.0 * parts * (double)s.slab * 4.0 / 10.0e6;
}

Plan make_plan(const Problem &p)
{
    Plan best;
    if (tl_inside || !eligible(p)) return best;
    const int64_t cus = compute_units();
    const int64_t tm = (p.M + kTile - 1) / kTile, tn = (p.N + kTile - 1) / kTile, tiles = tm * tn;
    if (tiles <= cus || tiles % cus == 0 || tiles % cus > cus / 2) return best;     // last round at most half full
    const double plain_us = (double)((tiles + cus - 1) / cus) * tile_us(p.K);
    for (int64_t r = 0; r <= 2; ++r)
        for (int64_t c = 0; c <= 2; ++c) {
            if ((r == 0 && c == 0) || r >= tm || c >= tn) continue;
            const int64_t main_tiles = (tm - r) * (tn - c), rounds = (main_tiles + cus - 1) / cus;
            if (main_tiles * 100 < rounds * cus * 93 || tiles - main_tiles > cus / 2) continue;
            Plan pl;
            pl.Mm = r > 0 ? (tm - r) * kTile : p.M;
            pl.Nm = c > 0 ? (tn - c) * kTile : p.N;
            pl.us = (double)rounds * tile_us(p.K);
            bool fine = true;
            if (r > 0) {
                Strip &s = pl.strip[pl.nstrips++];
                s.row0 = pl.Mm; s.col0 = 0; s.M = p.M - pl.Mm; s.N = p.N;
                fine = fine && split_strip(p, s);
            }
            if (c > 0 && fine) {
                Strip &s = pl.strip[pl.nstrips++];
                s.row0 = 0; s.col0 = pl.Nm; s.M = pl.Mm; s.N = p.N - pl.Nm;
                fine = fine && split_strip(p, s);
            }
            if (!fine) continue;
            for (int i = 0; i < pl.nstrips; ++i) {
                // every part has to be a problem the unrounded-product kernel takes
                const Strip &s = pl.strip[i];
                fine = fine && unrounded_products_supported(part_problem(p, s, 0, s.Kc, s.S));
                if (s.Krem > 0) fine = fine && unrounded_products_supported(part_problem(p, s, s.S * s.Kc, s.Krem, 1));
                pl.us += strip_us(p, s);
            }
            if (!fine || pl.us >= 0.9 * plain_us || pl.us >= best.us) continue;
            pl.ok = true;
            best = pl;
        }
    return best;
}

// C strip = act(sum of the parts' slabs in order + bias), four columns a thread
template <int DT>
__global__ __launch_bounds__(256) void tail_reduce_kernel(const float *__restrict__ Z, int parts, int64_t slab, int64_t ldz, int64_t M,
                                                          int64_t N, const float *__restrict__ bias, int bias_row, int act,
                                                          unsigned short *__restrict__ C, int64_t ldc)
{
    const int64_t quads = (N + 3) / 4;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= M * quads) return;
    const int64_t row = id / quads, col = (id % quads) * 4;
    floatx4 z = *reinterpret_cast<const floatx4 *>(Z + row * ldz + col);
    for (int s = 1; s < parts; ++s) z += *reinterpret_cast<const floatx4 *>(Z + s * slab + row * ldz + col);
    float y[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float b = !bias ? 0.0f : bias_row ? bias[row] : (col + e < N ? bias[col + e] : 0.0f);
        y[e] = apply_act(z[e] + b, act);
    }
    unsigned short *dst = C + row * ldc + col;
    if (col + 4 <= N && ((reinterpret_cast<uintptr_t>(dst) & 7) == 0)) {
        *reinterpret_cast<uintx2 *>(dst) = uintx2{pack2_16<DT>(y[0], y[1]), pack2_16<DT>(y[2], y[3])};
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < N) dst[e] = to_16<DT>(y[e]);
    }
}

size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

bool tail_supports(const Problem &p) { return make_plan(p).ok; }

double tail_estimate(const Problem &p)
{
    const Plan pl = make_plan(p);
    return pl.ok ? pl.us : 1e30;
}

hipError_t tail_launch(const Problem &p, hipStream_t stream)
{
    const Plan pl = make_plan(p);
    if (!pl.ok) return hipErrorInvalidValue;
    size_t need = 0;
    for (int i = 0; i < pl.nstrips; ++i) {
        const Strip &s = pl.strip[i];
        const size_t parts = (size_t)(s.S + (s.Krem > 0 ? 1 : 0));
        const size_t bytes = align256(parts * (size_t)s.slab * 4) + align256(parts * (size_t)s.pair_floats * 4);
        need = bytes > need ? bytes : need;                              // the strips run one after the other
    }
    void *ws = nullptr;
    hipError_t e = workspace(need, &ws, stream);
    if (e != hipSuccess) return e;

    // the main block: whatever the dispatcher picks for it among the one-launch tile kernels
    struct Inside { Inside() { tl_inside = true; } ~Inside() { tl_inside = false; } } inside;
    const Problem main = sub_problem(p, 0, 0, pl.Mm, pl.Nm);
    const Variant *v = variant_at(select_variant(main, nullptr, false));
    if (!v || v->estimate_us) return hipErrorInvalidValue;               // a single kernel without scratch of its own
    e = v->launch(main, stream);
    if (e != hipSuccess) return e;

    for (int i = 0; i < pl.nstrips; ++i) {
        const Strip &s = pl.strip[i];
        const int parts = (int)(s.S + (s.Krem > 0 ? 1 : 0));
        float *Z = static_cast<float *>(ws);
        float *pairs = reinterpret_cast<float *>(static_cast<char *>(ws) + align256((size_t)parts * (size_t)s.slab * 4));
        e = launch_unrounded_products(part_problem(p, s, 0, s.Kc, s.S), Z, s.ldz, pairs, stream);
        if (e != hipSuccess) return e;
        if (s.Krem > 0) {
            e = launch_unrounded_products(part_problem(p, s, s.S * s.Kc, s.Krem, 1), Z + s.S * s.slab, s.ldz,
                                          pairs + s.S * s.pair_floats, stream);
            if (e != hipSuccess) return e;
        }
        const Problem q = sub_problem(p, s.row0, s.col0, s.M, s.N);
        const int64_t threads = s.M * ((s.N + 3) / 4);
        const dim3 grid((unsigned)((threads + 255) / 256));
        if (p.dtype == DT_F16)
            hipLaunchKernelGGL(tail_reduce_kernel<DT_F16>, grid, dim3(256), 0, stream, Z, parts, s.slab, s.ldz, s.M, s.N, q.bias,
                               p.bias_row ? 1 : 0, p.act, static_cast<unsigned short *>(q.C), p.ldc);
        else
            hipLaunchKernelGGL(tail_reduce_kernel<DT_BF16>, grid, dim3(256), 0, stream, Z, parts, s.slab, s.ldz, s.M, s.N, q.bias,
                               p.bias_row ? 1 : 0, p.act, static_cast<unsigned short *>(q.C), p.ldc);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

const Variant *tail_variants()
{
    static const Variant v[kNumTailVariants] = {{"xtail_split", tail_supports, tail_launch, 256, 256,
                                                 reinterpret_cast<const void *>(&tail_reduce_kernel<DT_BF16>), nullptr, true,
                                                 tail_estimate}};
    return v;
}

}  // namespace optiml

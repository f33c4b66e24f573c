// C-ABI entry points: argument validation (host integers only, before any GPU
// call), variant selection, launch.  See include/optiml.h for the contract.
#include "../../include/optiml.h"
#include "common.hpp"

#include <mutex>
#include <vector>

// Device memory for optiml_gemm_epilogue_noalloc: one copy per GPU the library runs on, held until
// the process ends.  In host code this name is a stand-in, not a device address: the address comes
// from hipGetSymbolAddress (static_scratch() below) and only that pointer is ever handed to kernels.
static __device__ __align__(256) unsigned char scratch[OPTIML_NOALLOC_SCRATCH_BYTES];

namespace optiml {

namespace {

thread_local int tls_last_hip_error = 0;
thread_local size_t tls_workspace_head = 0;      // see WorkspaceHead
// workspace() refused (too small and not allowed to grow): the entry points report
// OPTIML_ERR_UNSUPPORTED instead of a HIP error
thread_local bool tls_workspace_refused = false;

int status_of(hipError_t e)
{
    if (e == hipSuccess) return OPTIML_OK;
    if (tls_workspace_refused) {
        tls_workspace_refused = false;
        return OPTIML_ERR_UNSUPPORTED;
    }
    tls_last_hip_error = (int)e;
    return OPTIML_ERR_HIP;
}


struct Table {
    std::vector<const Variant *> v;
    int first_skinny = 0, first_tile = 0;
    Table()
    {
        for (int i = 0; i < kNumGenericVariants; ++i) v.push_back(&generic_variants()[i]);
        first_skinny = (int)v.size();
        for (int i = 0; i < kNumSkinnyVariants; ++i) v.push_back(&skinny_variants()[i]);
        for (int i = 0; i < kNumSkinny16Variants; ++i) v.push_back(&skinny16_variants()[i]);
        for (int i = 0; i < kNumSkinnyRcVariants; ++i) v.push_back(&skinny_rc_variants()[i]);
        first_tile = (int)v.size();
        for (int i = 0; i < kNumTileVariants; ++i) v.push_back(&tile_variants()[i]);
        for (int i = 0; i < kNumTransposeVariants; ++i) v.push_back(&transpose_variants()[i]);
        for (int i = 0; i < kNumPadVariants; ++i) v.push_back(&pad_variants()[i]);
        for (int i = 0; i < kNumTailVariants; ++i) v.push_back(&tail_variants()[i]);
        for (int i = 0; i < kNumF6Variants; ++i) v.push_back(&f6_variants()[i]);
    }
};

const Table &table()
{
    static const Table t;
    return t;
}

bool enum_ok(int layout, int dtype, int act)
{
    return layout >= 0 && layout <= 3 && dtype >= DT_F32 && dtype <= DT_BF6 && act >= 0 && act <= 3;
}

// OPTIML_OK when the arguments describe a valid problem (possibly an empty one).
int validate(const Problem &p)
{
    if (!enum_ok(p.layout, p.dtype, p.act)) return OPTIML_ERR_INVALID_ARG;
    if (p.pre_status != OPTIML_OK) return p.pre_status;
    if (p.batch < 0 || p.M < 0 || p.N < 0 || p.K < 0) return OPTIML_ERR_INVALID_ARG;
    if (p.strideA < 0 || p.strideB < 0 || p.strideBias < 0 || p.strideC < 0) return OPTIML_ERR_INVALID_ARG;
    if (p.lda < 0 || p.ldb < 0 || p.ldc < 0) return OPTIML_ERR_INVALID_ARG;
    // Every operand must span fewer than 2^47 elements (batch stride and leading dimension
    // included), so that no index or byte offset formed from these numbers can leave int64.
    constexpr int64_t kMaxSpan = int64_t(1) << 47;
    auto span_ok = [](int64_t batch, int64_t stride, int64_t rows, int64_t ld, int64_t cols) {
        const __int128 span = (__int128)(batch > 0 ? batch - 1 : 0) * stride + (__int128)(rows > 0 ? rows - 1 : 0) * ld + cols;
        return span < kMaxSpan;
    };
    if (!span_ok(p.batch, p.strideC, p.M, p.ldc, p.N) || !span_ok(p.batch, p.strideBias, 1, 0, p.bias_row ? p.M : p.N) ||
        !span_ok(p.batch, p.strideA, p.a_col() ? p.K : p.M, p.lda, p.a_col() ? p.M : p.K) ||
        !span_ok(p.batch, p.strideB, p.b_col() ? p.N : p.K, p.ldb, p.b_col() ? p.K : p.N))
        return OPTIML_ERR_INVALID_ARG;
    if (p.batch == 0 || p.M == 0 || p.N == 0) return OPTIML_OK;
    if (!p.C || p.ldc < p.N) return OPTIML_ERR_INVALID_ARG;
    if (p.batch > 1 && p.strideC < (p.M - 1) * p.ldc + p.N) return OPTIML_ERR_INVALID_ARG;
    if (p.K > 0) {
        if (!p.A || !p.B) return OPTIML_ERR_INVALID_ARG;
        if (p.lda < (p.a_col() ? p.M : p.K)) return OPTIML_ERR_INVALID_ARG;
        if (p.ldb < (p.b_col() ? p.K : p.N)) return OPTIML_ERR_INVALID_ARG;
    }
    return OPTIML_OK;
}

// a variant can run p: its own shape / alignment test, and the row-wise bias if p carries one
bool can_run(const Variant *v, const Problem &p)
{
    return (!(p.bias_row && p.bias) || v->row_bias) && v->supports(p);
}

bool is_empty(const Problem &p) { return p.batch == 0 || p.M == 0 || p.N == 0; }

// ---- Variant selection: a small cost model, calibrated on this chip -------------------------
//
// Tile kernels.  Time = rounds x (fixed + flop per tile / rate of one workgroup).  `fixed` is the
// part of a tile that is not its k loop (first loads in flight, epilogue), `rate` what one
// workgroup sustains when the whole chip runs the kernel, `share` how many workgroups' worth of
// that rate a CU delivers when it holds several (1: rounds are whole, a 257th tile costs a second
// round).  `boost`: the 16-bit direct-to-LDS kernels are bounded by the board's power, and a
// partly filled chip clocks up to 1.5 x higher (64 tiles of 256 x 256 at K = 2048: 43.6 us, where
// the full-chip rate would give 63).  Numbers from 4096^3 (full chip) and from 64 x 4096 x 4096,
// 128 x 8192 x 8192, 1024^3, 2048^3 (part of the chip), in us and TFLOP/s:
//   ring 256x256 (16-bit) 8 + f / 4.9      ring 256x256 (8-bit, 64-deep) 8 + f / 9.0, else f / 6.6
//   ring 128x256 (four waves, two workgroups to a CU) 6.9 + f / 2.53 per workgroup, both running:
//     32 x 2048 x 2048 x K: 0.106 / 0.161 ms at K = 256 / 512 (0.123 / 0.170 for 256x256), 8 x 4096 x 4096 x 1024
//     0.267 (0.2585), so 7 % are taken off its rate from K = 1024
//   persistent ring       6.5 + f / 4.59   (more tiles than CUs only; 0.096 / 0.169 ms at K = 192 / 512)
//   direct 256x256 8.5 + f / 4.4           direct 256x128 7.5 + f / 3.86
//   direct 128x128 2.7 + f / 2.56, 1.45 workgroups' worth per CU
//   staged 16-bit 256x256 5 + f / 2.0, 256x128 4 + f / 1.8, 128x128 3 + f / 1.17 (1.8 per CU)
//   fp32 ring 128x128 3 + f / 0.548, 256x128 3 + f / 0.53
//   staged fp32 256x128 4 + f / 0.41, 128x128 3 + f / 0.33, 64x64 3 + f / 0.151 (2.3 per CU)
// A CU reaches its `share` only gradually: with n workgroups per CU it delivers min(share,
// 1 + 0.45 (n - 1)) (64x64 fp32 tiles at 1536^3, 2.25 per CU: 124 us, not the 86 us of n = share).
// The staged 128- and 256-row kernels lose about a fifth on a K with a partial last k-tile
// (3000^3: 878 us estimated 633 without it).
struct Cost {
    float fixed_us = 0, tf_wg = 0, share = 1;
    bool boost = false, many_tiles_only = false;
};

Cost cost_of(const Variant *v)
{
    Cost c;
    switch (v->family) {
    case FAM_RINGP: c.fixed_us = 6.5f; c.tf_wg = 4.59f; c.boost = true; c.many_tiles_only = true; break;
    case FAM_RINGF: c.fixed_us = 3.0f; c.tf_wg = v->bm == 128 ? 0.548f : 0.53f; break;
    // (10 us of start and end: 512 x 8192 x 256 takes 13.1 us, 8 x 512^3 15.0 us, against 11.3 and 13.0 for the 128 x 256 kernel)
    case FAM_RING8_K64: c.fixed_us = 10.0f; c.tf_wg = 9.0f; c.boost = true; break;
    case FAM_RING8:
        if (v->bm == 128) { c.fixed_us = 6.9f; c.tf_wg = 3.4f; c.share = 2.0f; c.boost = true; }
        else { c.fixed_us = 8.0f; c.tf_wg = 6.6f; c.boost = true; }
        break;
    case FAM_RING16:
        if (v->bm == 128) { c.fixed_us = 6.9f; c.tf_wg = 2.53f; c.share = 2.0f; c.boost = true; }     // two workgroups to a CU
        else { c.fixed_us = 8.0f; c.tf_wg = 4.9f; c.boost = true; }
        break;
    case FAM_DIRECT:
        c.boost = true;
        if (v->bm == 256 && v->bn == 256) { c.fixed_us = 8.5f; c.tf_wg = 4.4f; }
        else if (v->bm == 256) { c.fixed_us = 7.5f; c.tf_wg = 3.86f; }
        else { c.fixed_us = 2.7f; c.tf_wg = 2.56f; c.share = 1.45f; }
        break;
    case FAM_TILEF:
        if (v->bm == 256) { c.fixed_us = 4.0f; c.tf_wg = 0.41f; }
        else if (v->bm == 128) { c.fixed_us = 3.0f; c.tf_wg = 0.33f; c.share = 1.07f; }
        else { c.fixed_us = 3.0f; c.tf_wg = 0.151f; c.share = 2.3f; }
        break;
    case FAM_TILE16:
        if (v->bm == 256 && v->bn == 256) { c.fixed_us = 5.0f; c.tf_wg = 2.0f; }
        else if (v->bm == 256) { c.fixed_us = 4.0f; c.tf_wg = 1.8f; }
        else { c.fixed_us = 3.0f; c.tf_wg = 1.17f; c.share = 1.8f; }
        break;
    default: break;                    // no model: the variant brings its own estimate or none
    }
    return c;
}

double tile_estimate_us(const Variant *v, const Cost &c, const Problem &p)
{
    const double kCUs = (double)compute_units();
    const double tiles = (double)((p.M + v->bm - 1) / v->bm) * (double)((p.N + v->bn - 1) / v->bn) * (double)p.batch;
    if (c.many_tiles_only && tiles <= kCUs) return 1e30;
    const double fill = tiles < kCUs ? tiles / kCUs : 1.0;
    double rate = c.tf_wg * (c.boost ? 1.5 - 0.5 * fill : 1.0);                // TFLOP/s = flop per us / 1e6
    if ((v->family == FAM_TILE16 || v->family == FAM_TILEF) && v->bm >= 128 && p.K % (p.dtype == DT_F32 ? 16 : 32) != 0) rate *= 0.8;
    // the direct kernels fetch 128-byte row segments: with a row pitch that is not a multiple of 128 bytes each
    // straddles two cache lines (3000^3 bf16: 101 us where the estimate without this says 64)
    if (v->family == FAM_DIRECT && ((p.lda * 2) % 128 != 0 || (p.ldb * 2) % 128 != 0)) rate *= 0.65;
    // (the 16-bit kernel with B column-major loses more: 8448^2 x 4096 594 against 522 us for the 256 x 256 kernel, where B
    // row-major gives 522 against 507)
    if ((v->family == FAM_RING16 || v->family == FAM_RING8) && v->bm == 128 && p.K >= 1024)
        rate *= v->family == FAM_RING16 && p.b_col() ? 0.76 : 0.93;
    const double tile_us = c.fixed_us + 2.0 * v->bm * v->bn * (double)p.K / (rate * 1e6);
    if (c.share == 1.0f) return tile_us * (double)(int64_t)((tiles + kCUs - 1.0) / kCUs);
    const double n = tiles / kCUs;                                             // workgroups per CU
    if (n <= 1.0) return tile_us;
    const double grown = 1.0 + 0.45 * (n - 1.0);
    return tile_us * n / (grown < c.share ? grown : c.share);
}

// Streaming kernels (B read once per 16 rows of A, the blocks of rows side by side): the first
// pass comes from memory at about 6.5 TB/s, the others largely from the caches, at a rate that
// grows with the length of a workgroup's k range: row-major B 20 K / (K + 150) TB/s (16-bit) and
// 14 K / (K + 120) TB/s (fp32, where the matrix instruction is the slower side); column-major B
// 16 K / (K + 900) and 12 K / (K + 600).  Measured from 8 x 512^3 and 64 x 4096 x 4096 to 4096^3,
// within 20 %; 4 us for the two launches.
double stream_estimate_us(const Problem &p)
{
    const double rb = (double)((p.M + 15) / 16), K = (double)p.K;
    // whole column blocks are read: 64 columns (128 in 16-bit) at least, else multiples of 128 (256)
    const int64_t cols = p.layout == 1 ? 16 : p.dtype == DT_F32 ? (p.N <= 64 ? 64 : 128) : (p.N <= 128 ? 128 : 256);
    const double bytes = (double)p.batch * K * (double)((p.N + cols - 1) / cols * cols) * (double)p.esize();
    double again;                                                              // bytes per us
    if (p.layout == 1) again = p.dtype == DT_F32 ? 12e6 * K / (K + 600.0) : 16e6 * K / (K + 900.0);
    else again = p.dtype == DT_F32 ? 14e6 * K / (K + 120.0) : 20e6 * K / (K + 150.0);
    return 4.0 + bytes / 6.5e6 + bytes * (rb - 1.0) / again;
}

// workgroups the streaming kernels launch: column blocks x row blocks x batch x the split along k
// they choose (never ranges shorter than `k_min` per workgroup)
int64_t stream_workgroups(const Problem &p, int64_t cols, int64_t k_min)
{
    const int64_t blocks = (p.N + cols - 1) / cols * p.batch * ((p.M + 15) / 16);
    const int64_t cus = compute_units();
    int64_t split = cus / blocks;                                  // whole rounds, as the launchers choose
    const int64_t by_k = p.K / k_min > 0 ? p.K / k_min : 1;
    split = split < by_k ? split : by_k;
    return blocks * (split < 1 ? 1 : split > 64 ? 64 : split);
}

// The streaming variant for p, or -1.  Within a family the first entry is the one tuned on 16 rows
// x 16384 x 16384; problems on which it would launch fewer than 192 workgroups take the entry
// with half the columns per workgroup (8 x 4096 x 4096: 13.5 against 20.6 us in bf16, 17.3 against
// 19.7 us in fp32, 8.0 against 10.5 us with B column-major), and more than one block of rows takes
// the entries that leave B in the caches (32 x 16384 x 1024 in bf16: 9.5 against 18.5 us) or,
// for a short K and few columns, the four-wave entry (768 x 3072 x 768: 23 against 31 us).
int stream_variant(const Table &t, const Problem &p)
{
    // entries are found by the role their table gives them; a variant's own support test keeps to its
    // storage type and layouts, so the first entry of a role that can run p is the one of p's family
    auto by_role = [&](int role) {
        for (int i = t.first_skinny; i < t.first_tile; ++i)
            if (t.v[i]->role == role && can_run(t.v[i], p)) return i;
        return -1;
    };
    if (p.layout > 1) return -1;
    int want = ROLE_STREAM_DEFAULT;
    const int64_t enough = compute_units() * 3 / 4;               // workgroups below which the chip is starved
    if (p.layout == 0 && p.dtype == DT_F32) {
        // (the narrow entry only while its workgroups still fit in one round: 16 x 20480 x 8192 takes 160 us
        // with 320 of them against 122 us with 160 of the wide one)
        const bool starved = stream_workgroups(p, 128, 1024) < enough && stream_workgroups(p, 64, 1024) > stream_workgroups(p, 128, 1024) &&
                             stream_workgroups(p, 64, 1024) <= compute_units();
        // a few blocks of rows over a small B: 64 columns a workgroup (128 x 4096 x 4096: 46 against 50 us,
        // 128 x 2048 x 2048: 15 against 19 us; 256 x 4096 x 4096: 86 against 81 us)
        // (not over a short K: 32 x 16384 x 1024 takes 20.9 against 15.7 us), and whenever N is at most 64
        const bool few_rows = (p.M <= 128 && p.K >= 2048 && (double)p.K * (double)p.N <= 16777216.0) || p.N <= 64;
        // a B of up to 16 MiB under at most 16 blocks of rows (one block: up to 4 MiB): eight waves deep in k
        // (128 x 2048 x 2048: 12.3 against 15.1 us, 96 x 1024 x 4096: 15.2 against 18.6 us, 16 x 1024 x 1024: 8.1
        // against 9.3 us; 16 x 2048 x 2048: 13.8 against 11.8 us, 512 x 2048 x 2048: 60 against 44 us)
        const double kn = (double)p.K * (double)p.N * (double)p.batch;
        const bool small = p.M <= 256 && (p.M > 16 ? kn <= 4194304.0 : kn <= 1048576.0);
        if (small) want = ROLE_STREAM_SMALL;
        else if (p.M > 16) want = starved || few_rows ? ROLE_STREAM_NARROW : ROLE_STREAM_ROWS;
        else want = starved ? ROLE_STREAM_NARROW : ROLE_STREAM_DEFAULT;
    } else if (p.layout == 0 && (p.dtype == DT_BF16 || p.dtype == DT_F16)) {
        // 128 columns a workgroup while B has up to 100 M elements (16 x 8192 x 8192: 27.5 against 29.2 us,
        // 13 x 10000 x 12000: 53.8 against 51.6 us, 16 x 28672 x 8192: 85.8 against 75.6 us) or the wide entry
        // would leave CUs without a workgroup
        const bool starved = stream_workgroups(p, 256, 1024) < enough && stream_workgroups(p, 128, 1024) > stream_workgroups(p, 256, 1024) &&
                             stream_workgroups(p, 128, 1024) <= compute_units();
        const double kn = (double)p.K * (double)p.N * (double)p.batch;
        const bool narrow = starved || kn <= 100e6;
        want = narrow ? ROLE_STREAM_NARROW : p.M > 16 ? ROLE_STREAM_ROWS : ROLE_STREAM_DEFAULT;
        // a B of up to 8 MiB under at most 16 blocks of rows: eight waves deep in k (16 x 2048 x 2048: 10.1
        // against 12.6 us, 128 x 2048 x 2048: 9.9 against 11.3 us)
        if (kn <= 4194304.0 && p.M <= 256) want = ROLE_STREAM_SMALL;
    } else if (p.layout == 1) {
        const int64_t k_min = 32 * 256 / p.esize();               // 32 steps of 256 bytes
        const bool starved = stream_workgroups(p, 64, k_min) < enough && stream_workgroups(p, 32, k_min) > stream_workgroups(p, 64, k_min) &&
                             stream_workgroups(p, 32, k_min) <= compute_units();
        want = starved ? ROLE_STREAM_NARROW : ROLE_STREAM_DEFAULT;
        // 8-bit operands over a short K: the register-only kernel (1024^3: 14.8 against 17.2 us, 1008^3: 15.5
        // against 25.8 us)
        if (is_f8(p.dtype) && p.K <= 2048 && p.M > 16) want = ROLE_STREAM_REGS;
    } else {
        return -1;
    }
    int id = by_role(want);
    if (id < 0 && want != ROLE_STREAM_DEFAULT) id = by_role(p.M > 16 && want != ROLE_STREAM_ROWS ? ROLE_STREAM_ROWS : ROLE_STREAM_DEFAULT);
    if (id < 0) id = by_role(ROLE_STREAM_DEFAULT);
    if (id >= 0) return id;
    // any other streaming entry that takes the problem
    for (int i = t.first_skinny; i < t.first_tile; ++i)
        if (can_run(t.v[i], p)) return i;
    return -1;
}

// Up to 16 rows: the streaming kernels.  Else a variant that copies an operand into the layout
// a faster kernel wants and declares the problem worth it; else the smallest estimate among the
// streaming variant, the tile kernels and the variants that bring their own estimate; then tile
// kernels without an estimate (the first whose grid gives every CU a workgroup, else the one with
// most workgroups); then the fallback.
int select(const Problem &p, double *estimate_us = nullptr, bool allow_streaming = true)
{
    const Table &t = table();
    const int64_t kComputeUnits = compute_units();
    double unused;
    double &us_out = estimate_us ? *estimate_us : unused;
    us_out = 1e30;
    // the element-wise fallback: a launch, then 64 x 64 blocks at 0.047 TFLOP/s each, four of them to a CU (48
    // TFLOP/s with the chip full, in every storage type; 1025 x 1031 x 2051: 405 us, 4097^3: 2.9 ms)
    const double fallback_tiles = (double)((p.M + 63) / 64) * (double)((p.N + 63) / 64) * (double)p.batch;
    const double fallback_us = 5.0 + (fallback_tiles < 1024.0 ? 1.0 : fallback_tiles / 1024.0) * 2.0 * 4096.0 * (double)p.K / 0.047e6;
    if (p.K > 0 && vector_friendly(p)) {
        const int sv = allow_streaming ? stream_variant(t, p) : -1;
        const double stream_us = sv >= 0 ? stream_estimate_us(p) : 1e30;
        if (sv >= 0 && p.M <= 16) { us_out = stream_us; return sv; }
        static const std::vector<Cost> costs = [&t] {
            std::vector<Cost> c;
            for (const Variant *v : t.v) c.push_back(cost_of(v));
            return c;
        }();
        for (int i = t.first_tile; i < (int)t.v.size(); ++i)
            if (costs[i].tf_wg == 0 && !t.v[i]->estimate_us && t.v[i]->prefers && t.v[i]->prefers(p) && can_run(t.v[i], p))
                return i;
        int best = -1;
        double best_us = 1e30;
        for (int i = t.first_tile; i < (int)t.v.size(); ++i) {
            if ((costs[i].tf_wg == 0 && !t.v[i]->estimate_us) || !can_run(t.v[i], p)) continue;
            const double us = t.v[i]->estimate_us ? t.v[i]->estimate_us(p) : tile_estimate_us(t.v[i], costs[i], p);
            if (t.v[i]->estimate_us && us >= 0.7 * fallback_us) continue;    // a copy path that the one-launch fallback matches
            if (us < best_us) { best = i; best_us = us; }
        }
        if (sv >= 0 && (best < 0 || stream_us < best_us)) { us_out = stream_us; return sv; }
        if (best >= 0) { us_out = best_us; return best; }
        int64_t best_blocks = -1;
        for (int i = t.first_tile; i < (int)t.v.size(); ++i) {
            if (!can_run(t.v[i], p)) continue;
            const int64_t blocks = ((p.M + t.v[i]->bm - 1) / t.v[i]->bm) * ((p.N + t.v[i]->bn - 1) / t.v[i]->bn) * p.batch;
            if (blocks >= kComputeUnits) return i;
            if (blocks > best_blocks) { best = i; best_blocks = blocks; }
        }
        if (best >= 0) return best;
    }
    // nothing above takes the problem as it is: a variant that first copies it into a form they take, if it
    // expects to beat the element-wise fallback (about 50 TFLOP/s in every storage type)
    if (p.K > 0) {
        int best = -1;
        double best_us = 0.7 * fallback_us;          // several launches against one: only for a clear gain
        for (int i = t.first_tile; i < (int)t.v.size(); ++i) {
            if (!t.v[i]->estimate_us || !can_run(t.v[i], p)) continue;
            const double us = t.v[i]->estimate_us(p);
            if (us < best_us) { best = i; best_us = us; }
        }
        if (best >= 0) { us_out = best_us; return best; }
    }
    for (int i = 0; i < t.first_skinny; ++i)
        if (can_run(t.v[i], p)) return i;
    return OPTIML_ERR_UNSUPPORTED;
}

int run(const Problem &p, int variant_id, void *stream)
{
    const Table &t = table();
    if (variant_id < 0 || variant_id >= (int)t.v.size()) return OPTIML_ERR_INVALID_ARG;
    if (!can_run(t.v[variant_id], p)) return OPTIML_ERR_UNSUPPORTED;
    hipError_t e = t.v[variant_id]->launch(p, static_cast<hipStream_t>(stream));
    return status_of(e);
}

Problem make(int64_t batch, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, int64_t strideA,
             const void *B, int64_t ldb, int64_t strideB, const float *bias, int64_t strideBias,
             void *C, int64_t ldc, int64_t strideC, int layout, int dtype, int act)
{
    Problem p;
    p.batch = batch; p.M = M; p.N = N; p.K = K;
    p.A = A; p.lda = lda; p.strideA = strideA;
    p.B = B; p.ldb = ldb; p.strideB = strideB;
    p.bias = bias; p.strideBias = strideBias;
    p.C = C; p.ldc = ldc; p.strideC = strideC;
    p.layout = layout; p.dtype = dtype; p.act = act;
    if (layout >= 4 && layout <= 7) {
        // Column-major C (bit 2): C^T = B^T . A^T is the same problem with a row-major result.
        // B^T takes A's place - it is row-major exactly when B was column-major - and A^T takes
        // B's; the bias, one value per column of C, runs down the rows of C^T.
        p.M = N; p.N = M;
        p.A = B; p.lda = ldb; p.strideA = strideB;
        p.B = A; p.ldb = lda; p.strideB = strideA;
        p.layout = ((layout & 1) ? 0 : 2) | ((layout & 2) ? 0 : 1);
        p.bias_row = true;
    }
    if (dtype == DT_F4) {
        // Two E2M1 values to a byte along k: from here on the problem is described in bytes of k.  That needs k
        // contiguous in both operands and whole bytes in every row.
        if (K < 0 || (K & 1) || (p.lda & 1) || (p.ldb & 1) || (p.strideA & 1) || (p.strideB & 1)) p.pre_status = OPTIML_ERR_INVALID_ARG;
        else if (p.layout != 1) p.pre_status = OPTIML_ERR_UNSUPPORTED;
        p.K = K / 2; p.lda /= 2; p.ldb /= 2; p.strideA /= 2; p.strideB /= 2;
    }
    if (is_f6(dtype)) {
        // Dense 6-bit codes, four to three bytes: every row and every matrix of a batch starts on a byte.  (Any
        // layout: the element-wise fallback addresses single codes; the matrix-pipe path takes k contiguous in both
        // operands and K a multiple of 4.)
        if ((p.lda & 3) || (p.ldb & 3) || (p.strideA & 3) || (p.strideB & 3)) p.pre_status = OPTIML_ERR_INVALID_ARG;
    }
    return p;
}

// The per-device workspace: either the library's own buffer (allocated on first need; a larger
// need allocates a new one and RETIRES the old one, which stays allocated until the process ends:
// work already enqueued, and HIP graphs captured earlier, may still hold its address) or a buffer
// the caller handed over with optiml_set_workspace (never grown, never freed here).
struct DeviceScratch {
    void *own = nullptr;           // the library's buffer
    size_t own_bytes = 0;
    std::vector<void *> retired;
    void *callers = nullptr;       // optiml_set_workspace's, used instead while set
    size_t callers_bytes = 0;
};
std::mutex g_scratch_mutex;
DeviceScratch g_scratch[64];

// Set while an entry point that must not allocate runs on this thread: workspace() then hands out
// this fixed buffer and refuses anything larger.
struct FixedWorkspace { void *ptr = nullptr; size_t bytes = 0; };
thread_local FixedWorkspace tls_fixed_workspace;
}  // namespace

bool vector_friendly(const Problem &p)
{
    const int64_t chunk = 16 / p.esize(), cchunk = 16 / p.csize();
    auto aligned = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; };
    if (!aligned(p.A) || !aligned(p.B) || !aligned(p.C)) return false;
    if (p.lda % chunk || p.ldb % chunk || p.ldc % cchunk) return false;
    if (p.batch > 1 && (p.strideA % chunk || p.strideB % chunk || p.strideC % cchunk)) return false;
    if (p.bias && (!aligned(p.bias) || (p.batch > 1 && p.strideBias % 4))) return false;
    return true;
}

int select_variant(const Problem &p, double *estimate_us, bool allow_streaming) { return select(p, estimate_us, allow_streaming); }

const Variant *variant_at(int id)
{
    const Table &t = table();
    return id >= 0 && id < (int)t.v.size() ? t.v[id] : nullptr;
}

WorkspaceHead::WorkspaceHead(size_t bytes) { tls_workspace_head = (bytes + 255) & ~size_t(255); }
WorkspaceHead::~WorkspaceHead() { tls_workspace_head = 0; }

int compute_units()
{
    static int cus[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

hipError_t workspace(size_t bytes, void **ptr, hipStream_t stream)
{
    const size_t head = tls_workspace_head;
    bytes += head;
    if (tls_fixed_workspace.ptr) {
        if (tls_fixed_workspace.bytes < bytes) {
            tls_workspace_refused = true;
            return hipErrorOutOfMemory;
        }
        *ptr = static_cast<char *>(tls_fixed_workspace.ptr) + head;
        return hipSuccess;
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    DeviceScratch &s = g_scratch[dev];
    if (s.callers) {
        if (s.callers_bytes < bytes) {
            tls_workspace_refused = true;
            return hipErrorOutOfMemory;
        }
        *ptr = static_cast<char *>(s.callers) + head;
        return hipSuccess;
    }
    if (s.own_bytes < bytes) {
        // not grown when the holder of the head did not size the buffer (a new one would not hold
        // its copy) or while the stream is being captured (an allocation would end the capture, and
        // the graph would keep the address of a buffer that the next growth retires)
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (head || (hipStreamIsCapturing(stream, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone)) {
            tls_workspace_refused = true;
            return hipErrorOutOfMemory;
        }
        // at least double, so that all retired buffers together stay below the live one
        size_t want = bytes > 2 * s.own_bytes ? bytes : 2 * s.own_bytes;
        want = (want + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
        void *fresh = nullptr;
        e = hipMalloc(&fresh, want);
        if (e != hipSuccess) return e;
        if (s.own) s.retired.push_back(s.own);
        s.own = fresh;
        s.own_bytes = want;
    }
    *ptr = static_cast<char *>(s.own) + head;
    return hipSuccess;
}

}  // namespace optiml

using namespace optiml;

extern "C" {

int optiml_gemm_epilogue_strided_batched(int64_t batch, int64_t M, int64_t N, int64_t K,
                                         const void *A, int64_t lda, int64_t strideA,
                                         const void *B, int64_t ldb, int64_t strideB,
                                         const float *bias, int64_t strideBias,
                                         void *C, int64_t ldc, int64_t strideC,
                                         int layout, int dtype, int act, void *stream)
{
    const Problem p = make(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias, C, ldc, strideC,
                           layout, dtype, act);
    const int st = validate(p);
    if (st != OPTIML_OK || is_empty(p)) return st;
    const int id = select(p);
    if (id < 0) return id;
    return run(p, id, stream);
}

int optiml_gemm_epilogue_ex(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B,
                            int64_t ldb, const float *bias, void *C, int64_t ldc, int layout, int dtype,
                            int act, void *stream)
{
    return optiml_gemm_epilogue_strided_batched(1, M, N, K, A, lda, 0, B, ldb, 0, bias, 0, C, ldc, 0, layout,
                                                dtype, act, stream);
}

int optiml_gemm_epilogue(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                         const float *bias, void *C, int64_t ldc, int dtype, int act, void *stream)
{
    return optiml_gemm_epilogue_ex(M, N, K, A, lda, B, ldb, bias, C, ldc, OPTIML_LAYOUT_RR, dtype, act, stream);
}

int optiml_variant_count(void) { return (int)table().v.size(); }

const char *optiml_variant_name(int id)
{
    const Table &t = table();
    return (id >= 0 && id < (int)t.v.size()) ? t.v[id]->name : nullptr;
}

int optiml_select_variant(int64_t batch, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                          int64_t strideA, const void *B, int64_t ldb, int64_t strideB, const float *bias,
                          int64_t strideBias, void *C, int64_t ldc, int64_t strideC, int layout, int dtype,
                          int act)
{
    const Problem p = make(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias, C, ldc, strideC,
                           layout, dtype, act);
    const int st = validate(p);
    if (st != OPTIML_OK) return st;
    return select(p);
}

int optiml_variant_supports(int variant_id, int64_t batch, int64_t M, int64_t N, int64_t K, const void *A,
                            int64_t lda, int64_t strideA, const void *B, int64_t ldb, int64_t strideB,
                            const float *bias, int64_t strideBias, void *C, int64_t ldc, int64_t strideC,
                            int layout, int dtype, int act)
{
    const Problem p = make(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias, C, ldc, strideC,
                           layout, dtype, act);
    const int st = validate(p);
    if (st != OPTIML_OK) return st;
    const Table &t = table();
    if (variant_id < 0 || variant_id >= (int)t.v.size()) return OPTIML_ERR_INVALID_ARG;
    return can_run(t.v[variant_id], p) ? OPTIML_OK : OPTIML_ERR_UNSUPPORTED;
}

int optiml_gemm_epilogue_variant(int64_t batch, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda,
                                 int64_t strideA, const void *B, int64_t ldb, int64_t strideB,
                                 const float *bias, int64_t strideBias, void *C, int64_t ldc, int64_t strideC,
                                 int layout, int dtype, int act, void *stream, int variant_id)
{
    const Problem p = make(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias, C, ldc, strideC,
                           layout, dtype, act);
    const int st = validate(p);
    if (st != OPTIML_OK) return st;
    if (variant_id < 0 || variant_id >= optiml_variant_count()) return OPTIML_ERR_INVALID_ARG;
    if (is_empty(p)) return OPTIML_OK;
    return run(p, variant_id, stream);
}

int optiml_variant_resources(int variant_id, int *num_regs, int *scratch_bytes, int *lds_bytes)
{
    const Table &t = table();
    if (variant_id < 0 || variant_id >= (int)t.v.size()) return OPTIML_ERR_INVALID_ARG;
    hipFuncAttributes attr;
    hipError_t e = hipFuncGetAttributes(&attr, t.v[variant_id]->kernel);
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    if (num_regs) *num_regs = attr.numRegs;
    if (scratch_bytes) *scratch_bytes = (int)attr.localSizeBytes;
    if (lds_bytes) *lds_bytes = (int)attr.sharedSizeBytes;
    return OPTIML_OK;
}

namespace optiml {
// Workgroup b copies the b-th block of 8 x 256 vectors (32 KiB): consecutive workgroups touch
// consecutive memory, which this board rewards (6.4 TB/s against 4.5 TB/s for a grid-stride loop).
typedef unsigned int copy_vec __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void copy_kernel(const copy_vec *__restrict__ src, copy_vec *__restrict__ dst, int64_t n16)
{
    const int64_t base = (int64_t)blockIdx.x * 2048 + threadIdx.x;
    if (base + 7 * 256 < n16) {
        copy_vec v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(src + base + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) __builtin_nontemporal_store(v[u], dst + base + u * 256);
    } else {
        for (int u = 0; u < 8; ++u)
            if (base + u * 256 < n16) dst[base + u * 256] = src[base + u * 256];
    }
}
}  // namespace optiml

int optiml_copy_bytes(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (nbytes < 0 || nbytes % 16 != 0) return OPTIML_ERR_INVALID_ARG;
    if (nbytes == 0) return OPTIML_OK;
    if (!dst || !src || (reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
        return OPTIML_ERR_INVALID_ARG;
    const int64_t n16 = nbytes / 16;
    const int64_t blocks = (n16 + 2047) / 2048;
    if (blocks > 0x7fffffffLL) return OPTIML_ERR_INVALID_ARG;
    hipLaunchKernelGGL(optiml::copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const optiml::copy_vec *>(src), static_cast<optiml::copy_vec *>(dst), n16);
    hipError_t e = hipGetLastError();
    return status_of(e);
}

int optiml_elementwise(int64_t n, const float *x, float *y, int op, void *stream)
{
    if (n < 0 || (op != OPTIML_EW_RELU && op != OPTIML_EW_SIGMOID)) return OPTIML_ERR_INVALID_ARG;
    if (n == 0) return OPTIML_OK;
    if (!x || !y) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_elementwise(n, x, y, op, static_cast<hipStream_t>(stream));
    return status_of(e);
}

int optiml_reduce(int64_t n, const float *x, const float *y, int op, float *out, void *stream)
{
    if (n < 0 || (op != OPTIML_RED_SUM && op != OPTIML_RED_DOT && op != OPTIML_RED_MSE) || !out)
        return OPTIML_ERR_INVALID_ARG;
    if (n > 0 && (!x || (op != OPTIML_RED_SUM && !y))) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_reduce(n, x, y, op, out, static_cast<hipStream_t>(stream));
    return status_of(e);
}

int optiml_cross_entropy(int64_t N, int64_t C, const float *logits, int64_t ld, const int32_t *labels, float *loss,
                         void *stream)
{
    if (N < 0 || C < 1 || ld < C || !loss) return OPTIML_ERR_INVALID_ARG;
    if (N > 0 && (!logits || !labels)) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_cross_entropy(N, C, logits, ld, labels, loss, static_cast<hipStream_t>(stream));
    return status_of(e);
}

int optiml_layernorm(int64_t rows, int64_t len, const float *x, float *y, float eps, void *stream)
{
    if (rows < 0 || len < 0 || !(eps >= 0.0f)) return OPTIML_ERR_INVALID_ARG;
    if (rows == 0 || len == 0) return OPTIML_OK;
    if (!x || !y) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_layernorm(rows, len, x, y, eps, static_cast<hipStream_t>(stream));
    return status_of(e);
}

int optiml_transpose(int64_t rows, int64_t cols, const void *src, int64_t ld_src, void *dst, int64_t ld_dst, int elem_bytes,
                     void *stream)
{
    if (rows < 0 || cols < 0 || (elem_bytes != 2 && elem_bytes != 4) || ld_src < cols || ld_dst < rows)
        return OPTIML_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return OPTIML_OK;
    if (!src || !dst) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_transpose(rows, cols, src, ld_src, dst, ld_dst, elem_bytes, static_cast<hipStream_t>(stream));
    return status_of(e);
}

namespace {
int gemm_cross_entropy(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                       const float *bias, const int32_t *labels, float *loss, float *row_loss, int layout, int dtype,
                       void *stream)
{
    if (!enum_ok(layout, dtype, 0) || is_8bit(dtype)) return OPTIML_ERR_INVALID_ARG;
    if (M < 0 || N < 1 || K < 0 || lda < 0 || ldb < 0) return OPTIML_ERR_INVALID_ARG;
    {
        // operand spans below 2^47 elements, as in validate()
        constexpr int64_t kMaxSpan = int64_t(1) << 47;
        const bool ac = (layout & 2) != 0, bc = (layout & 1) != 0;
        const __int128 a_span = (__int128)((ac ? K : M) > 0 ? (ac ? K : M) - 1 : 0) * lda + (ac ? M : K);
        const __int128 b_span = (__int128)((bc ? N : K) > 0 ? (bc ? N : K) - 1 : 0) * ldb + (bc ? K : N);
        if (a_span >= kMaxSpan || b_span >= kMaxSpan) return OPTIML_ERR_INVALID_ARG;
    }
    Problem p{};
    p.batch = 1; p.M = M; p.N = N; p.K = K;
    p.A = A; p.lda = lda; p.B = B; p.ldb = ldb; p.bias = bias;
    p.layout = layout; p.dtype = dtype; p.act = ACT_NONE;
    if (M > 0) {
        if (!labels) return OPTIML_ERR_INVALID_ARG;
        if (K > 0) {
            if (!A || !B) return OPTIML_ERR_INVALID_ARG;
            if (lda < (p.a_col() ? M : K) || ldb < (p.b_col() ? K : N)) return OPTIML_ERR_INVALID_ARG;
        }
    }
    return status_of(optiml::launch_linear_ce(p, labels, loss, row_loss, static_cast<hipStream_t>(stream)));
}
}  // namespace

int optiml_gemm_cross_entropy(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                              const float *bias, const int32_t *labels, float *loss, int layout, int dtype, void *stream)
{
    if (!loss) return OPTIML_ERR_INVALID_ARG;
    return gemm_cross_entropy(M, N, K, A, lda, B, ldb, bias, labels, loss, nullptr, layout, dtype, stream);
}

int optiml_gemm_cross_entropy_rows(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                                   const float *bias, const int32_t *labels, float *row_loss, float *loss, int layout,
                                   int dtype, void *stream)
{
    if (!row_loss && M > 0) return OPTIML_ERR_INVALID_ARG;
    return gemm_cross_entropy(M, N, K, A, lda, B, ldb, bias, labels, loss, row_loss, layout, dtype, stream);
}

namespace {
// shared argument checks of the contraction + LayerNorm entry points; fills p
int gemm_layernorm_problem(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                           const float *bias, void *Y, int64_t ldy, int layout, int dtype, Problem &p)
{
    if (!enum_ok(layout, dtype, 0) || is_8bit(dtype)) return OPTIML_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || lda < 0 || ldb < 0 || ldy < N) return OPTIML_ERR_INVALID_ARG;
    p = Problem{};
    p.batch = 1; p.M = M; p.N = N; p.K = K;
    p.A = A; p.lda = lda; p.B = B; p.ldb = ldb; p.bias = bias; p.C = Y; p.ldc = ldy;
    p.layout = layout; p.dtype = dtype; p.act = ACT_NONE;
    return validate(p);
}
}  // namespace

int optiml_gemm_layernorm(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                          const float *bias, void *Y, int64_t ldy, float eps, int layout, int dtype, void *stream)
{
    if (!(eps >= 0.0f)) return OPTIML_ERR_INVALID_ARG;
    Problem p;
    const int st = gemm_layernorm_problem(M, N, K, A, lda, B, ldb, bias, Y, ldy, layout, dtype, p);
    if (st != OPTIML_OK || M == 0 || N == 0) return st;
    return status_of(optiml::launch_linear_ln(p, (double)eps, static_cast<hipStream_t>(stream)));
}

int optiml_gemm_layernorm_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                               const float *bias, void *Y, int64_t ldy, int layout, int dtype)
{
    Problem p;
    const int st = gemm_layernorm_problem(M, N, K, A, lda, B, ldb, bias, Y, ldy, layout, dtype, p);
    if (st != OPTIML_OK) return st;
    return optiml::linear_ln_path(p);
}

int optiml_gemm_cross_entropy_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                                   const float *bias, int layout, int dtype)
{
    if (!enum_ok(layout, dtype, 0) || is_8bit(dtype) || M < 0 || N < 1 || K < 0 || lda < 0 || ldb < 0)
        return OPTIML_ERR_INVALID_ARG;
    Problem p{};
    p.batch = 1; p.M = M; p.N = N; p.K = K;
    p.A = A; p.lda = lda; p.B = B; p.ldb = ldb; p.bias = bias;
    p.layout = layout; p.dtype = dtype; p.act = ACT_NONE;
    return optiml::linear_ce_path(p);
}

int optiml_mhsa(int64_t batch, int64_t N, int64_t d_model, int64_t heads, const void *Q, const void *K, const void *V,
                void *O, int dtype, void *stream)
{
    if (batch < 0 || N < 0 || d_model < 1 || heads < 1 || d_model % heads != 0) return OPTIML_ERR_INVALID_ARG;
    if (dtype != OPTIML_F32 && dtype != OPTIML_BF16 && dtype != OPTIML_F16) return OPTIML_ERR_INVALID_ARG;
    if (batch == 0 || N == 0) return OPTIML_OK;
    if (!Q || !K || !V || !O) return OPTIML_ERR_INVALID_ARG;
    const int path = optiml::mhsa_path(d_model, heads, dtype, Q, K, V, O);
    if (path < 0) return OPTIML_ERR_UNSUPPORTED;
    hipError_t e = optiml::launch_mhsa(batch, N, d_model, heads, Q, K, V, O, dtype, path, static_cast<hipStream_t>(stream));
    return status_of(e);
}

namespace {
std::mutex g_static_mutex;
void *g_static_ptr[64] = {};

// device address of this GPU's copy of `scratch` (looked up once per device, with it current)
hipError_t static_scratch(void **ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *q = nullptr;
        e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!q) return hipErrorInvalidSymbol;
        g_static_ptr[dev] = q;
    }
    *ptr = g_static_ptr[dev];
    return hipSuccess;
}

struct FixedWorkspaceScope {
    FixedWorkspaceScope(void *p, size_t bytes) { tls_fixed_workspace.ptr = p; tls_fixed_workspace.bytes = bytes; }
    ~FixedWorkspaceScope() { tls_fixed_workspace = FixedWorkspace(); }
};
}  // namespace

int optiml_gemm_epilogue_noalloc(int64_t batch, int64_t M, int64_t N, int64_t K,
                                 const void *A, int64_t lda, int64_t strideA,
                                 const void *B, int64_t ldb, int64_t strideB,
                                 const float *bias, int64_t strideBias,
                                 void *C, int64_t ldc, int64_t strideC,
                                 int layout, int dtype, int act, void *stream)
{
    const Problem p = make(batch, M, N, K, A, lda, strideA, B, ldb, strideB, bias, strideBias, C, ldc, strideC,
                           layout, dtype, act);
    const int st = validate(p);
    if (st != OPTIML_OK || is_empty(p)) return st;
    void *fixed = nullptr;
    const hipError_t e = static_scratch(&fixed);
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    const int id = select(p);
    if (id < 0) return id;
    // while this lives, workspace() hands out the static array and refuses what does not fit
    const FixedWorkspaceScope scope(fixed, OPTIML_NOALLOC_SCRATCH_BYTES);
    return run(p, id, stream);
}

int optiml_set_workspace(void *ptr, int64_t bytes)
{
    if (bytes < 0 || (ptr == nullptr) != (bytes == 0) || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return OPTIML_ERR_INVALID_ARG;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess && (dev < 0 || dev >= 64)) e = hipErrorInvalidDevice;
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    g_scratch[dev].callers = ptr;
    g_scratch[dev].callers_bytes = (size_t)bytes;
    return OPTIML_OK;
}

static int mx_validate(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
                       int64_t ldb, const void *scaleB, int64_t lds_b, void *C, int64_t ldc, int dtype, int act)
{
    if (!is_8bit(dtype) || act < 0 || act > 3 || M < 0 || N < 0 || K < 0 || K % 32 != 0) return OPTIML_ERR_INVALID_ARG;
    if (lda < 0 || ldb < 0 || ldc < 0 || lds_a < 0 || lds_b < 0 || (dtype == DT_F4 && ((lda & 1) || (ldb & 1))) ||
        (is_f6(dtype) && ((lda & 3) || (ldb & 3)))) return OPTIML_ERR_INVALID_ARG;
    constexpr int64_t kMaxSpan = int64_t(1) << 47;
    if (M >= kMaxSpan / (lda + 1) || N >= kMaxSpan / (ldb + 1) || M >= kMaxSpan / (ldc + 1)) return OPTIML_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return OPTIML_OK;
    if (!C || ldc < N) return OPTIML_ERR_INVALID_ARG;
    if (K > 0 && (!A || !B || !scaleA || !scaleB || lda < K || ldb < K || lds_a < K / 32 || lds_b < K / 32)) return OPTIML_ERR_INVALID_ARG;
    return OPTIML_OK;
}

int optiml_gemm_epilogue_mx(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
                            int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc, int dtype, int act,
                            void *stream)
{
    const int st = mx_validate(M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, C, ldc, dtype, act);
    if (st != OPTIML_OK || M == 0 || N == 0) return st;
    return status_of(optiml::launch_mx(dtype, M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc, act,
                                       static_cast<hipStream_t>(stream)));
}

int optiml_gemm_epilogue_mx_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a,
                                 const void *B, int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc,
                                 int dtype)
{
    const int st = mx_validate(M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, C, ldc, dtype, 0);
    if (st != OPTIML_OK) return st;
    return optiml::mx_path(dtype, M, N, K, A, lda, scaleA, lds_a, B, ldb, scaleB, lds_b, bias, C, ldc);
}

void optiml_set_wait_limit(int64_t clocks) { optiml::set_wait_limit((long long)clocks); }

int64_t optiml_workspace_bytes(void)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return (int64_t)(g_scratch[dev].callers ? g_scratch[dev].callers_bytes : g_scratch[dev].own_bytes);
}

const char *optiml_status_string(int status)
{
    switch (status) {
    case OPTIML_OK: return "ok";
    case OPTIML_ERR_INVALID_ARG: return "invalid argument";
    case OPTIML_ERR_UNSUPPORTED: return "variant does not support these arguments, or the workspace is too small and may not grow";
    case OPTIML_ERR_HIP: return "HIP runtime error (see optiml_last_hip_error)";
    default: return "unknown status";
    }
}

int optiml_last_hip_error(void) { return tls_last_hip_error; }

}  // extern "C"

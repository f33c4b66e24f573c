// C-ABI entry points: argument validation (host integers only, before any GPU
// call), variant selection, launch.  See include/optiml.h for the contract.
#include "../../include/optiml.h"
#include "common.hpp"

#include <mutex>
#include <vector>

namespace optiml {

namespace {

thread_local int tls_last_hip_error = 0;

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
    }
};

const Table &table()
{
    static const Table t;
    return t;
}

bool enum_ok(int layout, int dtype, int act)
{
    return layout >= 0 && layout <= 3 && dtype >= DT_F32 && dtype <= DT_F8 && act >= 0 && act <= 3;
}

// OPTIML_OK when the arguments describe a valid problem (possibly an empty one).
int validate(const Problem &p)
{
    if (!enum_ok(p.layout, p.dtype, p.act)) return OPTIML_ERR_INVALID_ARG;
    if (p.batch < 0 || p.M < 0 || p.N < 0 || p.K < 0) return OPTIML_ERR_INVALID_ARG;
    if (p.strideA < 0 || p.strideB < 0 || p.strideBias < 0 || p.strideC < 0) return OPTIML_ERR_INVALID_ARG;
    if (p.lda < 0 || p.ldb < 0 || p.ldc < 0) return OPTIML_ERR_INVALID_ARG;
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

// The streaming kernels re-read B once per 16 rows of A.  For more than 16 rows that is worth it
// while the re-reads (from L2, about 8 TB/s measured at 1024^3) take less time than an MFMA tile
// kernel needs when its 128x128 tiles cover only part of the chip (140 TFLOP/s when every CU has
// a tile).  Measured: 256^3 8 us against 37 us, 1024^3 29-37 us against more than 60 us,
// 256 x 2048 x 2048 32 us against 250 us; from 2048^3 on the tile kernel wins.
bool streaming_beats_tiles(const Problem &p)
{
    if (p.dtype != DT_F32 || p.layout != 0) return false;
    const double blocks16 = (double)((p.M + 15) / 16), batch = (double)p.batch;
    const double t_stream = batch * blocks16 * (double)p.K * (double)p.N * 4.0 / 8e12;
    const double tm = (double)((p.M + 127) / 128), tn = (double)((p.N + 127) / 128);
    const double tiles = tm * tn * batch;
    const double share = tiles < 256.0 ? tiles / 256.0 : 1.0;
    const double t_tiles = 2.0 * tiles * 128.0 * 128.0 * (double)p.K / (140e12 * share);   // whole tiles are computed
    return t_stream < t_tiles;
}

// The same question for 16-bit storage and up to 128 rows.  The 256 x 256 ring tiles waste most of
// their rows there and, for one row of tiles, use N/256 CUs; the streaming kernel reads B once
// per 16 rows, the blocks of rows running side by side and sharing much of B through the caches.
// Calibrated on 16..64 x 16384 x 16384 (86, 121, 210 us streamed against 270 us) and
// 16 x 32768 x 4096 (47 us against 80 us).
bool streaming16_beats_tiles(const Problem &p)
{
    if (p.dtype == DT_F32 || p.layout != 0 || p.M > 128) return false;
    const double rb = (double)((p.M + 15) / 16), batch = (double)p.batch;
    const double t_stream = batch * (double)p.K * (double)p.N * 2.0 / 5.8e12 * (0.55 + 0.45 * rb);
    const double tiles = (double)((p.M + 255) / 256) * (double)((p.N + 255) / 256) * batch;
    const double rounds = (double)(int64_t)((tiles + 255.0) / 256.0);
    const double t_tiles = rounds * 2.0 * 65536.0 * (double)p.K / 7e12;
    return t_stream < t_tiles;
}

// Preference order: the streaming split-K kernels for at most 16 rows, and for small fp32
// problems of more rows (without the non-temporal hint: B is meant to stay in L2); then the MFMA
// tile kernels - one that declares a measured preference for the shape, else in table order
// (direct-to-LDS kernels before staged ones) the first whose grid gives every CU a workgroup,
// else the one with most workgroups; then the fallback.
int select(const Problem &p)
{
    const Table &t = table();
    constexpr int64_t kComputeUnits = 256;
    if (p.K > 0 && vector_friendly(p)) {
        if (p.M <= 16)
            for (int i = t.first_skinny; i < t.first_tile; ++i)
                if (can_run(t.v[i], p)) return i;
        if (streaming_beats_tiles(p) && t.first_skinny + 1 < t.first_tile && can_run(t.v[t.first_skinny + 1], p))
            return t.first_skinny + 1;
        // column-major B, up to 32 rows, and one row of ring tiles would not fill the chip: two passes
        // over B still beat it (measured at 16 x 16384 x 16384: fp32 225 against 920 us, bf16 112
        // against 235, E4M3 57 against 157)
        if (p.layout == 1 && p.M <= 32 && (p.N + 127) / 128 * p.batch < 2 * kComputeUnits)
            for (int i = t.first_skinny + kNumSkinnyVariants + kNumSkinny16Variants; i < t.first_tile; ++i)
                if (can_run(t.v[i], p)) return i;
        if (streaming16_beats_tiles(p))
            for (int i = t.first_skinny + kNumSkinnyVariants; i < t.first_tile; ++i)
                if (can_run(t.v[i], p)) return i;
        for (int i = t.first_tile; i < (int)t.v.size(); ++i)
            if (t.v[i]->prefers && t.v[i]->prefers(p) && can_run(t.v[i], p)) return i;
        int best = -1;
        int64_t best_blocks = -1;
        for (int i = t.first_tile; i < (int)t.v.size(); ++i) {
            if (!can_run(t.v[i], p)) continue;
            const int64_t blocks = ((p.M + t.v[i]->bm - 1) / t.v[i]->bm) * ((p.N + t.v[i]->bn - 1) / t.v[i]->bn) * p.batch;
            if (blocks >= kComputeUnits) return i;
            if (blocks > best_blocks) { best = i; best_blocks = blocks; }
        }
        if (best >= 0) return best;
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
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
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
    return p;
}

struct DeviceScratch { void *ptr = nullptr; size_t bytes = 0; };
std::mutex g_scratch_mutex;
DeviceScratch g_scratch[64];

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

hipError_t workspace(size_t bytes, void **ptr)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    DeviceScratch &s = g_scratch[dev];
    if (s.bytes < bytes) {
        if (s.ptr) {
            e = hipFree(s.ptr);      // waits for work that may still read the old buffer
            s.ptr = nullptr; s.bytes = 0;
            if (e != hipSuccess) return e;
        }
        const size_t want = (bytes + (size_t(1) << 20) - 1) & ~((size_t(1) << 20) - 1);
        e = hipMalloc(&s.ptr, want);
        if (e != hipSuccess) { s.ptr = nullptr; return e; }
        s.bytes = want;
    }
    *ptr = s.ptr;
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
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_elementwise(int64_t n, const float *x, float *y, int op, void *stream)
{
    if (n < 0 || (op != OPTIML_EW_RELU && op != OPTIML_EW_SIGMOID)) return OPTIML_ERR_INVALID_ARG;
    if (n == 0) return OPTIML_OK;
    if (!x || !y) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_elementwise(n, x, y, op, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_reduce(int64_t n, const float *x, const float *y, int op, float *out, void *stream)
{
    if (n < 0 || (op != OPTIML_RED_SUM && op != OPTIML_RED_DOT && op != OPTIML_RED_MSE) || !out)
        return OPTIML_ERR_INVALID_ARG;
    if (n > 0 && (!x || (op != OPTIML_RED_SUM && !y))) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_reduce(n, x, y, op, out, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_cross_entropy(int64_t N, int64_t C, const float *logits, int64_t ld, const int32_t *labels, float *loss,
                         void *stream)
{
    if (N < 0 || C < 1 || ld < C || !loss) return OPTIML_ERR_INVALID_ARG;
    if (N > 0 && (!logits || !labels)) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_cross_entropy(N, C, logits, ld, labels, loss, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_layernorm(int64_t rows, int64_t len, const float *x, float *y, float eps, void *stream)
{
    if (rows < 0 || len < 0 || !(eps >= 0.0f)) return OPTIML_ERR_INVALID_ARG;
    if (rows == 0 || len == 0) return OPTIML_OK;
    if (!x || !y) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_layernorm(rows, len, x, y, eps, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_transpose(int64_t rows, int64_t cols, const void *src, int64_t ld_src, void *dst, int64_t ld_dst, int elem_bytes,
                     void *stream)
{
    if (rows < 0 || cols < 0 || (elem_bytes != 2 && elem_bytes != 4) || ld_src < cols || ld_dst < rows)
        return OPTIML_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return OPTIML_OK;
    if (!src || !dst) return OPTIML_ERR_INVALID_ARG;
    hipError_t e = optiml::launch_transpose(rows, cols, src, ld_src, dst, ld_dst, elem_bytes, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_gemm_cross_entropy(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                              const float *bias, const int32_t *labels, float *loss, int layout, int dtype, void *stream)
{
    if (!enum_ok(layout, dtype, 0) || dtype == DT_F8) return OPTIML_ERR_INVALID_ARG;
    if (M < 0 || N < 1 || K < 0 || lda < 0 || ldb < 0 || !loss) return OPTIML_ERR_INVALID_ARG;
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
    hipError_t e = optiml::launch_linear_ce(p, labels, loss, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

int optiml_gemm_cross_entropy_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                                   const float *bias, int layout, int dtype)
{
    if (!enum_ok(layout, dtype, 0) || dtype == DT_F8 || M < 0 || N < 1 || K < 0 || lda < 0 || ldb < 0)
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
    if (e != hipSuccess) {
        tls_last_hip_error = (int)e;
        return OPTIML_ERR_HIP;
    }
    return OPTIML_OK;
}

const char *optiml_status_string(int status)
{
    switch (status) {
    case OPTIML_OK: return "ok";
    case OPTIML_ERR_INVALID_ARG: return "invalid argument";
    case OPTIML_ERR_UNSUPPORTED: return "variant does not support these arguments";
    case OPTIML_ERR_HIP: return "HIP runtime error (see optiml_last_hip_error)";
    default: return "unknown status";
    }
}

int optiml_last_hip_error(void) { return tls_last_hip_error; }

}  // extern "C"

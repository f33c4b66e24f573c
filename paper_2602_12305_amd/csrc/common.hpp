// Shared host/device declarations of the library: the problem descriptor that
// every kernel launcher receives and the variant table entry.
#pragma once
#include <cmath>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace optiml {

// DT_F8: A, B in OCP E4M3, C in bf16; DT_BF8: the same with OCP E5M2 operands.  DT_F4: A, B in OCP E2M1, two values to a byte along k (the even k in the
// low half), C in bf16; inside the library such a problem is described in BYTES of k: K, lda, ldb and the operand
// strides are halved on entry, an "element" of A or B is a byte holding two values.
// DT_F6 / DT_BF6: A, B in OCP E2M3 / E3M2, stored densely (element i of an array in bits 6 i .. 6 i + 5 of its
// little-endian bit stream; leading dimensions and strides in elements, multiples of 4), C in bf16.  The matrix-pipe
// kernel sees such operands in SLOT form (kernel_f6.hip): a copy in the workspace with every 32 elements (24 bytes) in
// a 32-byte slot, i.e. one byte per element position, which is what K, lda, ldb count there.
enum : int { DT_F32 = 0, DT_BF16 = 1, DT_F16 = 2, DT_F8 = 3, DT_F4 = 4, DT_BF8 = 5, DT_F6 = 6, DT_BF6 = 7 };
constexpr bool is_f8(int dt) { return dt == DT_F8 || dt == DT_BF8; }                   // one 8-bit value per byte
constexpr bool is_f6(int dt) { return dt == DT_F6 || dt == DT_BF6; }
constexpr bool is_8bit(int dt) { return is_f8(dt) || is_f6(dt) || dt == DT_F4; }        // one byte per stored element of A and B
enum : int { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU_TANH = 2, ACT_SILU = 3 };

// C = act(A.B + bias) for `batch` problems; leading dimensions and strides in elements.
struct Problem {
    int64_t batch, M, N, K;
    const void *A; int64_t lda, strideA;
    const void *B; int64_t ldb, strideB;
    const float *bias; int64_t strideBias;
    void *C; int64_t ldc, strideC;
    int layout;   // bit 0: B column-major, bit 1: A column-major
    int dtype, act;
    // the bias is indexed by the ROW of C instead of the column: how a column-major C is served
    // (C^T = B^T A^T is a row-major problem whose bias runs down the rows)
    bool bias_row = false;
    int pre_status = 0;     // a status the construction of the problem found (an OPTIML_ERR_* for validate() to return)
    bool a_col() const { return (layout & 2) != 0; }
    bool b_col() const { return (layout & 1) != 0; }
    int esize() const { return dtype == DT_F32 ? 4 : is_8bit(dtype) ? 1 : 2; }   // bytes per element of A and B
    int csize() const { return dtype == DT_F32 ? 4 : 2; }                        // ... of C
};

// Kernel family of a variant: what the dispatcher's cost model is keyed on (with the tile shape).
enum : int { FAM_NONE = 0, FAM_RING16, FAM_RING8, FAM_RING8_K64, FAM_RINGP, FAM_RINGF, FAM_DIRECT, FAM_TILE16, FAM_TILEF };
// What the dispatcher uses a streaming variant for (at most one variant per role and storage type):
//   DEFAULT  the entry tuned on 16 rows x 16384 x 16384;  ROWS  more than one block of 16 rows;
//   UNSPLIT  a few blocks of rows over a long K, eight waves and no split along k;
//   NARROW   half the columns per workgroup, for problems that would otherwise launch too few workgroups
//            (and, 16-bit, for a short K); REGS  the register-only kernel (8-bit operands over a short K);
//   SMALL    a B of a few MiB under up to 16 blocks of rows: eight waves deep in k, half the columns.
enum : int { ROLE_NONE = 0, ROLE_STREAM_DEFAULT, ROLE_STREAM_ROWS, ROLE_STREAM_UNSPLIT, ROLE_STREAM_NARROW, ROLE_STREAM_REGS,
             ROLE_STREAM_SMALL };

struct Variant {
    const char *name;
    bool (*supports)(const Problem &);
    hipError_t (*launch)(const Problem &, hipStream_t);
    int bm, bn;   // C block computed by one workgroup (0, 0 where that does not apply)
    const void *kernel;   // host handle of the variant's main kernel, for hipFuncGetAttributes
    // optional: true for problems on which this variant was measured faster than the ones
    // before it in the table; the dispatcher asks it of variants it has no time estimate for
    bool (*prefers)(const Problem &) = nullptr;
    bool row_bias = false;   // handles Problem::bias_row
    // optional: the variant's own estimate of its time on p in microseconds (the dispatcher compares
    // it with its estimates for the other kernels)
    double (*estimate_us)(const Problem &) = nullptr;
    int family = FAM_NONE;   // cost-model key of the tile kernels
    int role = ROLE_NONE;    // streaming kernels: what the dispatcher picks this entry for
};

// The dispatcher's choice for p: index into the variant table (or a negative OPTIML_ERR_*) and,
// if asked, the time it expects in microseconds.  allow_streaming = false leaves out the kernels
// that take a second buffer in the workspace.
int select_variant(const Problem &p, double *estimate_us, bool allow_streaming = true);
const Variant *variant_at(int id);

// every pointer 16-byte aligned, every ld / batch stride a whole number of 16-byte chunks
bool vector_friendly(const Problem &p);

// number of compute units of the current device (256 if the query fails)
int compute_units();

// Parts along k for a streaming kernel whose grid is `blocks` column blocks (times row blocks and
// batches) of `block_bytes` of B each: the count with the smallest estimated time.  The estimate:
// the chip moves 6.7 TB/s and one CU at most 36 GB/s; the workgroups are dealt to the CUs in
// turn, so with p = ceil(workgroups / CUs) the CUs that hold p - 1 run dry first and the rest
// finish at the CUs' own rate; a split costs a second launch and its partial sums (`out_bytes`
// per part, written and read).  (16 x 16000 x 16000: two parts 153 us, three 176 us; 130 column
// blocks: one part 233 us, four 223 us.)  A larger count has to be 3 % better to be taken.
inline int64_t stream_split(int64_t blocks, double block_bytes, int64_t by_k, double out_bytes)
{
    const double cus = (double)compute_units(), cu_rate = 36e3, hbm = 6.7e6;       // bytes per microsecond
    double best = 1e30;
    int64_t best_s = 1;
    for (int64_t s = 1; s <= by_k && s <= 64; ++s) {
        const double w = block_bytes / (double)s, wgs = (double)(blocks * s);
        const double p = std::ceil(wgs / cus), n_hi = wgs - (p - 1.0) * cus;
        const double active = wgs < cus ? wgs : cus;
        const double r1 = cu_rate < hbm / active ? cu_rate : hbm / active, r2 = cu_rate < hbm / n_hi ? cu_rate : hbm / n_hi;
        double t = (p - 1.0) * w / r1 + w / r2;
        if (s > 1) t += 5.0 + 2.0 * (double)s * out_bytes / 5e6;
        if (t < best * 0.97) { best = t; best_s = s; }
    }
    return best_s;
}


// per-device scratch (split-K partial sums, reduction partials, the row-major copy of a
// column-major A): the caller's buffer if one was set, else the library's own, which is replaced
// by a larger one on demand (the old one stays allocated) unless `stream` is being captured.
// When the buffer is too small and may not grow, the error is reported to the caller of the
// entry point as OPTIML_ERR_UNSUPPORTED.
hipError_t workspace(size_t bytes, void **ptr, hipStream_t stream);
// While one of these lives, workspace() on this thread hands out the memory behind the first
// `bytes` of the buffer: a launcher that keeps a copy of an operand there can call kernels that
// ask for scratch of their own.  It must have sized the buffer for both beforehand (one
// workspace(bytes + the callee's need) call): growing the buffer would drop the copy.
struct WorkspaceHead {
    explicit WorkspaceHead(size_t bytes);
    ~WorkspaceHead();
    WorkspaceHead(const WorkspaceHead &) = delete;
    WorkspaceHead &operator=(const WorkspaceHead &) = delete;
};

// streaming siblings (kernel_streams.hip); arguments already validated
hipError_t launch_elementwise(int64_t n, const float *x, float *y, int op, hipStream_t stream);
hipError_t launch_reduce(int64_t n, const float *x, const float *y, int op, float *out, hipStream_t stream);
// row-wise siblings (kernel_rows.hip)
hipError_t launch_cross_entropy(int64_t N, int64_t C, const float *z, int64_t ld, const int *labels, float *loss,
                                hipStream_t stream);
hipError_t launch_layernorm(int64_t rows, int64_t len, const float *x, float *y, float eps, hipStream_t stream);
void set_wait_limit(long long clocks);
// kernel_mx.hip: the contraction on block-scaled E2M1, E4M3, E5M2, E2M3 or E3M2 operands (dtype; K, lda, ldb in elements; scales one E8M0 byte per
// 32 elements of k, pitches lds_a, lds_b in bytes)
int mx_path(int dtype, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B, int64_t ldb,
            const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc);
hipError_t launch_mx(int dtype, int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
                     int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc, int act, hipStream_t stream);
// kernel_f6.hip: 6-bit operands.  Slot form of `batch` dense matrices of `rows` x K 6-bit elements (pitch ld, batch
// stride `stride`, both in elements and multiples of 4): dst[b][r][Kp bytes], Kp = f6_slot_k(K), every k-tile of 64
// elements (48 bytes) as four 16-byte chunks: bytes 0-15 of the first block of 32, bytes 0-15 of the second, bytes
// 16-23 of the first + 8 zero bytes, bytes 16-23 of the second + 8 zero bytes; elements at or beyond K are zero.
int64_t f6_slot_k(int64_t K);
hipError_t launch_f6_slots(const void *src, int64_t ld, int64_t stride, int64_t batch, int64_t rows, int64_t K, void *dst, hipStream_t s);
// kernel_linear_ln.hip: unrounded fp32 products of p.batch 16-bit problems by the ring kernel (used to split a
// contraction along k); `pairs` needs 2 * 4 * ceil(N / 256) * M floats per batch
bool unrounded_products_supported(const Problem &p);
hipError_t launch_unrounded_products(const Problem &p, float *Z, int64_t ldz, float *pairs, hipStream_t stream);

// attention (kernel_attention.hip): which kernel would serve (0 flash, 1 fallback, -1 none), launch
int mhsa_path(int64_t d_model, int64_t heads, int dtype, const void *Q, const void *K, const void *V, const void *O);
hipError_t launch_mhsa(int64_t batch, int64_t N, int64_t d_model, int64_t heads, const void *Q, const void *K,
                       const void *V, void *O, int dtype, int path, hipStream_t stream);

// contraction + cross-entropy (kernel_linear_ce.hip): which path would serve (0 ring kernel with the
// log-sum-exp epilogue, 1 row-per-workgroup fallback), launch; p.C, ldc, act and batch are ignored
int linear_ce_path(const Problem &p);
// loss: the mean over rows (may be null); row_loss: every row's loss (may be null)
hipError_t launch_linear_ce(const Problem &p, const int *labels, float *loss, float *row_loss, hipStream_t stream);

// contraction + LayerNorm over the rows of the product (kernel_linear_ln.hip): which path would serve (0 ring
// kernel with the statistics epilogue, 1 row-per-workgroup fallback), launch; p.C, p.ldc are Y; act and batch
// are ignored
int linear_ln_path(const Problem &p);
hipError_t launch_linear_ln(const Problem &p, double eps, hipStream_t stream);

// transpose (kernel_transpose.hip), arguments already validated
hipError_t launch_transpose(int64_t rows, int64_t cols, const void *src, int64_t ld_src, void *dst, int64_t ld_dst, int esize,
                            hipStream_t s);

// tables defined next to the kernels they launch
const Variant *generic_variants();         extern const int kNumGenericVariants;
const Variant *skinny_variants();          constexpr int kNumSkinnyVariants = 24;
const Variant *skinny16_variants();        constexpr int kNumSkinny16Variants = 28;
const Variant *skinny_rc_variants();       constexpr int kNumSkinnyRcVariants = 24;
// the MFMA tile kernels are compiled per (dtype, layout) and gathered by tile_variants.hip
const Variant *tile_variants();            extern const int kNumTileVariants;
const Variant *transpose_variants();       extern const int kNumTransposeVariants;
const Variant *pad_variants();             extern const int kNumPadVariants;      // kernel_pad.hip
const Variant *tail_variants();            constexpr int kNumTailVariants = 1;    // kernel_tail.hip
const Variant *f6_variants();              constexpr int kNumF6Variants = 16;      // kernel_f6.hip
constexpr int kTilesPerUnit = 3;           // tile shapes per (dtype, layout) unit
constexpr int kDirectPerUnit = 4;          // direct-to-LDS kernels per (16-bit dtype, B layout)
constexpr int kRingPerUnit = 5;            // ring-of-stages 16-bit kernels per B layout (three one-tile, one persistent, one 128 x 256)
constexpr int kRingF32PerUnit = 3;         // ring-of-stages fp32 kernels per B layout

}  // namespace optiml

/*
 * optiml.h - C-ABI of the MI355X (gfx950) library for the fused dense contraction
 *
 *                     C = act(A . B + bias)
 *
 * The operation is the Matrix Multiplication task of the OptiML paper (Table 4,
 * task 2: A is M x K, B is K x N, C = A x B is M x N, 32-bit floats), in the
 * row-major convention of its matmul case study (appendix "One-task kernel
 * snapshots": C[row*N+col] = sum_k A[row*K+k] * B[k*N+col], any M and N as in
 * the guarded listing there), with a fused epilogue: a length-N bias added to
 * every row of the product, then an elementwise activation - ReLU max(0,x)
 * (Table 4, task 10), SiLU x*sigmoid(x) with sigmoid(x) = 1/(1+exp(-x))
 * (Table 4, task 1), or the tanh form of GELU
 * 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))).  Bias, SiLU, GELU, 16-bit
 * storage, column-major operands and batching extend the paper's task; they
 * take their standard definitions.
 *
 * Conventions for every entry point
 *   Pointers   A, B, bias, C are DEVICE pointers owned by the caller.  The library
 *              keeps no reference after the call's work has run, never frees or
 *              reallocates them.  C must not overlap A, B or bias (not checked).
 *   Units      lda, ldb, ldc and all strides are in ELEMENTS of the operand's type.
 *   Layouts    C is row-major, C[i,j] at C[i*ldc + j], ldc >= N, unless the layout code has
 *              OPTIML_LAYOUT_C_COLUMN_MAJOR added: then C[i,j] at C[j*ldc + i], ldc >= M,
 *              and a batch's C spans (N-1)*ldc + M elements.  (Served as the transposed
 *              problem C^T = B^T A^T with the bias running down the rows; the streaming
 *              and persistent kernels do not take that form, the others do.)
 *              A row-major: A[i,k] at A[i*lda + k], lda >= K;
 *              A column-major: A[i,k] at A[k*lda + i], lda >= M.
 *              B row-major: B[k,j] at B[k*ldb + j], ldb >= N;
 *              B column-major: B[k,j] at B[j*ldb + k], ldb >= K.
 *   dtype      OPTIML_F32: A, B, C are float.  OPTIML_BF16: A, B, C are bfloat16,
 *              OPTIML_F16: IEEE binary16 (16-bit storage either way); products are
 *              accumulated in fp32, bias is added and the activation applied in fp32,
 *              and C is rounded once, to nearest even (binary16: beyond 65504 to
 *              infinity).  OPTIML_F8E4M3: A and B are 8-bit OCP E4M3 (1 sign, 4 exponent
 *              bits with bias 7, 3 fraction bits; no infinities, largest finite 448), one
 *              byte per element, decoded exactly; C is bfloat16; no scale factors.
 *              OPTIML_F8E5M2: the same with 8-bit OCP E5M2 operands (1 sign, 5 exponent bits
 *              with bias 15, 2 fraction bits: the upper byte of binary16, with its
 *              infinities and NaNs; largest finite 57344).
 *              OPTIML_F4E2M1: A and B are 4-bit OCP E2M1 (1 sign, 2 exponent bits with bias
 *              1, 1 fraction bit: 0, 0.5, 1, 1.5, 2, 3, 4, 6 and their negatives), two
 *              elements per byte along k, the element with the even k in the low half;
 *              decoded exactly, no scale factors; C is bfloat16.  K, lda, ldb and the
 *              operand strides still count ELEMENTS and must be even
 *              (OPTIML_ERR_INVALID_ARG otherwise), and k must be contiguous in both
 *              operands: A row-major and B column-major, i.e. OPTIML_LAYOUT_RC, or its
 *              mirror image with a column-major C; other layouts return
 *              OPTIML_ERR_UNSUPPORTED.
 *              OPTIML_F6E2M3, OPTIML_F6E3M2: A and B are 6-bit OCP E2M3 (1 sign, 2 exponent
 *              bits with bias 1, 3 fraction bits; largest 7.5) or E3M2 (3 exponent bits with
 *              bias 3, 2 fraction bits; largest 28); no infinities, no NaN.  Stored densely:
 *              an operand is one little-endian bit stream in which element e (row * ld + k,
 *              or k * ld + column, as for the other types) occupies bits 6 e .. 6 e + 5, so
 *              four elements fill three bytes.  lda, ldb and the operand strides count
 *              ELEMENTS and must be multiples of 4 (every row starts on a byte;
 *              OPTIML_ERR_INVALID_ARG otherwise).  Decoded exactly, no scale factors; C is
 *              bfloat16.  Every layout is accepted; the matrix-pipe kernel serves
 *              OPTIML_LAYOUT_RC (and its mirror image with a column-major C) with K a
 *              multiple of 4, after copying both operands into the workspace with every 32
 *              elements in 32 bytes ((M + N) * max(320, K rounded up to 64) bytes per batch).
 *              Up to 128 rows (OPTIML_LAYOUT_RC, K and the pitches multiples of 32) the dense form is
 *              streamed as it lies in memory, without a copy.
 *              bias is always float; NULL means no bias.  The
 *              contraction entry points take all eight; the other entry points say
 *              which they take.
 *   Shapes     M, N, K, batch >= 0.  M == 0, N == 0 or batch == 0: nothing is
 *              written, OPTIML_OK.  K == 0: C = act(bias) (the empty sum is 0).
 *   Stream     `stream` is a hipStream_t passed as void* (NULL = the default
 *              stream).  Calls only enqueue work and never synchronise with the
 *              host; buffers must stay valid until the stream has run the work.
 *   Alignment  Any alignment and any ld is accepted.  The fast kernels need
 *              16-byte aligned bases and ld (and batch strides) that keep rows
 *              16-byte aligned; other arguments are first copied into that form in
 *              the workspace when the problem is large enough to pay for it, else
 *              served by a guarded element-wise kernel, with the same results to
 *              rounding either way.
 *   Results    Repeating a call with the same arguments gives bitwise the same C
 *              (no floating-point atomics; split-K partial sums are combined in a
 *              fixed order).
 *   Workspace  Split-K kernels (the streaming kernels for few rows, and the split of a tiled
 *              contraction's nearly empty last round of tiles) keep partial sums, and the fast paths for a column-major
 *              A, for 8-bit operands whose k is not contiguous and for unaligned or
 *              odd-sized problems keep copies of operands (batch x M x K, batch x N x K
 *              elements; the last also a temporary C), in one per-device buffer.
 *              By default the library allocates it on first need and, when a call needs
 *              more, allocates a larger one (at least double) and keeps the old one
 *              allocated until the process ends, because enqueued work and HIP graphs
 *              captured earlier may still hold its address; these are the only
 *              allocations the library makes.  It is never grown while `stream` is being
 *              captured: such a call returns OPTIML_ERR_UNSUPPORTED, so run every call
 *              of a graph once before capturing it (or hand over a buffer).  With
 *              optiml_set_workspace the caller supplies the buffer instead; the library
 *              then never allocates, and a call that needs more than the buffer holds
 *              returns OPTIML_ERR_UNSUPPORTED.  Calls that use the workspace are ordered
 *              by the stream they are enqueued on; two streams must not run such calls
 *              on one device at the same time (not checked).
 *   Errors     The return value is an optiml_status_t; nothing is thrown or
 *              aborted.  OPTIML_ERR_INVALID_ARG: a NULL A/B (with K > 0) or C, a
 *              negative size or stride, an ld shorter than the row it spans, an
 *              unknown enum - decided on the host BEFORE any GPU call, so it is
 *              reportable on a machine without a GPU.  OPTIML_ERR_UNSUPPORTED: a
 *              forced variant cannot run this shape / alignment, or the workspace is
 *              too small and may not grow (see Workspace).  OPTIML_ERR_HIP:
 *              the runtime refused a launch; optiml_last_hip_error() has the code.
 */
#ifndef OPTIML_H
#define OPTIML_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    OPTIML_F32 = 0, OPTIML_BF16 = 1, OPTIML_F16 = 2, OPTIML_F8E4M3 = 3, OPTIML_F4E2M1 = 4, OPTIML_F8E5M2 = 5,
    OPTIML_F6E2M3 = 6, OPTIML_F6E3M2 = 7
} optiml_dtype_t;

typedef enum {
    OPTIML_ACT_NONE = 0,
    OPTIML_ACT_RELU = 1,
    OPTIML_ACT_GELU_TANH = 2,
    OPTIML_ACT_SILU = 3
} optiml_act_t;

/* bit 0: B is column-major; bit 1: A is column-major */
typedef enum {
    OPTIML_LAYOUT_RR = 0,
    OPTIML_LAYOUT_RC = 1,
    OPTIML_LAYOUT_CR = 2,
    OPTIML_LAYOUT_CC = 3,
    OPTIML_LAYOUT_C_COLUMN_MAJOR = 4   /* added to any of the four: C[i,j] at C[j*ldc + i] */
} optiml_layout_t;

typedef enum {
    OPTIML_OK = 0,
    OPTIML_ERR_INVALID_ARG = -1,
    OPTIML_ERR_UNSUPPORTED = -2,
    OPTIML_ERR_HIP = -3
} optiml_status_t;

/*
 * C[M x N] = act(A[M x K] . B[K x N] + bias[N]), every operand row-major:
 * the paper's task 2 with the fused epilogue described above.
 */
int optiml_gemm_epilogue(int64_t M, int64_t N, int64_t K,
                         const void *A, int64_t lda,
                         const void *B, int64_t ldb,
                         const float *bias,
                         void *C, int64_t ldc,
                         int dtype, int act, void *stream);

/* The same with a storage layout for A and B (optiml_layout_t). */
int optiml_gemm_epilogue_ex(int64_t M, int64_t N, int64_t K,
                            const void *A, int64_t lda,
                            const void *B, int64_t ldb,
                            const float *bias,
                            void *C, int64_t ldc,
                            int layout, int dtype, int act, void *stream);

/*
 * `batch` independent problems of one shape: problem b uses A + b*strideA,
 * B + b*strideB, bias + b*strideBias and C + b*strideC.  strideA or strideB may
 * be 0 (operand shared by all problems); strideBias 0 shares one bias vector.
 * strideC must be >= (M-1)*ldc + N when batch > 1 (outputs may not overlap).
 */
int optiml_gemm_epilogue_strided_batched(int64_t batch, int64_t M, int64_t N, int64_t K,
                                         const void *A, int64_t lda, int64_t strideA,
                                         const void *B, int64_t ldb, int64_t strideB,
                                         const float *bias, int64_t strideBias,
                                         void *C, int64_t ldc, int64_t strideC,
                                         int layout, int dtype, int act, void *stream);

/*
 * Kernel variants (tile shapes, split factors, the guarded fallback), for the
 * profiler-driven sweep in the spirit of the paper's search over kernel
 * candidates (section 3.2: each candidate is checked, timed and profiled).
 * Ids are 0 .. optiml_variant_count()-1 and stable within one build.
 */
int optiml_variant_count(void);

/* Name of a variant; static storage, never freed by the caller; NULL if id is out of range. */
const char *optiml_variant_name(int variant_id);

/*
 * Which variant the dispatcher would run for these arguments (>= 0), or a negative
 * optiml_status_t.  Pure host logic: touches no GPU, reads no device memory; the
 * pointers are used for their alignment only.
 */
int optiml_select_variant(int64_t batch, int64_t M, int64_t N, int64_t K,
                          const void *A, int64_t lda, int64_t strideA,
                          const void *B, int64_t ldb, int64_t strideB,
                          const float *bias, int64_t strideBias,
                          void *C, int64_t ldc, int64_t strideC,
                          int layout, int dtype, int act);

/* OPTIML_OK if `variant_id` can run these arguments, OPTIML_ERR_UNSUPPORTED if not. Host only. */
int optiml_variant_supports(int variant_id,
                            int64_t batch, int64_t M, int64_t N, int64_t K,
                            const void *A, int64_t lda, int64_t strideA,
                            const void *B, int64_t ldb, int64_t strideB,
                            const float *bias, int64_t strideBias,
                            void *C, int64_t ldc, int64_t strideC,
                            int layout, int dtype, int act);

/* optiml_gemm_epilogue_strided_batched through one chosen variant. */
int optiml_gemm_epilogue_variant(int64_t batch, int64_t M, int64_t N, int64_t K,
                                 const void *A, int64_t lda, int64_t strideA,
                                 const void *B, int64_t ldb, int64_t strideB,
                                 const float *bias, int64_t strideBias,
                                 void *C, int64_t ldc, int64_t strideC,
                                 int layout, int dtype, int act, void *stream,
                                 int variant_id);

/*
 * Registers per lane, scratch (spill) bytes per lane and static LDS bytes per workgroup of a
 * variant's main kernel, as the HIP runtime reports them: the inputs of the register and
 * spill guardrails in the paper's reward (section 3.2, "Guardrails").  Any out pointer may be
 * NULL.  Needs a GPU (the code object is loaded); OPTIML_ERR_HIP if the query fails.
 */
int optiml_variant_resources(int variant_id, int *num_regs, int *scratch_bytes, int *lds_bytes);

/*
 * Plain device-to-device copy of nbytes (a multiple of 16; both pointers 16-byte aligned) with
 * 128-bit loads and stores: the Matrix Copy task of the paper's Table 4 (task 13).  It exists
 * to measure the HBM bandwidth a streaming kernel can reach on this GPU and to calibrate the
 * profiler's byte counters against a transfer of known size.  Enqueued on `stream`.
 */
int optiml_copy_bytes(void *dst, const void *src, int64_t nbytes, void *stream);

/*
 * Matrix-pipe rate probe, the companion of optiml_copy_bytes for the other roof: one workgroup per
 * compute unit runs `iters` rounds of sixteen 32x32x16 matrix instructions (OPTIML_BF16 or
 * OPTIML_F16) with no global-memory traffic in the loop, so the time of a launch gives the rate
 * the board sustains on operands of that value distribution (the paper's reward prices kernels in
 * percent of a speed of light, section 3.2; on a power-limited board that light is slower for
 * operands whose bits toggle more, and slower again when the operands have to come from LDS).
 * lds_reads: 0 - operand fragments are read once and stay in registers; 8, 12 or 16 - every
 * k-step's operands are read from LDS (filled once from `operands`), that many 16-byte-per-lane
 * reads per sixteen instructions: the ratio of a 128x128, 128x64 or 64x64 wave tile.
 * `operands`: DEVICE pointer, 16-byte aligned, at least 65536 bytes per compute unit of 16-bit
 * values, read only; `sink`: DEVICE pointer to at least 256 floats per compute unit, overwritten
 * (checksums, so that the loop is not optimised away).  *flops (HOST pointer, may be NULL) receives
 * the number of floating-point operations the launch performs.  Enqueued on `stream`.
 * OPTIML_ERR_INVALID_ARG: iters < 0, another dtype or lds_reads, a NULL or misaligned pointer,
 * buffers too small.  The size checks need the device's compute-unit count and so a GPU.
 */
int optiml_mfma_probe(const void *operands, int64_t operand_bytes, float *sink, int64_t sink_floats,
                      int64_t iters, int dtype, int lds_reads, double *flops, void *stream);

/*
 * Bandwidth-bound siblings of the contraction from the paper's Table 4, on float arrays of n
 * elements (DEVICE pointers, any alignment; 16-byte aligned arrays take the 128-bit path).
 *
 * optiml_elementwise: y[i] = max(0, x[i]) (OPTIML_EW_RELU, task 10) or 1 / (1 + exp(-x[i]))
 * (OPTIML_EW_SIGMOID, task 1; about 3 ulp).  y may be x itself; any other overlap is undefined.
 * n == 0 writes nothing.
 *
 * optiml_reduce: *out (one float, DEVICE pointer) = sum_i x[i] (OPTIML_RED_SUM, task 14; y is
 * ignored and may be NULL), sum_i x[i] * y[i] (OPTIML_RED_DOT, task 15) or
 * (1/n) sum_i (x[i] - y[i])^2 (OPTIML_RED_MSE, task 7; 0 for n == 0).  Terms are formed and added
 * in fp64 in a fixed order and the total is rounded once to float, so the result is the exact
 * value's nearest float up to fp64 rounding of the sum, and repeating a call gives the same bits.
 * Uses the per-device workspace (see Workspace above) and enqueues two kernels.  n == 0 writes 0.
 *
 * OPTIML_ERR_INVALID_ARG (before any GPU call): n < 0, unknown op, NULL out, NULL x (or y where it
 * is read) with n > 0.
 */
typedef enum { OPTIML_EW_RELU = 0, OPTIML_EW_SIGMOID = 1 } optiml_ew_t;
typedef enum { OPTIML_RED_SUM = 0, OPTIML_RED_DOT = 1, OPTIML_RED_MSE = 2 } optiml_red_t;
int optiml_elementwise(int64_t n, const float *x, float *y, int op, void *stream);
int optiml_reduce(int64_t n, const float *x, const float *y, int op, float *out, void *stream);

/*
 * Row-wise siblings from the paper's Table 4, float arrays, DEVICE pointers.
 *
 * optiml_cross_entropy (task 17): *loss (one float, DEVICE pointer) = (1/N) sum_j
 * ( log(sum_k exp(z[j][k])) - z[j][labels[j]] ) for logits z[j][k] at logits[j*ld + k], ld >= C,
 * and labels[j] in [0, C) (32-bit integers).  Evaluated in the stable form with the row maximum;
 * exponentials and the running sum in fp32 (about 2e-7 of absolute error on a row's loss), row
 * losses and their mean in fp64 in a fixed order, one rounding to float.  A label outside
 * [0, C) makes the result NaN.  N == 0 writes 0.  Uses the per-device workspace; two kernels.
 *
 * optiml_layernorm (task 4): every row of `len` values (one sample with all its features) is
 * replaced by (x - mean) / sqrt(var + eps), mean and biased variance (divide by len) of that
 * row; no scale or shift (the task names none; eps is the caller's, 1e-5 in common use).
 * x[r*len + i] -> y[r*len + i]; y may be x itself.  Statistics and the normalisation are
 * evaluated in fp64 and rounded once to float.  Rows longer than 32768 (8192 unless x, y are
 * 16-byte aligned and len % 4 == 0) use the per-device workspace.  Aligned rows of up to 4 Mi
 * values are still read once: the workgroups that share a row exchange their partial sums
 * through the workspace inside one kernel and wait for each other, for at most the number of
 * shader clocks set by optiml_set_wait_limit (default 2^22, about 2 ms; 0 = no waiting); a
 * workgroup whose wait runs out leaves its part of the row to a second kernel, which reads x
 * again, so the result does not depend on the limit.  Other long rows take two kernels per
 * group of rows of about 256 MiB (x is then read twice).  rows == 0 or len == 0 writes nothing.
 *
 * OPTIML_ERR_INVALID_ARG (before any GPU call): negative sizes, C < 1, ld < C, NULL loss, NULL
 * logits / labels / x / y with work to do, eps negative or NaN.
 */
int optiml_cross_entropy(int64_t N, int64_t C, const float *logits, int64_t ld, const int32_t *labels, float *loss,
                         void *stream);
int optiml_layernorm(int64_t rows, int64_t len, const float *x, float *y, float eps, void *stream);
/* Process-wide bound, in shader clocks, of the wait described under optiml_layernorm; negative values count as 0. */
void optiml_set_wait_limit(int64_t clocks);

/*
 * Transpose (the paper's Table 4, task 8): dst[j * ld_dst + i] = src[i * ld_src + j] for a
 * rows x cols row-major matrix of elements of elem_bytes (2 or 4) bytes; dst is cols x rows.
 * DEVICE pointers, src and dst must not overlap; pitches in elements, ld_src >= cols,
 * ld_dst >= rows; padding is neither read nor written.  Bytes are moved, never interpreted.
 * 16-byte aligned bases with extents and pitches that are whole 16-byte chunks take the
 * vectorised kernel, everything else an element-wise one.  rows == 0 or cols == 0 writes nothing.
 * OPTIML_ERR_INVALID_ARG (before any GPU call): negative sizes, elem_bytes not 2 or 4, a pitch
 * shorter than its row, NULL src or dst with work to do.
 */
int optiml_transpose(int64_t rows, int64_t cols, const void *src, int64_t ld_src, void *dst, int64_t ld_dst, int elem_bytes,
                     void *stream);

/*
 * The contraction feeding the cross-entropy (the paper's Table 4, task 2 into task 17), fused:
 *     *loss = (1/M) sum_i [ log sum_j exp(z[i][j]) - z[i][labels[i]] ],   z = A.B + bias
 * for M rows (samples) and N classes, with A, B, bias, layouts, leading dimensions and dtype
 * exactly as in optiml_gemm_epilogue_ex (no activation, no batch, none of the 8-, 6- and 4-bit types); labels are M 32-bit integers in
 * [0, N), loss one float; all DEVICE pointers.  The logits are not written anywhere: products
 * are accumulated in fp32, each row's maximum and sum of exponentials are formed in fp32 from
 * the unrounded fp32 logits, the row losses and their mean in fp64 in a fixed order, rounded
 * once to float; repeating a call gives the same bits.  A row-major with a shape the ring kernels
 * take (16-byte aligned operands; 16-bit storage: K a multiple of 8 and at least 128, N a
 * multiple of 8 for a row-major B; fp32: K a multiple of 4 and at least 64, N a multiple of 4 for
 * a row-major B) runs on the matrix pipe; everything else runs a one-workgroup-per-row fp32
 * kernel.  Uses the per-device workspace (8 bytes per row and 64 columns, 32 for fp32); three
 * kernels.  A label outside [0, N) makes the result NaN; M == 0 writes 0.
 * optiml_gemm_cross_entropy_path says which kernel a call would use (0 matrix pipe, 1 fallback;
 * host only).
 *
 * OPTIML_ERR_INVALID_ARG (before any GPU call): M < 0, N < 1, K < 0, unknown layout or dtype, NULL
 * loss, NULL labels with M > 0, NULL A or B with M > 0 and K > 0, an ld shorter than the row it
 * spans.
 */
int optiml_gemm_cross_entropy(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                              const float *bias, const int32_t *labels, float *loss, int layout, int dtype, void *stream);
int optiml_gemm_cross_entropy_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                                   const float *bias, int layout, int dtype);

/*
 * The same fused operation with the per-row losses handed out (the "no reduction" form of task 17):
 * row_loss[i] = log sum_j exp(z[i][j]) - z[i][labels[i]] for every row i, M floats, DEVICE pointer,
 * each rounded once from the fp64 value the mean is formed from (NaN for a label outside [0, N)).
 * loss (one float, DEVICE pointer) receives the mean as above and may be NULL.  Same kernels, same
 * workspace use, same argument rules; OPTIML_ERR_INVALID_ARG also for a NULL row_loss with M > 0.
 */
int optiml_gemm_cross_entropy_rows(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                                   const float *bias, const int32_t *labels, float *row_loss, float *loss, int layout,
                                   int dtype, void *stream);

/*
 * The contraction followed by LayerNorm over each row of the product (the paper's Table 4, task 2
 * into task 4), fused:
 *     Y[i][j] = (z[i][j] - mean_i) / sqrt(var_i + eps),   z = A.B + bias,
 * mean_i and var_i the mean and the biased variance (divide by N) of the N entries of row i; no
 * scale or shift, eps is the caller's (as in optiml_layernorm).  A, B, bias, layouts, leading
 * dimensions and dtype exactly as in optiml_gemm_epilogue_ex (no activation, no batch, not
 * OPTIML_F8E4M3); Y is M x N row-major with pitch ldy >= N in the storage type of dtype; all DEVICE
 * pointers.  The product is accumulated in fp32 and is NOT rounded to the storage type before it
 * is normalised: the contraction's epilogue keeps z in fp32 (in Y itself for OPTIML_F32, in the
 * per-device workspace - 4 bytes per entry - for 16-bit storage) and takes, in registers, each
 * row's mean and sum of squared deviations per wave-wide slice of columns; a second kernel merges
 * them per row (fp64, fixed order), subtracts, scales and rounds once.  Repeating a call gives the
 * same bits.  A row-major with a shape the ring kernels take (as for optiml_gemm_cross_entropy;
 * fp32 also needs Y 16-byte aligned and ldy % 4 == 0) runs on the matrix pipe, everything else a
 * one-workgroup-per-row fp32 kernel; optiml_gemm_layernorm_path says which (0 matrix pipe,
 * 1 fallback; host only).  K == 0: LayerNorm of the bias in every row.  M == 0 or N == 0 writes
 * nothing.  OPTIML_ERR_INVALID_ARG (before any GPU call): negative sizes, ldy < N, unknown layout
 * or dtype, eps negative or NaN, NULL Y, NULL A or B with K > 0, an ld shorter than the row it spans.
 */
int optiml_gemm_layernorm(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                          const float *bias, void *Y, int64_t ldy, float eps, int layout, int dtype, void *stream);
int optiml_gemm_layernorm_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *B, int64_t ldb,
                               const float *bias, void *Y, int64_t ldy, int layout, int dtype);

/*
 * Multi-head self-attention (the paper's Table 4, task 6): for Q, K, V of shape [batch][N][d_model]
 * (row-major, contiguous, DEVICE pointers; float for OPTIML_F32, 16-bit for OPTIML_BF16 / OPTIML_F16) and
 * `heads` heads of width d_k = d_model / heads,
 *     O[b][:, i d_k : (i+1) d_k] = softmax( Q_i K_i^T / sqrt(d_k) ) V_i      (softmax over the keys of a query)
 * with no projections and no mask.  O has the shape and type of Q and must not overlap the inputs.
 * 16-bit storage with d_k = 64 or 128 and 16-byte aligned pointers runs on the matrix pipe (16-bit
 * products, fp32 accumulation, fp32 online softmax whose weights are rounded to the storage type before the
 * second product, one rounding of O); everything else with d_k <= 256 runs a one-wave-per-query
 * fp32 kernel; d_k > 256 is OPTIML_ERR_UNSUPPORTED.  batch == 0 or N == 0 writes nothing.
 * OPTIML_ERR_INVALID_ARG (before any GPU call): negative sizes, d_model < 1, heads < 1, d_model not
 * a multiple of heads, unknown dtype, a NULL pointer with work to do.
 */
int optiml_mhsa(int64_t batch, int64_t N, int64_t d_model, int64_t heads, const void *Q, const void *K, const void *V,
                void *O, int dtype, void *stream);

/*
 * The contraction on block-scaled ("microscaling") operands, the form the scaled matrix instructions of this
 * hardware take (one of the low-precision formats of the hot path's breadth row; the paper names none):
 *     C[i][j] = act( sum_k (sA[i][k/32] a[i][k]) (sB[j][k/32] b[j][k]) + bias[j] )
 * A is M x K row-major and B is N x K (column-major B: k contiguous in both).  dtype is OPTIML_F4E2M1 (two elements to
 * a byte along k as in the plain contraction; lda, ldb >= K count elements and must be even), OPTIML_F8E4M3 or
 * OPTIML_F8E5M2 (one element to a byte), OPTIML_F6E2M3 or OPTIML_F6E3M2 (dense 6-bit codes as in the plain
 * contraction; lda, ldb multiples of 4).  Every 32 consecutive k of a row of A (a column of B) share one scale, a
 * power of two stored as an OCP E8M0 byte: scaleA[i * lds_a + k / 32], scaleB[j * lds_b + k / 32], value
 * 2^(byte - 127), byte 255 = NaN; lds_a, lds_b >= K / 32 count bytes.  K must be a multiple of 32.  C is M x N
 * bfloat16, row-major, ldc >= N; bias (N floats) may be NULL; act as above.  All pointers DEVICE.  Products are exact;
 * block sums are scaled exactly and accumulated in fp32 (E2M1: the block sums themselves are exact too); C is
 * rounded once.  M == 0 or N == 0 writes nothing; K == 0 gives act(bias).
 * optiml_gemm_epilogue_mx_path: 0 when the call would run on the matrix-pipe tile kernel (K a multiple of 128 for
 * E2M1, of 64 for the 8-bit and 6-bit types; 16-byte aligned operands and rows, except the 6-bit types, which are
 * copied; at least 65536 entries of C; any address and pitch of the scales), 1 for the one-thread-per-entry kernel, or
 * an error; 2 for E2M1 with at most 128 rows (at most 48 when B is larger than 48 MB), at least 1024 columns and K a
 * multiple of 128 (16-byte aligned operands and rows): a streaming kernel that reads operands and scales once, as they lie in memory, and needs no workspace.  The tile kernel keeps a copy of the scales, (M + N) K / 32 bytes for E2M1 and (M + N) K / 16 for the
 * others, in the workspace (see Workspace above), and for the 6-bit types also both operands with every 32 elements
 * in 32 bytes ((M + N) * max(320, K) bytes); the other kernel needs none.
 * OPTIML_ERR_INVALID_ARG (before any GPU call): negative sizes, K % 32 != 0, odd (E2M1) or too small lda / ldb, lda
 * or ldb not a multiple of 4 (6-bit), lds_a
 * or lds_b < K / 32, ldc < N, another dtype, unknown act, a NULL pointer with work to do.
 */
int optiml_gemm_epilogue_mx(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a, const void *B,
                            int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc, int dtype, int act,
                            void *stream);
int optiml_gemm_epilogue_mx_path(int64_t M, int64_t N, int64_t K, const void *A, int64_t lda, const void *scaleA, int64_t lds_a,
                                 const void *B, int64_t ldb, const void *scaleB, int64_t lds_b, const float *bias, void *C, int64_t ldc,
                                 int dtype);

/*
 * Hands the library a workspace for the current device (see Workspace above): `bytes` bytes of
 * DEVICE memory at `ptr`, 256-byte aligned, owned by the caller, which keeps it valid and
 * otherwise untouched until every call that may use it has run and another buffer (or none) has
 * been set.  ptr == NULL with bytes == 0 returns to the library's own buffer.  The split-K
 * partial sums of the contraction need split x batch x 16 ceil(M/16) x N floats (split <= 64;
 * 8 MiB for M = 16, N = K = 16384), the copy paths the operand sizes given above.
 * optiml_workspace_bytes() is the capacity of the buffer in use on the current device (0 before
 * the first allocation).  OPTIML_ERR_INVALID_ARG (before any GPU call): bytes < 0, ptr not
 * 256-byte aligned, exactly one of ptr and bytes zero.
 */
int optiml_set_workspace(void *ptr, int64_t bytes);
int64_t optiml_workspace_bytes(void);

/*
 * optiml_gemm_epilogue_strided_batched for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bitwise the same C; what the kernels need beyond A, B, bias and C (split-K partial
 * sums, operand copies) lives in a static array of OPTIML_NOALLOC_SCRATCH_BYTES in the library's
 * device image - one copy per GPU, held until the process ends - instead of the workspace, so the
 * call never allocates or frees, on the first call or any other, and never touches the buffer of
 * optiml_set_workspace.  A problem whose kernels need more than that returns OPTIML_ERR_UNSUPPORTED
 * and enqueues nothing (the split-K partial sums of M <= 16 fit for every N x split <= 262144; the
 * copy paths for column-major A, 8-bit operands in other layouts and unaligned problems fit while
 * their copies do).  The array keeps the last call's contents; nothing in it has to start at zero.
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (different
 * streams, or graphs replayed concurrently) race; calls ordered on one stream do not.
 */
#define OPTIML_NOALLOC_SCRATCH_BYTES (16u << 20)
int optiml_gemm_epilogue_noalloc(int64_t batch, int64_t M, int64_t N, int64_t K,
                                 const void *A, int64_t lda, int64_t strideA,
                                 const void *B, int64_t ldb, int64_t strideB,
                                 const float *bias, int64_t strideBias,
                                 void *C, int64_t ldc, int64_t strideC,
                                 int layout, int dtype, int act, void *stream);

/* Human-readable text for a status code; static storage. */
const char *optiml_status_string(int status);

/* The hipError_t behind the calling thread's most recent OPTIML_ERR_HIP (0 if none). */
int optiml_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* OPTIML_H */

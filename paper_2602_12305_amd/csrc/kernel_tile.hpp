// MFMA tile kernel for C = act(A.B + bias), fp32 and 16-bit (bf16, fp16) inputs, all four
// operand layouts, single and strided-batched.
//
// The paper's matmul case study arrives at a 16x16 shared-memory tile with one
// output per thread on an A100 (appendix "Final OptiML kernel").  The idea that
// carries over is staging operand tiles on chip for reuse; everything else here
// is shaped by gfx950: 64-lane waves feeding v_mfma_f32_32x32x2_f32 /
// v_mfma_f32_32x32x16_bf16, wave tiles of up to 128x128 held in accumulator
// registers, 128-byte LDS rows with an XOR swizzle, double-buffered LDS, and a
// workgroup order that keeps the tiles sharing an operand panel on one XCD's L2.
//
// LDS format (both operands, both dtypes).  A tile is ROWS x 128 bytes: row r is
// one row of A (an m index) or one column of B (an n index), and holds BK
// consecutive k (32 fp32 or 64 bf16) as eight 16-byte chunks; chunk c of row r
// lives at byte r*128 + ((c ^ ((r >> 1) & 7)) << 4).  The LDS of gfx950 has 64
// four-byte banks (a 128-bit access is served 16 lanes at a time, 256 bytes per
// clock, measured), so a row pair spans all banks once; with the key taken from
// r >> 1, sixteen lanes that touch sixteen consecutive rows at one logical chunk,
// or two rows at eight chunks each, hit every bank exactly once: both the 128-bit
// stores that fill the tile and the 128-bit fragment loads are conflict-free.
//
// Filling a tile.  If k is the operand's contiguous direction in memory (A
// row-major, B column-major) a thread copies 16-byte chunks as they are.  If not
// (A column-major, B row-major) a thread loads a CH x CH block (CH = elements per
// chunk: 4 fp32 or 8 bf16) as CH 128-bit loads along the contiguous direction,
// transposes it in registers, and stores CH chunks.
//
// MFMA operands.  For k-step s a lane reads chunk 2s + lane/32 of row lane%32 of a
// 32-row fragment.  bf16: the 16 bytes are the 8-element operand of one 32x32x16
// MFMA.  fp32: the four floats feed four 32x32x2 MFMAs.  Both operands use the
// same k assignment, so the order of k inside a step is immaterial.  The MFMA
// takes the B fragment as its first operand and the A fragment as its second:
// the accumulator then holds D[n][m] with m = lane%32 and n = 8*(r/4) + 4*(lane/32)
// + r%4 for register r, i.e. four consecutive n per lane, which is what a
// row-major C wants for vector stores.
#pragma once
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace tile {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));

struct Params {
    int64_t M, N, K, batch;
    const char *A; int64_t lda, strideA;     // strides and ld in elements
    const char *B; int64_t ldb, strideB;
    const float *bias; int64_t strideBias;
    char *C; int64_t ldc, strideC;
    int64_t tiles_m, tiles_n;
    int act;
    int bias_row;        // bias[m] instead of bias[n]
};

template <int DT, int BM_, int BN_, int WM_, int WN_, bool A_KC_, bool B_KC_>
struct Cfg {
    static constexpr int dt = DT;
    static constexpr int ES = DT == DT_F32 ? 4 : 2;
    static constexpr int CH = 16 / ES;            // elements per 16-byte chunk
    static constexpr int BK = 128 / ES;           // k extent of one LDS tile
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr bool A_KC = A_KC_, B_KC = B_KC_;
    static constexpr int THREADS = 64 * WM * WN;
    static constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // 32x32 MFMA tiles per wave
    static constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0, "wave tile must be whole MFMA tiles");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "chunks must divide over threads");
};

// ---- global -> registers -> LDS ---------------------------------------------------------------

// Operand tile loader.  ROWS = tile rows (m or n indices), KC = k contiguous in memory.
// `base` points at the operand of this batch; row0 is the tile's first row; extent the
// operand's row count (M or N); ld its leading dimension.
template <int ES, int ROWS, int THREADS, bool KC>
struct Loader {
    static constexpr int CH = 16 / ES;
    static constexpr int BK = 128 / ES;
    static constexpr int CHUNKS = ROWS * 8;
    // copy mode: chunks per thread; transpose mode: CH x CH blocks per thread (possibly a
    // fraction of the threads take one block each)
    static constexpr int PER_THREAD = KC ? CHUNKS / THREADS : (CHUNKS / CH + THREADS - 1) / THREADS;
    static constexpr int BLOCKS = CHUNKS / CH;
    static constexpr int NREG = KC ? PER_THREAD : PER_THREAD * CH;

    uintx4 reg[NREG];

    // Issue the global loads of the k-tile starting at k0.  GUARD: rows/chunks at k >= K read as zero.
    template <bool GUARD>
    __device__ __forceinline__ void load(const char *base, int64_t ld, int64_t row0, int64_t extent, int64_t k0,
                                         int64_t K, int tid)
    {
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                const int id = tid + i * THREADS;
                const int c = id & 7, r = id >> 3;
                int64_t row = row0 + r;
                row = row < extent ? row : extent - 1;           // rows past the edge duplicate the last one
                const int64_t k = k0 + c * CH;
                if (!GUARD || k < K)
                    reg[i] = *reinterpret_cast<const uintx4 *>(base + (row * ld + k) * ES);
                else
                    reg[i] = uintx4{0, 0, 0, 0};
            }
        } else {
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                const int id = tid + i * THREADS;
                const int kc = id & 7, ng = id >> 3;
                if (BLOCKS % THREADS != 0 && id >= BLOCKS) break;
                int64_t col = row0 + ng * CH;
                col = col + CH <= extent ? col : extent - CH;      // extent % CH == 0 and extent >= CH
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int64_t k = k0 + kc * CH + j;
                    if (!GUARD || k < K)
                        reg[i * CH + j] = *reinterpret_cast<const uintx4 *>(base + (k * ld + col) * ES);
                    else
                        reg[i * CH + j] = uintx4{0, 0, 0, 0};
                }
            }
        }
    }

    // Write the held registers into the LDS tile at `lds` (byte address of the tile).
    __device__ __forceinline__ void store(char *lds, int tid)
    {
        if constexpr (KC) {
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                const int id = tid + i * THREADS;
                const int c = id & 7, r = id >> 3;
                *reinterpret_cast<uintx4 *>(lds + r * 128 + ((c ^ ((r >> 1) & 7)) << 4)) = reg[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < PER_THREAD; ++i) {
                const int id = tid + i * THREADS;
                const int kc = id & 7, ng = id >> 3;
                if (BLOCKS % THREADS != 0 && id >= BLOCKS) break;
                uintx4 out[CH];
                if constexpr (ES == 4) {
                    // 4x4 transpose of 32-bit elements: register renaming only
#pragma unroll
                    for (int n = 0; n < 4; ++n)
                        out[n] = uintx4{reg[i * 4 + 0][n], reg[i * 4 + 1][n], reg[i * 4 + 2][n], reg[i * 4 + 3][n]};
                } else {
                    // 8x8 transpose of 16-bit elements: in[k] holds n = 0..7 as four dwords of two;
                    // out[n] dword d packs (in[2d][n], in[2d+1][n])
#pragma unroll
                    for (int n = 0; n < 8; ++n)
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const unsigned lo = reg[i * 8 + 2 * d][n >> 1], hi = reg[i * 8 + 2 * d + 1][n >> 1];
                            out[n][d] = (n & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)   // high halves
                                                : __builtin_amdgcn_perm(hi, lo, 0x05040100u);  // low halves
                        }
                }
#pragma unroll
                for (int n = 0; n < CH; ++n) {
                    const int r = ng * CH + n;
                    *reinterpret_cast<uintx4 *>(lds + r * 128 + ((kc ^ ((r >> 1) & 7)) << 4)) = out[n];
                }
            }
        }
    }
};

// ---- the kernel ---------------------------------------------------------------------------

template <class C>
__global__ __launch_bounds__(C::THREADS) void gemm_tile_kernel(Params p)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int ES = C::ES, BK = C::BK, TM = C::TM, TN = C::TN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % C::WM, wn = wave / C::WM;

    // Workgroup -> tile.  Consecutive workgroup ids go round-robin over the 8 XCDs; undo that so
    // each XCD works on a contiguous range of tiles, then walk tiles in bands of 8 tile rows,
    // column by column, so that the tiles in flight on an XCD share A and B panels in its L2.
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

    const char *A = p.A + batch * p.strideA * ES;
    const char *B = p.B + batch * p.strideB * ES;

    Loader<ES, C::BM, C::THREADS, C::A_KC> la;
    Loader<ES, C::BN, C::THREADS, C::B_KC> lb;

    floatx16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.0f;

    // fp32 only: sums of the current block of k-tiles
    constexpr int FLUSH = 4;
    constexpr bool F32 = C::dt == DT_F32;
    floatx16 part[F32 ? TN : 1][F32 ? TM : 1];

    // per-lane fragment addressing: row lane%32 of a 32-row fragment, chunk (2s + lane/32) ^ ((row >> 1) & 7)
    const int frag_row = lane & 31, half = lane >> 5;
    int frag_off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) frag_off[s] = frag_row * 128 + (((2 * s + half) ^ ((frag_row >> 1) & 7)) << 4);
    const int a_wave = wm * (C::BM / C::WM) * 128, b_wave = wn * (C::BN / C::WN) * 128;

    const int64_t nk = (p.K + BK - 1) / BK;
    auto fetch = [&](int64_t kt) {
        const int64_t k0 = kt * BK;
        if (k0 + BK <= p.K) {
            la.template load<false>(A, p.lda, m0, p.M, k0, p.K, tid);
            lb.template load<false>(B, p.ldb, n0, p.N, k0, p.K, tid);
        } else {
            la.template load<true>(A, p.lda, m0, p.M, k0, p.K, tid);
            lb.template load<true>(B, p.ldb, n0, p.N, k0, p.K, tid);
        }
    };

    if (nk > 0) {
        fetch(0);
        la.store(lds, tid);
        lb.store(lds + C::A_BYTES, tid);
    }
    __syncthreads();

    auto k_tile = [&](int64_t kt) {
        const char *cur = lds + (kt & 1) * C::STAGE_BYTES;
        char *nxt = lds + ((kt + 1) & 1) * C::STAGE_BYTES;
        const bool more = kt + 1 < nk;
        if (more) fetch(kt + 1);

        const char *a_base = cur + a_wave, *b_base = cur + C::A_BYTES + b_wave;
        if constexpr (C::dt != DT_F32) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uintx4 fa[TM], fb[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[i] = *reinterpret_cast<const uintx4 *>(a_base + i * 32 * 128 + frag_off[s]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[j] = *reinterpret_cast<const uintx4 *>(b_base + j * 32 * 128 + frag_off[s]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
                        acc[j][i] = mfma_32x32x16<C::dt>(fb[j], fa[i], acc[j][i]);
            }
        } else {
            // fp32: k-tiles are summed into a second accumulator set that is added to the
            // running sums on the vector ALU every FLUSH k-tiles (128 k) and cleared.  Blocked
            // summation keeps the rounding error of a long k loop near sqrt(K * 128) * 2^-24
            // instead of K * 2^-24 relative to the terms' size; the additions cost about 5 % of
            // a block's MFMA time.
            uintx4 fa[4][TM], fb[4][TN];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    fa[s][i] = *reinterpret_cast<const uintx4 *>(a_base + i * 32 * 128 + frag_off[s]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[s][j] = *reinterpret_cast<const uintx4 *>(b_base + j * 32 * 128 + frag_off[s]);
            }
#pragma unroll
            for (int s = 0; s < 4; ++s)
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
#pragma unroll
                        for (int i = 0; i < TM; ++i)
                            part[j][i] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fb[s][j][e]),
                                                                              __uint_as_float(fa[s][i][e]),
                                                                              part[j][i], 0, 0, 0);
        }

        if (more) {
            la.store(nxt, tid);
            lb.store(nxt + C::A_BYTES, tid);
        }
        __syncthreads();
    };

    if constexpr (F32) {
        for (int64_t kb = 0; kb < nk; kb += FLUSH) {
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) part[j][i][r] = 0.0f;
            const int64_t ke = kb + FLUSH < nk ? kb + FLUSH : nk;
            for (int64_t kt = kb; kt < ke; ++kt) k_tile(kt);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int i = 0; i < TM; ++i) acc[j][i] += part[j][i];
        }
    } else {
        for (int64_t kt = 0; kt < nk; ++kt) k_tile(kt);
    }

    // epilogue: register r of acc[j][i] is Z[m][n], m = mw + 32 i + lane%32,
    // n = nw + 32 j + 8 (r/4) + 4 (lane/32) + r%4
    const int64_t mw = m0 + wm * (C::BM / C::WM), nw = n0 + wn * (C::BN / C::WN);
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    char *Cb = p.C + batch * p.strideC * ES;
    dispatch_act(p.act, [&](auto act_tag) {
    constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int64_t n = nw + 32 * j + 8 * g + 4 * half;
            if (n >= p.N) continue;
            const bool whole = n + 3 < p.N;
            float bj[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (bias && !p.bias_row) {
                if (whole) {
                    const floatx4 v = *reinterpret_cast<const floatx4 *>(bias + n);
                    bj[0] = v[0]; bj[1] = v[1]; bj[2] = v[2]; bj[3] = v[3];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < p.N) bj[e] = bias[n + e];
                }
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int64_t m = mw + 32 * i + frag_row;
                if (m >= p.M) continue;
                const float bi = (bias && p.bias_row) ? bias[m] : 0.0f;
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = apply_act(acc[j][i][4 * g + e] + (bj[e] + bi), ACT);
                char *dst = Cb + (m * p.ldc + n) * ES;
                if constexpr (C::dt == DT_F32) {
                    if (whole) {
                        *reinterpret_cast<floatx4 *>(dst) = floatx4{y[0], y[1], y[2], y[3]};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < p.N) reinterpret_cast<float *>(dst)[e] = y[e];
                    }
                } else {
                    unsigned short h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = to_16<C::dt>(y[e]);
                    if (whole) {
                        *reinterpret_cast<uintx2 *>(dst) =
                            uintx2{(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16)};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < p.N) reinterpret_cast<unsigned short *>(dst)[e] = h[e];
                    }
                }
            }
        }
    });
}

// ---- host side -----------------------------------------------------------------------------

template <class C>
bool supports(const Problem &p)
{
    if (p.dtype != C::dt || p.a_col() == C::A_KC || p.b_col() != C::B_KC) return false;
    if (p.K < 1 || !vector_friendly(p)) return false;
    // the contiguous direction of each operand must be whole 16-byte chunks
    if (C::A_KC ? (p.K % C::CH != 0) : (p.M % C::CH != 0)) return false;
    if (C::B_KC ? (p.K % C::CH != 0) : (p.N % C::CH != 0)) return false;
    const int64_t tiles = ((p.M + C::BM - 1) / C::BM) * ((p.N + C::BN - 1) / C::BN);
    if (tiles <= 0 || p.batch > 0x7fffffffLL / tiles) return false;
    return true;
}

template <class C>
hipError_t launch(const Problem &p, hipStream_t stream)
{
    static bool configured[64] = {};
    auto kernel = gemm_tile_kernel<C>;
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
    q.bias = p.bias; q.strideBias = p.strideBias; q.bias_row = p.bias_row ? 1 : 0;
    q.C = static_cast<char *>(p.C); q.ldc = p.ldc; q.strideC = p.strideC;
    q.tiles_m = (p.M + C::BM - 1) / C::BM;
    q.tiles_n = (p.N + C::BN - 1) / C::BN;
    q.act = p.act;
    const int64_t total = q.tiles_m * q.tiles_n * p.batch;
    hipLaunchKernelGGL(kernel, dim3((unsigned)total), dim3(C::THREADS), C::LDS_BYTES, stream, q);
    return hipGetLastError();
}

}  // namespace tile
}  // namespace optiml

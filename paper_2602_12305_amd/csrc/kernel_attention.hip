// Multi-head self-attention (paper Table 4, task 6):
//     head_i = softmax(Q_i K_i^T / sqrt(d_k)) V_i,  output = Concat(head_1 .. head_h)
// for Q, K, V of shape [batch][N][d_model] (row-major), heads of width d_k = d_model / h, no mask.
//
// Three kernels.
//
// mhsa_pingpong_kernel (bf16 or fp16 storage, d_k = 128, N >= 256): the arithmetic of mhsa_flash_kernel in
// a workgroup of eight waves whose two halves alternate, barrier by barrier, between the matrix
// instructions of one key block and the softmax of the block before; described where it is defined.
//
// mhsa_flash_kernel (bf16 or fp16 storage, d_k = 64 or 128): the two chained contractions on the
// 16-bit matrix pipe with an online softmax between them, never writing the N x N scores anywhere.
// A workgroup of 4 waves owns 128 queries of one (batch, head); a wave owns 32 of them and
// keeps their Q fragments, the running maximum / sum, and the output accumulators in
// registers while the workgroup walks the keys 64 at a time.  The K and V tiles of a key block
// come in by LDS-DMA (no staging registers) into one of two LDS buffers while the arithmetic of
// the block before runs from the other: one barrier per block.  Two workgroups share a compute
// unit, so one's softmax arithmetic overlaps the other's matrix instructions.  Both products are
// computed TRANSPOSED:
//     S^T (keys x queries) = K_blk . Q^T          O^T (d_k x queries) += V_blk^T . P^T
// With v_mfma_f32_32x32x16_bf16 the accumulator lane l then holds column l%32 = one query, so
//   * all 16 registers of a lane's S^T tile are scores of ONE query: its maximum and sum need
//     one exchange with lane l^32 instead of a 32-lane reduction;
//   * every register of a lane's O^T accumulators belongs to that same query: rescaling by
//     exp(m_old - m_new) is a plain multiply;
//   * registers 8s..8s+7 of a lane's P^T tile are exactly the 8 k-slots that lane must supply as
//     the second MFMA operand of k-step s, up to a fixed permutation of the 16 keys of the step
//     (lane half h owns keys 4h..4h+3 and 8+4h..8+4h+3 instead of 8h..8h+7).  A contraction does
//     not care in which order its terms come, so the V^T operand is simply read with the same
//     permutation (two transposing LDS reads at rows 16s+4h and 16s+8+4h) and P never passes
//     through LDS or a shuffle.
// LDS tiles are XOR-swizzled 16-byte chunks (K: chunk ^ row for 256-byte rows, chunk ^ (row/2)
// for 128-byte rows; V: chunk ^ 4(row%4) or ^ 2(row%4)) so that the 128-bit fragment reads and
// the transposing reads spread over the 64 banks.
//
// mhsa_rows_kernel (fp32, bf16 or fp16 storage, any d_k up to 256): one wave per query, a key per
// lane, fp32 arithmetic throughout; the fallback for everything the flash kernel does not take.
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef unsigned int uintx2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) char lds_char;

// One wave-wide LDS-DMA load: lane l copies 16 bytes from base + off(l) to LDS byte lds_addr + 16 l
// (base and lds_addr wave-uniform).  In assembly, so that the kernel keeps its own count of the
// loads in flight (wait_all_loads_and_barrier below) instead of the compiler draining them
// before unrelated LDS reads.
__device__ __forceinline__ void dma_load16(const char *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(off), "s"(base), "s"(lds_addr)
                 : "m0");
}

__device__ __forceinline__ const char *scalar_ptr(const char *q)
{
    const uint64_t v = reinterpret_cast<uint64_t>(q);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

// s_waitcnt vmcnt(0) lgkmcnt(0), then the workgroup barrier, without the fences of
// __syncthreads(): every load of this wave has landed and its LDS reads have returned.
__device__ __forceinline__ void wait_all_loads_and_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

struct AttnParams {
    int64_t batch, N, d_model, heads;
    const char *Q, *K, *V;
    char *O;
    float scale2;        // log2(e) / sqrt(d_k)
};

[[maybe_unused]] constexpr int kBQ = 128, kBK = 64;       // queries per workgroup, keys per step

// The softmax of one key block, shared by the two matrix-pipe kernels.  A lane holds the raw scores of ONE
// query (its 32 of the block's 64 keys; lane l ^ 32 has the others).  The maximum is taken on the raw scores
// (the scale is positive) and the scale log2(e) / sqrt(d_k) and the reference point m are folded into the
// exponent's multiply-add, so a score costs one multiply-add, one exponential, half a conversion, half a
// three-way maximum and half a two-term dot product with (1, 1), which adds the ROUNDED weights to the row
// sum: the very values the second product uses, so numerator and denominator agree.
//
// The reference point only has to keep the exponents in range, so it follows the maximum lazily: it moves
// when the block's maximum is more than kLazy (in base-2 units) above it, which after the first block is
// rare; until then the weights are at most 2^kLazy and the output accumulators need no rescaling.  The final
// division by the row sum cancels the reference point exactly.
template <int DT> __device__ __forceinline__ float add_pair_16(unsigned int pair, float acc)
{
    typedef __bf16 bf16x2_ __attribute__((ext_vector_type(2), unused));
    typedef _Float16 halfx2_ __attribute__((ext_vector_type(2), unused));
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (DT == DT_F16)
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(halfx2_, pair), halfx2_{(_Float16)1.0f, (_Float16)1.0f}, acc, false);
    else
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_, pair), bf16x2_{(__bf16)1.0f, (__bf16)1.0f}, acc, false);
#else
    return acc;
#endif
}

constexpr float kLazy = 8.0f;            // slack of the exponents' reference point below the running maximum

template <int DT, int TU, class BeforeQuarter>
__device__ __forceinline__ void softmax_block(floatx16 (&acc_s)[2], floatx16 (&acc_o)[TU], uintx4 (&pf)[2][2], float &m,
                                              float &l, float scale2, BeforeQuarter before_quarter)
{
    float bm = acc_s[0][0];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) bm = __builtin_fmaxf(bm, acc_s[t][r]);
    bm = __builtin_fmaxf(bm, __shfl_xor(bm, 32, 64));
    const float cand = bm * scale2;
    const float m_new = cand > m + kLazy ? cand : m;
    const float corr = __builtin_amdgcn_exp2f(m - m_new);
    l *= corr;
    m = m_new;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            before_quarter(2 * t + s);
            unsigned int w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                w[i] = pack2_16<DT>(__builtin_amdgcn_exp2f(__builtin_fmaf(acc_s[t][8 * s + 2 * i], scale2, -m_new)),
                                    __builtin_amdgcn_exp2f(__builtin_fmaf(acc_s[t][8 * s + 2 * i + 1], scale2, -m_new)));
                l = add_pair_16<DT>(w[i], l);
            }
            pf[t][s] = uintx4{w[0], w[1], w[2], w[3]};
        }
    // skip the rescaling of the output accumulators when the reference moved for no query of this wave
    if (__builtin_amdgcn_ballot_w64(corr != 1.0f) != 0) {
#pragma unroll
        for (int u = 0; u < TU; ++u)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[u][r] *= corr;
    }
}

template <int DK, int DT>
__global__ __launch_bounds__(256, 2) void mhsa_flash_kernel(AttnParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int ROWB = DK * 2;                 // bytes per row of a tile
    constexpr int CHUNKS = DK / 8;               // 16-byte chunks per row
    constexpr int KS = DK / 16;                  // k-steps of the first product
    constexpr int TU = DK / 32;                  // 32-wide output tiles of the second product
    constexpr int VKEY = DK == 128 ? 4 : 2;      // V swizzle: chunk ^ VKEY * (row % 4)
    constexpr int TILE = kBK * ROWB;               // bytes of one K (or V) tile
    constexpr int RPL = 1024 / ROWB;               // tile rows one wave-wide load covers
    constexpr int LOADS = kBK / (4 * RPL);         // loads per wave per tile
    __shared__ __attribute__((aligned(1024))) char lds[4 * TILE];     // two buffers of (K tile, V tile)

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;
    const int64_t qblocks = (p.N + kBQ - 1) / kBQ;
    // Workgroups are dealt to the 8 XCDs round-robin by index.  When the (batch, head) pairs split
    // evenly, XCD x takes the pairs = x (mod 8), so that the workgroups sharing one pair's K and V
    // run behind the same L2.
    const int64_t pairs = p.batch * p.heads;
    int64_t qb, bh;
    if (pairs % 8 == 0) {
        const int64_t x = blockIdx.x % 8, j = blockIdx.x / 8;
        bh = x + 8 * (j / qblocks);
        qb = j % qblocks;
    } else {
        qb = blockIdx.x % qblocks;
        bh = blockIdx.x / qblocks;
    }
    const int64_t b = bh / p.heads, head = bh % p.heads;
    const int64_t ldb = p.d_model * 2;                                   // bytes per row of Q, K, V, O
    const char *Qb = p.Q + (b * p.N * p.d_model + head * DK) * 2;
    const char *Kb = p.K + (b * p.N * p.d_model + head * DK) * 2;
    const char *Vb = p.V + (b * p.N * p.d_model + head * DK) * 2;
    char *Ob = p.O + (b * p.N * p.d_model + head * DK) * 2;

    // this lane's query (clamped at the end of the sequence: computed, not stored)
    const int64_t q = qb * kBQ + wave * 32 + col;
    const int64_t qc = q < p.N ? q : p.N - 1;
    uintx4 qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const uintx4 *>(Qb + qc * ldb + (16 * s + 8 * half) * 2);

    floatx16 acc_o[TU];
#pragma unroll
    for (int u = 0; u < TU; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[u][r] = 0.0f;
    float m = -__builtin_inff(), l = 0.0f;

    // Tile loads: wave w's load i fills the 1 KiB of LDS that holds rows RPL (w + 4 i) .. of the
    // tile; a lane's slot there (row, position in the row) takes the chunk the swizzle assigns to
    // it, so the swizzle is applied on the global side.  The swizzle terms depend on row % 16 or
    // less and a load advances the row by a multiple of 16: one chunk offset per lane serves all.
    const int ld_row = RPL * wave + lane / CHUNKS, ld_slot = lane % CHUNKS;
    const uint32_t ld_kc = (DK == 128 ? (ld_slot ^ (ld_row & 15)) : (ld_slot ^ ((ld_row >> 1) & 7))) * 16;
    const uint32_t ld_vc = (ld_slot ^ (VKEY * (ld_row & 3))) * 16;
    const uint32_t ldb32 = (uint32_t)ldb;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>((lds_char *)lds) + wave * 1024);
    uint32_t ld_ro[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) ld_ro[i] = (uint32_t)(ld_row + 4 * RPL * i) * ldb32;
    auto issue = [&](int64_t key0, int buf) {
        const char *kb = scalar_ptr(Kb + key0 * ldb), *vb = scalar_ptr(Vb + key0 * ldb);
        const uint32_t dst = lds0 + buf * 2 * TILE;
        if (key0 + kBK <= p.N) {
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                dma_load16(kb, ld_ro[i] + ld_kc, dst + i * 4096);
                dma_load16(vb, ld_ro[i] + ld_vc, dst + TILE + i * 4096);
            }
        } else {
            const int last = (int)(p.N - key0) - 1;                      // rows past the end re-read the last key
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                const int row = ld_row + 4 * RPL * i;
                const uint32_t ro = (uint32_t)(row < last ? row : last) * ldb32;
                dma_load16(kb, ro + ld_kc, dst + i * 4096);
                dma_load16(vb, ro + ld_vc, dst + TILE + i * 4096);
            }
        }
    };

    // transposing read of V: a 16-lane group g reads rows r0 + (lane%16)/4, columns 16 (g%2) + 4 (lane%4) .. +3
    const int g = lane >> 4, jj = lane & 15;
    const int tr_row = 4 * (g >> 1) + (jj >> 2);          // + 16 s (+ 8 for the second half of the operand)
    const int tr_col = 16 * (g & 1) + 4 * (jj & 3);       // + 32 u

    // one key block from buffer BUF (a compile-time constant: every LDS address below is then a
    // loop-invariant register plus an immediate)
    auto block = [&](int64_t key0, auto bufc) {
        constexpr int BUF = decltype(bufc)::value;
        // this block's tiles have landed for every wave, and every wave is done with the other buffer
        wait_all_loads_and_barrier();
        if (key0 + kBK < p.N) issue(key0 + kBK, BUF ^ 1);                // in flight during the arithmetic below
        lds_char *const kt = (lds_char *)lds + BUF * 2 * TILE;
        lds_char *const vt = kt + TILE;

        // S^T = K_blk . Q^T : two 32-key tiles, their two accumulation chains interleaved
        floatx16 acc_s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_s[t][r] = 0.0f;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int row = 32 * t + col;
                const int c = 2 * s + half;
                const int kc = DK == 128 ? (c ^ (row & 15)) : (c ^ ((row >> 1) & 7));
                const uintx4 kf = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(kt + row * ROWB + kc * 16);
                acc_s[t] = mfma_32x32x16<DT>(kf, qf[s], acc_s[t]);
            }
        // order for the scheduler: K fragment reads run kAhead k-steps ahead of the matrix
        // instructions that consume them, so LDS latency is paid once, not per step
        constexpr int kAhead = KS < 4 ? KS : 4;
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            if (s + kAhead < KS) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }

        // keys past the end of the sequence (last block only) drop out with a score of -inf
        if (key0 + kBK > p.N) {
            const int left = (int)(p.N - key0);
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (32 * t + 8 * (r >> 2) + 4 * half + (r & 3) >= left) acc_s[t][r] = -__builtin_inff();
        }

        uintx4 pf[2][2];
        softmax_block<DT, TU>(acc_s, acc_o, pf, m, l, p.scale2, [](int) {});

        // O^T += V_blk^T . P^T : k-steps of 16 keys, lane half h supplying keys 4h..4h+3 and 8+4h..8+4h+3
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int r0 = 32 * t + 16 * s + tr_row;
#pragma unroll
                for (int u = 0; u < TU; ++u) {
                    const int cb = (32 * u + tr_col) * 2;                 // byte column
                    const int c = cb >> 4, within = cb & 15;
                    const lds_char *a0 = vt + r0 * ROWB + ((c ^ (VKEY * (r0 & 3))) << 4) + within;
                    const lds_char *a1 = vt + (r0 + 8) * ROWB + ((c ^ (VKEY * ((r0 + 8) & 3))) << 4) + within;
                    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4 *)(a0));
                    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4 *)(a1));
                    const uintx2 l2 = __builtin_bit_cast(uintx2, lo), h2 = __builtin_bit_cast(uintx2, hi);
                    const uintx4 vf = uintx4{l2[0], l2[1], h2[0], h2[1]};
                    acc_o[u] = mfma_32x32x16<DT>(vf, pf[t][s], acc_o[u]);
                }
            }
    };
    issue(0, 0);
    for (int64_t key0 = 0; key0 < p.N; key0 += 2 * kBK) {
        block(key0, std::integral_constant<int, 0>{});
        if (key0 + kBK < p.N) block(key0 + kBK, std::integral_constant<int, 1>{});
    }

    // normalise and store: register r of acc_o[u] is output column 32 u + 8 (r/4) + 4 half + r%4 of query q
    const float total = l + __shfl_xor(l, 32, 64);
    const float inv = 1.0f / total;
    if (q < p.N) {
#pragma unroll
        for (int u = 0; u < TU; ++u)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int dv = 32 * u + 8 * gq + 4 * half;
                *reinterpret_cast<uintx2 *>(Ob + q * ldb + dv * 2) =
                    uintx2{pack2_16<DT>(acc_o[u][4 * gq] * inv, acc_o[u][4 * gq + 1] * inv),
                           pack2_16<DT>(acc_o[u][4 * gq + 2] * inv, acc_o[u][4 * gq + 3] * inv)};
            }
    }
#endif
}

// ---- the same arithmetic with the matrix pipe and the vector ALU kept busy at the same time ------
//
// Counters of mhsa_flash_kernel on 4 x 4096 x 2048 (16 heads): matrix pipe busy 53 % of the launch,
// the softmax's vector instructions (4.8 per matrix instruction, one in five an exponential at a
// quarter of the rate) another 52 %, and only 16 % of the launch with both at work: two independent
// workgroups on a CU drift into the same phase, and then a SIMD's two waves want the matrix pipe
// together and the vector ALU together.  Here ONE workgroup of eight waves holds 256 queries and its
// two halves are kept in opposite phases by the workgroup barrier itself: time is cut into slots
// that begin with a barrier; group A (128 queries, one wave per SIMD) runs its matrix phase
//     M(i) = { O^T += V_{i-1}^T . P_{i-1}^T ;  S_i^T = K_i . Q^T }        (32 matrix instructions)
// in the even slots and the softmax of block i in the odd ones, group B (the other 128 queries, the
// SIMDs' other waves) does the same one slot later.  Every SIMD then has one wave on the matrix pipe
// and one on the vector ALU in every slot.  Both groups read the same K and V tiles, a slot apart:
// K_i is live in slots 2i, 2i+1 and V_i in slots 2i+2, 2i+3, so two buffers each suffice, and all
// eight waves issue the loads of K_{i+1} and V_i at the start of slot 2i, two slots before their
// first use (the barrier into an odd slot lets them stay in flight).
template <int ALLOW>
__device__ __forceinline__ void slot_barrier(bool relaxed)
{
    asm volatile("" ::: "memory");
    // lgkmcnt(0) always; vmcnt(ALLOW) where the newest loads may stay in flight, else vmcnt(0)
    if (relaxed) __builtin_amdgcn_s_waitcnt(0x0070 | (ALLOW & 15) | ((ALLOW >> 4) << 14));
    else __builtin_amdgcn_s_waitcnt(0x0070);
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

constexpr int kPQ = 256;                 // queries per workgroup of the ping-pong kernel

template <int DK, int DT>
__global__ __launch_bounds__(512, 2) void mhsa_pingpong_kernel(AttnParams p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    constexpr int ROWB = DK * 2, CHUNKS = DK / 8, KS = DK / 16, TU = DK / 32;
    constexpr int VKEY = DK == 128 ? 4 : 2;
    constexpr int TILE = kBK * ROWB;                 // bytes of one K (or V) tile
    constexpr int RPL = 1024 / ROWB;                 // tile rows one wave-wide load covers
    constexpr int LOADS = kBK / (4 * RPL);           // loads per loading wave per tile
    __shared__ __attribute__((aligned(1024))) char lds[4 * TILE];     // K buffers 0, 1, then V buffers 0, 1

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // a workgroup's waves go to the four SIMDs in turn (measured: the other split of the waves is 25 % slower),
    // so waves w and w + 4 share one: group A = waves 0-3, group B = waves 4-7
    const int grp = wave >> 2, sub = wave & 3;
    const int col = lane & 31, half = lane >> 5;
    const int64_t qblocks = (p.N + kPQ - 1) / kPQ;
    const int64_t pairs = p.batch * p.heads;
    int64_t qb, bh;
    if (pairs % 8 == 0) {                            // a pair's workgroups behind one XCD's L2 (see mhsa_flash_kernel)
        const int64_t x = blockIdx.x % 8, j = blockIdx.x / 8;
        bh = x + 8 * (j / qblocks);
        qb = j % qblocks;
    } else {
        qb = blockIdx.x % qblocks;
        bh = blockIdx.x / qblocks;
    }
    const int64_t b = bh / p.heads, head = bh % p.heads;
    const int64_t ldb = p.d_model * 2;
    const char *Qb = p.Q + (b * p.N * p.d_model + head * DK) * 2;
    const char *Kb = p.K + (b * p.N * p.d_model + head * DK) * 2;
    const char *Vb = p.V + (b * p.N * p.d_model + head * DK) * 2;
    char *Ob = p.O + (b * p.N * p.d_model + head * DK) * 2;

    const int64_t q = qb * kPQ + grp * 128 + sub * 32 + col;
    const int64_t qc = q < p.N ? q : p.N - 1;
    uintx4 qf[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const uintx4 *>(Qb + qc * ldb + (16 * s + 8 * half) * 2);

    floatx16 acc_o[TU], acc_s[2];
#pragma unroll
    for (int u = 0; u < TU; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[u][r] = 0.0f;
    float m = -__builtin_inff(), l = 0.0f;
    uintx4 pf[2][2];

    // Tile loads are group B's: its wave `sub` fills rows RPL (sub + 4 i) .. of a tile with its load i.  A wave
    // stalls at a load while the CU's address unit is busy with earlier ones, so the loads are not issued in a
    // burst at a barrier (where eight waves' worth queue up behind each other) but a few at a time between the
    // exponentials of group B's softmax, in the even slots, when that wave's vector ALU has work to hide them.
    const int ld_row = RPL * sub + lane / CHUNKS, ld_slot = lane % CHUNKS;
    const uint32_t ld_kc = (DK == 128 ? (ld_slot ^ (ld_row & 15)) : (ld_slot ^ ((ld_row >> 1) & 7))) * 16;
    const uint32_t ld_vc = (ld_slot ^ (VKEY * (ld_row & 3))) * 16;
    const uint32_t ldb32 = (uint32_t)ldb;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>((lds_char *)lds) + sub * 1024);
    const int64_t nb = (p.N + kBK - 1) / kBK;
    auto issue_part = [&](const char *base, uint32_t chunk, int64_t key0, uint32_t dst, int i0, int n) __attribute__((always_inline)) {
        const char *g = scalar_ptr(base + key0 * ldb);
        const int last = (int)(p.N - key0) - 1;                          // rows past the end re-read the last key
#pragma unroll
        for (int i = i0; i < i0 + n; ++i) {
            const int row = ld_row + 4 * RPL * i;
            dma_load16(g, (uint32_t)(row < last ? row : last) * ldb32 + chunk, __builtin_amdgcn_readfirstlane(dst + i * 4096));
        }
    };
    // Slot 2 j: K_{j+1} and V_j go out in four parts (part 0, 1: halves of K_{j+1}; 2, 3: halves of V_j).  Their
    // buffers were last read in slot 2 j - 1 and they are first read in slot 2 j + 2.
    auto issue_quarter = [&](int64_t j, int part) __attribute__((always_inline)) {
        if (part < 2) {
            if (j + 1 < nb) issue_part(Kb, ld_kc, (j + 1) * kBK, lds0 + (uint32_t)((j + 1) & 1) * TILE, (part & 1) * (LOADS / 2), LOADS / 2);
        } else {
            if (j < nb) issue_part(Vb, ld_vc, j * kBK, lds0 + 2 * TILE + (uint32_t)(j & 1) * TILE, (part & 1) * (LOADS / 2), LOADS / 2);
        }
    };

    const int g4 = lane >> 4, jj = lane & 15;
    const int tr_row = 4 * (g4 >> 1) + (jj >> 2);
    const int tr_col = 16 * (g4 & 1) + 4 * (jj & 3);

    // matrix phase of block i (PAR = i & 1): O^T += V_{i-1}^T . P_{i-1}^T, then S_i^T = K_i . Q^T
    auto matrix_phase = [&](int64_t i, auto parc, auto pvc, auto stc) __attribute__((always_inline)) {
        constexpr int PAR = decltype(parc)::value;
        constexpr bool PV = decltype(pvc)::value, ST = decltype(stc)::value;
        lds_char *const kt = (lds_char *)lds + PAR * TILE;
        lds_char *const vt = (lds_char *)lds + 2 * TILE + (PAR ^ 1) * TILE;
        if constexpr (PV) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int r0 = 32 * t + 16 * s + tr_row;
#pragma unroll
                    for (int u = 0; u < TU; ++u) {
                        const int cb = (32 * u + tr_col) * 2;
                        const int c = cb >> 4, within = cb & 15;
                        const lds_char *a0 = vt + r0 * ROWB + ((c ^ (VKEY * (r0 & 3))) << 4) + within;
                        const lds_char *a1 = vt + (r0 + 8) * ROWB + ((c ^ (VKEY * ((r0 + 8) & 3))) << 4) + within;
                        const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4 *)(a0));
                        const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4 *)(a1));
                        const uintx2 l2 = __builtin_bit_cast(uintx2, lo), h2 = __builtin_bit_cast(uintx2, hi);
                        acc_o[u] = mfma_32x32x16<DT>(uintx4{l2[0], l2[1], h2[0], h2[1]}, pf[t][s], acc_o[u]);
                    }
                }
        }
        if constexpr (ST) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_s[t][r] = 0.0f;
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const int row = 32 * t + col;
                    const int c = 2 * s + half;
                    const int kc = DK == 128 ? (c ^ (row & 15)) : (c ^ ((row >> 1) & 7));
                    const uintx4 kf = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(kt + row * ROWB + kc * 16);
                    acc_s[t] = mfma_32x32x16<DT>(kf, qf[s], acc_s[t]);
                }
        }
        // order for the scheduler: the transposing V reads run kAhead matrix instructions ahead of their
        // consumers, then the K fragment reads take over, so that LDS latency is paid once per phase
        constexpr int NPV = PV ? 4 * TU : 0, NST = ST ? 2 * KS : 0, kAhead = 4;
        if constexpr (PV) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2 * kAhead, 0);
#pragma unroll
            for (int k = 0; k < NPV; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (k + kAhead < NPV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                else if (ST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        } else if constexpr (ST) {
            __builtin_amdgcn_sched_group_barrier(0x100, kAhead, 0);
        }
        if constexpr (ST) {
#pragma unroll
            for (int k = 0; k < NST; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (k + kAhead < NST) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            const int64_t key0 = i * kBK;
            if (key0 + kBK > p.N) {                                       // keys past the end drop out
                const int left = (int)(p.N - key0);
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (32 * t + 8 * (r >> 2) + 4 * half + (r & 3) >= left) acc_s[t][r] = -__builtin_inff();
            }
        }
    };
    const bool first = grp == 0;                     // wave-uniform
    if (!first) issue_part(Kb, ld_kc, 0, lds0, 0, LOADS);
    slot_barrier<0>(false);                          // start of slot 0: K_0 is in place
    if (!first) {                                    // group B sits out slot 0 and sends K_1 and V_0 on their way
#pragma unroll
        for (int part = 0; part < 4; ++part) issue_quarter(0, part);
        slot_barrier<2 * LOADS>(true);
    }
    // One iteration = a matrix phase and a softmax, each ended by a barrier; one instruction stream serves both
    // groups.  Group A enters it at the start of an even slot, group B of an odd one, so B's softmax of block i
    // runs in slot 2 i + 2 and carries that slot's loads.  They may stay in flight over the barrier that follows
    // the softmax and must have landed at the one that follows the matrix phase (group A never has any).
    auto iteration = [&](int64_t i, auto parc, auto pvc, auto stc) __attribute__((always_inline)) {
        matrix_phase(i, parc, pvc, stc);
        slot_barrier<0>(false);                      // A: into slot 2 i + 1;  B: into slot 2 i + 2
        if constexpr (decltype(stc)::value)
            softmax_block<DT, TU>(acc_s, acc_o, pf, m, l, p.scale2,
                                  [&](int part) __attribute__((always_inline)) { if (!first) issue_quarter(i + 1, part); });
        slot_barrier<2 * LOADS>(true);               // A: into slot 2 i + 2;  B: into slot 2 i + 3
    };
    using c0 = std::integral_constant<int, 0>;
    using c1 = std::integral_constant<int, 1>;
    iteration(0, c0{}, std::false_type{}, std::true_type{});             // block 0: scores only
    for (int64_t i = 1; i < nb; i += 2) {
        iteration(i, c1{}, std::true_type{}, std::true_type{});
        if (i + 1 < nb) iteration(i + 1, c0{}, std::true_type{}, std::true_type{});
    }
    if (nb & 1) iteration(nb, c1{}, std::true_type{}, std::false_type{});   // the last block's second product
    else iteration(nb, c0{}, std::true_type{}, std::false_type{});
    if (first) slot_barrier<0>(false);               // group A ends one slot earlier: same number of barriers for all

    const float total = l + __shfl_xor(l, 32, 64);
    const float inv = 1.0f / total;
    if (q < p.N) {
#pragma unroll
        for (int u = 0; u < TU; ++u)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const int dv = 32 * u + 8 * gq + 4 * half;
                *reinterpret_cast<uintx2 *>(Ob + q * ldb + dv * 2) =
                    uintx2{pack2_16<DT>(acc_o[u][4 * gq] * inv, acc_o[u][4 * gq + 1] * inv),
                           pack2_16<DT>(acc_o[u][4 * gq + 2] * inv, acc_o[u][4 * gq + 3] * inv)};
            }
    }
#endif
}

// ---- fallback: one wave per query, fp32 arithmetic ---------------------------------------------

template <int DT>
__device__ __forceinline__ float load_elem(const char *base, int64_t idx)
{
    if (DT == DT_F32) return reinterpret_cast<const float *>(base)[idx];
    return from_16<DT>(reinterpret_cast<const unsigned short *>(base)[idx]);
}

template <int DT>
__global__ __launch_bounds__(256) void mhsa_rows_kernel(AttnParams p)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t dk = p.d_model / p.heads;
    const int64_t rows = p.batch * p.heads * p.N;
    const int64_t id = (int64_t)blockIdx.x * 4 + wave;
    if (id >= rows) return;
    const int64_t q = id % p.N, bh = id / p.N, b = bh / p.heads, head = bh % p.heads;
    const int64_t base = b * p.N * p.d_model + head * dk;
    const float scale = p.scale2;                       // scores are kept in base 2
    float m = -__builtin_inff(), l = 0.0f, o[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // lane owns columns lane, lane+64, ...
    for (int64_t key0 = 0; key0 < p.N; key0 += 64) {
        const int64_t n = key0 + lane;
        float s = -__builtin_inff();
        if (n < p.N) {
            float d = 0.0f;
            for (int64_t c = 0; c < dk; ++c)
                d = fmaf(load_elem<DT>(p.Q, base + q * p.d_model + c), load_elem<DT>(p.K, base + n * p.d_model + c), d);
            s = d * scale;
        }
        float bm = s;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float t = __shfl_xor(bm, off, 64);
            bm = t > bm ? t : bm;
        }
        const float m_new = m > bm ? m : bm;
        const float corr = __builtin_amdgcn_exp2f(m - m_new);
        const float pw = __builtin_amdgcn_exp2f(s - m_new);     // 0 for keys past the end
        float ps = pw;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ps += __shfl_xor(ps, off, 64);
        l = l * corr + ps;
        m = m_new;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] *= corr;
        const int64_t nk = p.N - key0 < 64 ? p.N - key0 : 64;
        for (int64_t j = 0; j < nk; ++j) {
            const float w = __shfl(pw, (int)j, 64);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t c = lane + 64 * t;
                if (c < dk) o[t] = fmaf(w, load_elem<DT>(p.V, base + (key0 + j) * p.d_model + c), o[t]);
            }
        }
    }
    const float inv = 1.0f / l;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int64_t c = lane + 64 * t;
        if (c < dk) {
            const float y = o[t] * inv;
            if (DT == DT_F32) reinterpret_cast<float *>(p.O)[base + q * p.d_model + c] = y;
            else reinterpret_cast<unsigned short *>(p.O)[base + q * p.d_model + c] = to_16<DT>(y);
        }
    }
}

bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

// 0: flash kernel, 1: fallback, -1: not supported (d_k > 256 without a flash kernel)
int mhsa_path(int64_t d_model, int64_t heads, int dtype, const void *Q, const void *K, const void *V, const void *O)
{
    const int64_t dk = d_model / heads;
    if (dtype != DT_F32 && (dk == 64 || dk == 128) && aligned16(Q) && aligned16(K) && aligned16(V) && aligned16(O))
        return 0;
    return dk <= 256 ? 1 : -1;
}

hipError_t launch_mhsa(int64_t batch, int64_t N, int64_t d_model, int64_t heads, const void *Q, const void *K,
                       const void *V, void *O, int dtype, int path, hipStream_t stream)
{
    const int64_t dk = d_model / heads;
    AttnParams p;
    p.batch = batch; p.N = N; p.d_model = d_model; p.heads = heads;
    p.Q = static_cast<const char *>(Q); p.K = static_cast<const char *>(K); p.V = static_cast<const char *>(V);
    p.O = static_cast<char *>(O);
    p.scale2 = (float)(1.4426950408889634 / sqrt((double)dk));
    if (path == 0 && dk == 128 && N >= kPQ) {
        // d_k = 128 and at least one full block of 256 queries: the eight-wave kernel with its two halves in
        // opposite phases (for d_k = 64 the four-wave kernel below is the faster one)
        const int64_t grid = batch * heads * ((N + kPQ - 1) / kPQ);
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        const dim3 g((unsigned)grid), b(512);
        if (dtype == DT_F16) hipLaunchKernelGGL((mhsa_pingpong_kernel<128, DT_F16>), g, b, 0, stream, p);
        else hipLaunchKernelGGL((mhsa_pingpong_kernel<128, DT_BF16>), g, b, 0, stream, p);
        return hipGetLastError();
    }
    if (path == 0) {
        const int64_t grid = batch * heads * ((N + kBQ - 1) / kBQ);
        if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
        const dim3 g((unsigned)grid), b(256);
        if (dtype == DT_F16) {
            if (dk == 128) hipLaunchKernelGGL((mhsa_flash_kernel<128, DT_F16>), g, b, 0, stream, p);
            else hipLaunchKernelGGL((mhsa_flash_kernel<64, DT_F16>), g, b, 0, stream, p);
        } else {
            if (dk == 128) hipLaunchKernelGGL((mhsa_flash_kernel<128, DT_BF16>), g, b, 0, stream, p);
            else hipLaunchKernelGGL((mhsa_flash_kernel<64, DT_BF16>), g, b, 0, stream, p);
        }
        return hipGetLastError();
    }
    const int64_t grid = (batch * heads * N + 3) / 4;
    if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dtype == DT_F32) hipLaunchKernelGGL(mhsa_rows_kernel<DT_F32>, dim3((unsigned)grid), dim3(256), 0, stream, p);
    else if (dtype == DT_F16) hipLaunchKernelGGL(mhsa_rows_kernel<DT_F16>, dim3((unsigned)grid), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(mhsa_rows_kernel<DT_BF16>, dim3((unsigned)grid), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace optiml

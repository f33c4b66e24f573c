// bf16 MFMA tile kernel with a ring of small LDS stages fed by direct global->LDS loads:
// 256x256 C block, 8 waves (2 x 4, wave tile 128 x 64), k-tiles of 32, NS stages of 32 KiB.
//
// Why a ring.  The two-stage kernel of kernel_tile_direct.hpp has at most one 64 KiB tile in
// flight per CU while it multiplies the other, and measurement shows its load path alone
// (L2 -> LDS, about a microsecond of latency under load) takes longer than its MFMAs.  With
// NS stages of half the depth, NS-2 stages are in flight while one is multiplied and one is
// being released: 64 KiB (NS = 4) or 96 KiB (NS = 5) in flight at the same LDS footprint per
// byte in use, at the price of a barrier every 32 instead of every 64 k.
//
// Per k-tile t (stage t % NS):   wait until at most (NS-2) stages' worth of this wave's loads
// are outstanding (loads complete in order, so tile t has landed); barrier (everybody's part of
// tile t has landed and everybody has finished tile t-1); start the loads of tile t+NS-1 into
// the stage tile t-1 occupied; multiply tile t.  Past the end the loads re-fetch the last tile
// (in bounds, never read) so that the wait counts stay uniform.
//
// Each stage is its own __shared__ array and each step is an inlined function with
// restrict-qualified stage pointers: that is what lets the compiler prove that the in-flight DMA
// writes cannot touch the stage being read, so it does not drain the loads before every
// fragment read.
//
// LDS formats.  A (and column-major B): 256 rows x 64 bytes, 16-byte chunk c of row r at
// r*64 + ((c ^ ((r >> 2) & 3)) << 4): sixteen consecutive rows at one logical chunk cover the 64
// banks once.  Row-major B: 32 k-rows x 512 bytes, chunk c of row k at k*512 + ((c ^ 4(k&3)) << 4):
// the four k-rows that a 16-lane group of ds_read_b64_tr_b16 touches (see kernel_tile_direct.hpp
// for its lane layout) sit in four different 64-byte bank groups, and so do those of the
// neighbouring group that reads the next 16 columns (measured 165 B/clk against 128 B/clk with a
// 32-byte shift per row).
#pragma once
#include "common.hpp"
#include "epilogue.hpp"

namespace optiml {
namespace ring {

typedef float floatx2 __attribute__((ext_vector_type(2)));
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
    // EPI == 1 only: class labels of the M rows and where the label's logit of each row goes;
    // C then points at the (max, sum) pairs [tiles_n * WN][M]
    // EPI == 2: C points at fp32 Z (pitch ldc floats) and `picked` at the (mean, sum of squared
    // deviations) pairs [tiles_n * WN][M]
    const int *labels;
    float *picked;
    int bias_row;        // EPI == 0: bias[m] instead of bias[n]
    // block-scaled operands (Cfg::MX): one E8M0 byte per row of A (column of B) and 32 elements of k,
    // the four scale bytes of k-tile t (128 k) of row i of A: scaleA + i * lds_a + t * sk_a, likewise for the columns of B
    const char *scaleA = nullptr, *scaleB = nullptr;
    int64_t lds_a = 0, lds_b = 0, sk_a = 4, sk_b = 4;
};

template <int NS_, bool B_KC_, bool PF_ = false, int WN_ = 4, int DT_ = DT_BF16, int EPI_ = 0, bool K64_ = false, int BAND_ = 8,
          int SWZ_ = 4, int WM_ = 2, bool MX_ = false>
struct Cfg {
    // Block-scaled E2M1 operands: every 32 consecutive k of a row of A (column of B) share an E8M0 scale.  A lane's
    // 16-byte fragment is exactly one such block, and the matrix instruction takes the block's scale from a byte of a
    // register of that lane.  The scales of a k-tile (four blocks = one dword per row) travel with the tile: one more
    // LDS-DMA load per wave and stage (4 bytes a lane) into 2 KiB behind the B tile.
    static constexpr bool MX = MX_;
    static_assert(!MX_ || (B_KC_ && EPI_ == 0 && WM_ == 2 && WN_ == 4 && ((DT_ == DT_F4 && PF_ && !K64_) || ((is_f8(DT_) || is_f6(DT_)) && K64_))),
                  "block scales: the 2 x 4 E2M1 kernel with fragment prefetch, or the 64-deep 8-bit kernel");
    // WM = 1: a 128 x 256 block computed by four waves (1 x 4, the same 128 x 64 wave tile) with 24 KiB
    // stages; with NS = 3 two such workgroups share a CU (144 KiB of LDS, at most 256 registers a lane),
    // so that one's first loads and epilogue run under the other's k loop: for many short tiles.
    static constexpr int MIN_WAVES_PER_SIMD = WM_ == 1 ? 2 : 1;
    // Tile walk: a band is BAND tile rows, walked column by column, so that the workgroups in flight on
    // an XCD share few panels of A and B.  SWZ: XOR key step of the row-major B tile in LDS, chunk c
    // of k-row k at (c ^ SWZ (k & 3)) - 4 measured best (165 B/clk against 128 B/clk for 2).  Both are
    // edit classes of the tree search.
    static constexpr int BAND = BAND_, SWZ = SWZ_;
    static_assert(BAND_ >= 1 && (SWZ_ == 2 || SWZ_ == 4 || SWZ_ == 8), "tile walk and swizzle key");
    // 8-bit operands only: one v_mfma_f32_32x32x64_f8f6f4 per k-tile and pair of fragments instead
    // of four v_mfma_f32_32x32x16_fp8_fp8
    static constexpr bool K64 = K64_;
    static_assert(!K64_ || ((is_f8(DT_) || is_f6(DT_)) && !PF_), "the 64-deep instruction: 8-bit or 6-bit operands, no fragment prefetch");
    static_assert(!is_f6(DT_) || K64_, "6-bit operands (in slot form): the 64-deep instruction only");
    static constexpr int DT = DT_;       // DT_BF16 or DT_F16: same tiles, another matrix instruction and rounding
    // 0: C = act(A.B + bias).  1: C is not written; each wave reduces its 64 columns of A.B + bias
    // to a (maximum, sum of exponentials) pair per row and hands out the label's logit: the
    // cross-entropy over the N columns without the logits ever reaching memory.  2: Z = A.B + bias
    // is written unrounded, as fp32, and each wave leaves the mean of its 64 columns of every row and
    // the sum of squared deviations from that mean: the row statistics of a LayerNorm over the N
    // columns come out of the registers that hold the product.
    static constexpr int EPI = EPI_;
    // DT_F8 / DT_BF8: A and B in 8-bit E4M3 / E5M2 (column-major B only), C in bf16.  The tile geometry is in
    // bytes, so a k-tile is 64 elements instead of 32 and each 16-byte fragment feeds two matrix
    // instructions.  DT_F4: the same with two E2M1 values in every byte (the problem arrives with K
    // counted in bytes) and one 64-deep scaled matrix instruction per pair of 16-byte fragments.
    static constexpr int ES = is_8bit(DT_) ? 1 : 2;          // bytes per element of A and B
    static constexpr int BKE = 64 / ES;                      // k elements per tile
    static constexpr int ODT = is_8bit(DT_) ? DT_BF16 : DT_; // storage type of C
    static_assert(!is_8bit(DT_) || B_KC_, "8-bit and 4-bit operands: k must be contiguous in both");
    static constexpr int NS = NS_;
    static constexpr bool B_KC = B_KC_;
    static constexpr bool PF = PF_;      // fetch the next tile's first fragments before the barrier
    static constexpr int AHEAD = PF_ ? NS_ - 3 : NS_ - 2;   // stages allowed in flight at the barrier
    static constexpr int BM = 128 * WM_, BN = 256, BK = 32, WM = WM_, WN = WN_, NW = WM * WN, THREADS = 64 * NW;
    static constexpr int WTM = BM / WM, WTN = BN / WN, TM = WTM / 32, TN = WTN / 32;
    static constexpr int A_BYTES = BM * 64, B_BYTES = BN * 64;
    static constexpr int SCALE_BYTES = MX_ ? (BM + BN) * 4 : 0;                                   // a dword per row and column
    static constexpr int STAGE_BYTES = A_BYTES + B_BYTES + SCALE_BYTES;                           // 32 KiB (34 with scales)
    static constexpr int A_INSTR = A_BYTES / 1024 / NW, B_INSTR = B_BYTES / 1024 / NW;
    static constexpr int LOADS = A_INSTR + B_INSTR + (MX_ ? 1 : 0);                               // per wave per stage
    static_assert(NS >= 3 && NS <= 5 && (!PF_ || NS_ >= 4), "ring depth");
    static_assert((WN == 2 || WN == 4) && (WM_ == 2 || (WM_ == 1 && WN_ == 4)), "2 x 2, 2 x 4 or 1 x 4 waves");
};

#if defined(__HIP_DEVICE_COMPILE__)

__device__ __forceinline__ const char *scalar_ptr(const char *q)
{
    const uint64_t v = reinterpret_cast<uint64_t>(q);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

// s_waitcnt vmcnt(N) lgkmcnt(0) (gfx9 encoding: vmcnt in bits 3:0 and 15:14, lgkmcnt in 11:8,
// expcnt in 6:4 left at its maximum): at most N of this wave's loads outstanding, and every LDS
// read it issued has returned.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0070 | (N & 15) | ((N >> 4) << 14));
}

// Workgroup barrier without the fences of __syncthreads(): a workgroup-scope release fence makes
// the compiler drain every outstanding LDS-DMA load (vmcnt(0)), which is exactly the prefetch
// depth this kernel is built to keep.  What the barrier must order is covered explicitly: the
// wait before it (this wave's part of the tile has landed in LDS and its LDS reads of the
// previous tile have returned), and the empty asm statements keep the compiler from moving
// memory operations across.
__device__ __forceinline__ void block_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

template <class C>
struct Ctx {
    uint32_t a_off[C::A_INSTR], b_off[C::B_INSTR];
    int a_frag[2], tr_cb[C::TN];
    int wave, a_wave, b_wave_kc, tr_row;
    uint32_t s_off;              // MX: this lane's row (waves 0-3: of A, 4-7: of B) times the pitch of the scales
    int sa_frag, sb_frag;        // MX: LDS offsets of this lane's first scale dwords within the stage
};

// One wave-wide LDS-DMA load: lane l copies 16 bytes from base + off(l) to LDS byte lds_addr + 16 l.
// Written as assembly so that the loads stay out of the compiler's wait-count bookkeeping: it
// cannot tell which ring stage a fragment read touches once more than a handful of these are
// in flight, and then drains all of them (vmcnt(0)) in front of LDS reads.  The kernel counts
// them itself (wait_vmcnt below).  base and lds_addr are wave-uniform.
__device__ __forceinline__ void dma_load16(const char *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(off), "s"(base), "s"(lds_addr)
                 : "m0");
}

// The same load with the non-temporal hint: for data that is read once, so that it does not push
// operands that many workgroups share out of the L2.
__device__ __forceinline__ void dma_load16_once(const char *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                 :
                 : "v"(off), "s"(base), "s"(lds_addr)
                 : "m0");
}

// ... and with 4 bytes a lane: lane l copies base + off(l) .. +3 to LDS byte lds_addr + 4 l
__device__ __forceinline__ void dma_load4(const char *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(off), "s"(base), "s"(lds_addr)
                 : "m0");
}

// gs (MX only): the scales of this wave's operand (A for waves 0-3, B for 4-7) at the tile's first block of k
template <class C>
__device__ __forceinline__ void issue_stage(const Ctx<C> &c, const char *__restrict__ ga, const char *__restrict__ gb,
                                            lds_char *__restrict__ dst, const char *__restrict__ gs = nullptr)
{
    ga = scalar_ptr(ga);
    gb = scalar_ptr(gb);
    const uint32_t d = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(dst) + c.wave * 1024);
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i) dma_load16(ga, c.a_off[i], d + i * C::NW * 1024);
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i) dma_load16(gb, c.b_off[i], d + C::A_BYTES + i * C::NW * 1024);
    if constexpr (C::MX) {
        // wave w fills dwords 64 w .. 64 w + 63 of the scale area: rows 0-255 of A, then columns 0-255 of B
        const uint32_t ds = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(dst) + C::A_BYTES + C::B_BYTES + c.wave * 256);
        dma_load4(scalar_ptr(gs), c.s_off, ds);
    }
}

template <class C>
struct Frags {
    uintx4 a[C::TM], b[C::TN];
};

// MX: the scale dwords of a wave's rows and columns for one stage, shifted so that byte 0 is this lane's block of
// k-step 0 and byte 2 that of k-step 1
template <class C>
struct Scales {
    unsigned int a[C::TM], b[C::TN];
};

template <class C>
__device__ __forceinline__ void load_scales(const Ctx<C> &c, const lds_char *rd, Scales<C> &sc)
{
    const int shift = (threadIdx.x & 32) ? 8 : 0;
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
        sc.a[i] = *reinterpret_cast<const __attribute__((address_space(3))) unsigned int *>(rd + c.sa_frag + i * 128) >> shift;
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
        sc.b[j] = *reinterpret_cast<const __attribute__((address_space(3))) unsigned int *>(rd + c.sb_frag + j * 128) >> shift;
}

// MFMA operands of k-step s (16 k) of the tile held in stage `rd`
template <class C>
__device__ __forceinline__ void load_frags(const Ctx<C> &c, const lds_char *rd, int s, Frags<C> &f)
{
    const lds_char *sa = rd + c.a_wave;
    const lds_char *sb = rd + C::A_BYTES;
#pragma unroll
    for (int i = 0; i < C::TM; ++i)
        f.a[i] = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(sa + i * 32 * 64 + c.a_frag[s]);
#pragma unroll
    for (int j = 0; j < C::TN; ++j) {
        if constexpr (C::B_KC) {
            f.b[j] = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(
                sb + c.b_wave_kc + j * 32 * 64 + c.a_frag[s]);
        } else {
            const lds_char *q0 = sb + (16 * s + c.tr_row) * (C::BN * 2) + c.tr_cb[j];
            const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) shortx4 *)(q0));
            const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) shortx4 *)(q0 + 4 * (C::BN * 2)));
            const uintx2 l2 = __builtin_bit_cast(uintx2, lo), h2 = __builtin_bit_cast(uintx2, hi);
            f.b[j] = uintx4{l2[0], l2[1], h2[0], h2[1]};
        }
    }
}

template <class C, int J0 = 0, int J1 = C::TN>
__device__ __forceinline__ void mma_frags(const Frags<C> &f, floatx16 (&acc)[C::TN][C::TM])
{
#pragma unroll
    for (int j = J0; j < J1; ++j)
#pragma unroll
        for (int i = 0; i < C::TM; ++i)
            acc[j][i] = mfma_32x32x16<C::DT>(f.b[j], f.a[i], acc[j][i]);
}

// The same with block scales: `sc` holds the scale dwords of the stage the fragments come from, SH = 0 for
// its k-step 0 and 16 for k-step 1.  The instruction's first operand is the B fragment (the tile is computed
// transposed), so its scale is the column's.
template <class C, int SH, int J0 = 0, int J1 = C::TN>
__device__ __forceinline__ void mma_frags_mx(const Frags<C> &f, const Scales<C> &sc, floatx16 (&acc)[C::TN][C::TM])
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef int intx8_ __attribute__((ext_vector_type(8)));
#pragma unroll
    for (int j = J0; j < J1; ++j)
#pragma unroll
        for (int i = 0; i < C::TM; ++i) {
            const intx8_ b = {(int)f.b[j][0], (int)f.b[j][1], (int)f.b[j][2], (int)f.b[j][3], 0, 0, 0, 0};
            const intx8_ a = {(int)f.a[i][0], (int)f.a[i][1], (int)f.a[i][2], (int)f.a[i][3], 0, 0, 0, 0};
            // byte SH / 8 of the scale dwords
            acc[j][i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b, a, acc[j][i], 4, 4, SH / 8, (int)sc.b[j], SH / 8, (int)sc.a[i]);
        }
#endif
}

// One k-tile of 32: see the file header for the order of events.  With C::PF the operands of
// the tile's first k-step arrive in `f0` (fetched during the previous step) and the step ends by
// fetching the next tile's first k-step from `nxt`, which the barrier at the top has made
// visible one tile early: the MFMAs then start right after the barrier instead of waiting for
// LDS.
// EXTRA: vector-memory operations of this wave, other than ring loads, that were issued after
// the loads this step waits for and may still be outstanding (they complete in issue order, so
// the count to wait for grows by that many).
template <class C, int EXTRA = 0>
__device__ __forceinline__ void ring_step(const Ctx<C> &c, const char *__restrict__ ga, const char *__restrict__ gb,
                                          lds_char *__restrict__ dma, const lds_char *__restrict__ rd,
                                          const lds_char *__restrict__ nxt, Frags<C> &f0,
                                          floatx16 (&acc)[C::TN][C::TM], const char *__restrict__ gs = nullptr,
                                          Scales<C> *carried = nullptr)
{
    static_assert(C::AHEAD * C::LOADS + EXTRA <= 63, "vmcnt is a 6-bit counter");
    wait_vmcnt<C::AHEAD * C::LOADS + EXTRA>();
    block_barrier();
    Frags<C> f1;
    if constexpr (C::PF) {
        // The MFMAs of the first k-step start right behind the barrier (their operands are in
        // f0 already); the loads of the new tile are issued in two batches between MFMA groups,
        // where the matrix pipe has a backlog to hide the issue slots.
        ga = scalar_ptr(ga);
        gb = scalar_ptr(gb);
        const uint32_t d = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(dma) + c.wave * 1024);
        constexpr int NR = C::TM + (C::B_KC ? C::TN : 2 * C::TN), H = C::TN / 2, NMH = C::TM * H;
        // MX: the scale dwords of this stage were fetched at the end of the previous step (below), into the
        // registers its own matrix instructions had just read for the last time
        load_frags<C>(c, rd, 1, f1);
        if constexpr (C::MX) mma_frags_mx<C, 0, 0, H>(f0, *carried, acc);
        else mma_frags<C, 0, H>(f0, acc);
#pragma unroll
        for (int i = 0; i < NMH; ++i) {            // second k-step's operands under these MFMAs
            __builtin_amdgcn_sched_group_barrier(0x100, (NR + NMH - 1) / NMH, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < C::A_INSTR; ++i) dma_load16(ga, c.a_off[i], d + i * C::NW * 1024);
        if constexpr (C::MX) mma_frags_mx<C, 0, H, C::TN>(f0, *carried, acc);
        else mma_frags<C, H, C::TN>(f0, acc);
#pragma unroll
        for (int i = 0; i < C::B_INSTR; ++i) dma_load16(gb, c.b_off[i], d + C::A_BYTES + i * C::NW * 1024);
        if constexpr (C::MX) {
            // wave w fills dwords 64 w .. 64 w + 63 of the scale area, as issue_stage does
            const uint32_t ds = __builtin_amdgcn_readfirstlane((uint32_t)reinterpret_cast<uintptr_t>(dma) + C::A_BYTES + C::B_BYTES + c.wave * 256);
            dma_load4(scalar_ptr(gs), c.s_off, ds);
        }
        load_frags<C>(c, nxt, 0, f0);
        if constexpr (C::MX) mma_frags_mx<C, 16>(f1, *carried, acc);
        else mma_frags<C>(f1, acc);
#pragma unroll
        for (int i = 0; i < 2 * NMH; ++i) {        // next tile's first operands under these MFMAs
            if (i < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        if constexpr (C::MX) {
            __builtin_amdgcn_sched_barrier(0);     // behind the step's last matrix instruction
            load_scales<C>(c, nxt, *carried);
        }
        return;
    }
    issue_stage<C>(c, ga, gb, dma, gs);
    __builtin_amdgcn_sched_barrier(0);      // the loads go out before the tile is multiplied
    {
        load_frags<C>(c, rd, 0, f0);
        load_frags<C>(c, rd, 1, f1);
        if constexpr (C::K64 && C::MX) {
            // block scales: lanes 0-31 supply the scale of the k-tile's first block, lanes 32-63 that of the second
            // (byte 0 of the shifted dword); the first operand is B's
            Scales<C> sc;
            load_scales<C>(c, rd, sc);
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int i = 0; i < C::TM; ++i)
                    acc[j][i] = mfma_32x32x64_f8_scaled<C::DT>(f0.b[j], f1.b[j], f0.a[i], f1.a[i], acc[j][i], sc.b[j], sc.a[i]);
        } else if constexpr (C::K64) {
            // both 16-byte fragments of a row are one 32-byte operand: 64 values of k (which value
            // sits in which byte only has to agree between the two operands)
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int i = 0; i < C::TM; ++i)
                    acc[j][i] = mfma_32x32x64_f8<C::DT>(f0.b[j], f1.b[j], f0.a[i], f1.a[i], acc[j][i]);
        } else {
            mma_frags<C>(f0, acc);
            mma_frags<C>(f1, acc);
        }
    }
}
#endif

template <class C>
__global__ __launch_bounds__(C::THREADS, C::MIN_WAVES_PER_SIMD) void gemm_ring_kernel(Params p)
{
#if defined(__HIP_DEVICE_COMPILE__)
    // one array per ring stage (distinct objects: see the file header); unused ones cost nothing
    __shared__ __attribute__((aligned(1024))) char st0[C::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char st1[C::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char st2[C::STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char st3[C::NS > 3 ? C::STAGE_BYTES : 1024];
    __shared__ __attribute__((aligned(1024))) char st4[C::NS > 4 ? C::STAGE_BYTES : 1024];
    constexpr int TM = C::TM, TN = C::TN, NW = C::NW, NS = C::NS;

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
    constexpr int BAND = C::BAND;
    const int64_t band = t / (BAND * p.tiles_n), first = band * BAND;
    const int64_t rows_in_band = p.tiles_m - first < BAND ? p.tiles_m - first : BAND;
    t -= band * BAND * p.tiles_n;
    const int64_t tile_m = first + t % rows_in_band, tile_n = t / rows_in_band;
    const int64_t m0 = tile_m * C::BM, n0 = tile_n * C::BN;

    const char *A = p.A + batch * p.strideA * C::ES;
    const char *B = p.B + batch * p.strideB * C::ES;

    Ctx<C> ctx;
    ctx.wave = wave;
    // A and column-major B: load q covers LDS rows 16q..16q+15; lane l fills row 16q + l/4, slot l%4
#pragma unroll
    for (int i = 0; i < C::A_INSTR; ++i) {
        const int q = wave + i * NW, r = 16 * q + (lane >> 2);
        const int c = (lane & 3) ^ ((r >> 2) & 3);
        int64_t row = m0 + r;
        row = row < p.M ? row : p.M - 1;
        ctx.a_off[i] = (uint32_t)(row * p.lda * C::ES + c * 16);
    }
#pragma unroll
    for (int i = 0; i < C::B_INSTR; ++i) {
        const int q = wave + i * NW;
        if constexpr (C::B_KC) {
            const int r = 16 * q + (lane >> 2);
            const int c = (lane & 3) ^ ((r >> 2) & 3);
            int64_t row = n0 + r;
            row = row < p.N ? row : p.N - 1;
            ctx.b_off[i] = (uint32_t)(row * p.ldb * C::ES + c * 16);
        } else {
            const int pidx = q * 64 + lane, k = pidx >> 5;          // 32 chunks per k-row
            const int c = (pidx & 31) ^ (C::SWZ * (k & 3));
            int64_t col = n0 + c * 8;
            col = col + 8 <= p.N ? col : p.N - 8;
            ctx.b_off[i] = (uint32_t)((k * p.ldb + col) * 2);
        }
    }
    const int64_t b_step = C::B_KC ? 64 : 32 * p.ldb * 2;           // bytes per k-tile

    floatx16 acc[TN][TM];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[j][i][r] = 0.0f;

    const int frag_row = lane & 31, half = lane >> 5;
    // fragment s of this lane is chunk 2 s + half of the row's 64 bytes.  (Block scales on 8-bit operands: the
    // 64-deep instruction takes the scale of k 0-31 from lanes 0-31 and that of k 32-63 from lanes 32-63, and reads
    // k 16 half .. + 15 from a lane's first four registers and k 32 + 16 half .. + 15 from its last four - which is
    // this very assignment; the tests with one-hot rows and single scale bytes changed pin it.)
#pragma unroll
    for (int s = 0; s < 2; ++s) ctx.a_frag[s] = frag_row * 64 + (((2 * s + half) ^ ((frag_row >> 2) & 3)) << 4);
    ctx.a_wave = wm * C::WTM * 64;
    ctx.b_wave_kc = wn * C::WTN * 64;
    const int g = lane >> 4, jj = lane & 15;
    ctx.tr_row = 8 * (g >> 1) + (jj >> 2);
    const int tr_col = wn * C::WTN + 16 * (g & 1) + 4 * (jj & 3);
    const int tr_key = C::SWZ * (jj >> 2);                   // SWZ * (row & 3)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = tr_col + 32 * j;
        ctx.tr_cb[j] = (((col >> 3) ^ tr_key) << 4) + ((col & 7) << 1);
    }

    lds_char *stage[5] = {(lds_char *)st0, (lds_char *)st1, (lds_char *)st2, (lds_char *)st3, (lds_char *)st4};
    const int64_t nk = p.K / C::BKE, last = nk - 1;        // nk >= NS - 1
    auto ga = [&](int64_t kt) { return A + (kt < last ? kt : last) * 64; };
    auto gb = [&](int64_t kt) { return B + (kt < last ? kt : last) * b_step; };
    // block scales: waves 0-3 fetch those of the tile's 256 rows of A, waves 4-7 those of its 256 columns of B
    // (rows and columns past the end re-read the last valid one), four bytes = four blocks of k per k-tile
    const char *S = nullptr;
    ctx.s_off = 0; ctx.sa_frag = 0; ctx.sb_frag = 0;
    if constexpr (C::MX) {
        const bool of_a = wave < 4;
        int64_t row = (of_a ? m0 : n0) + 64 * (wave & 3) + lane;
        const int64_t limit = of_a ? p.M : p.N;
        row = row < limit ? row : limit - 1;
        ctx.s_off = (uint32_t)(row * (of_a ? p.lds_a : p.lds_b));
        S = of_a ? p.scaleA : p.scaleB;                         // one problem per call
        ctx.sa_frag = C::A_BYTES + C::B_BYTES + (wm * C::WTM + frag_row) * 4;
        ctx.sb_frag = C::A_BYTES + C::B_BYTES + C::BM * 4 + (wn * C::WTN + frag_row) * 4;
    }
    const int64_t s_step = C::MX ? (wave < 4 ? p.sk_a : p.sk_b) : 0;
    auto gs = [&](int64_t kt) { return C::MX ? S + (kt < last ? kt : last) * s_step : nullptr; };

    // prologue: tiles 0 .. NS-2
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_stage<C>(ctx, ga(s), gb(s), stage[s], gs(s));
    Frags<C> f0;
    Scales<C> sc;
    if constexpr (C::PF) {
        wait_vmcnt<(NS - 2) * C::LOADS>();   // tile 0 has landed
        block_barrier();
        load_frags<C>(ctx, stage[0], 0, f0);
        if constexpr (C::MX) load_scales<C>(ctx, stage[0], sc);
    }

    int64_t kt = 0;
    for (; kt + NS <= nk; kt += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s)
            ring_step<C>(ctx, ga(kt + s + NS - 1), gb(kt + s + NS - 1), stage[(s + NS - 1) % NS], stage[s],
                         stage[(s + 1) % NS], f0, acc, gs(kt + s + NS - 1), &sc);
    }
    // the last nk % NS tiles, same stage order
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (kt + s < nk)
            ring_step<C>(ctx, ga(kt + s + NS - 1), gb(kt + s + NS - 1), stage[(s + NS - 1) % NS], stage[s],
                         stage[(s + 1) % NS], f0, acc, gs(kt + s + NS - 1), &sc);
    wait_vmcnt<0>();
    __syncthreads();                         // every load has landed, every wave is done with the stages

    // A K that ends inside a k-tile: the last, partial k-tile goes through stage 0 by ordinary
    // loads, 16-byte chunks at or beyond K written as zeros (K is a whole number of chunks), in
    // the places the DMA loads of a full tile would have filled.
    if (!C::MX && p.K % C::BKE != 0) {                       // (block scales: whole k-tiles only)
        constexpr int CHE = 16 / C::ES;                          // elements per chunk
        const int64_t k0 = nk * C::BKE;
        lds_char *const t0 = (lds_char *)st0;
#pragma unroll
        for (int i = 0; i < C::A_INSTR; ++i) {
            const int q = wave + i * NW, r = 16 * q + (lane >> 2);
            const int c = (lane & 3) ^ ((r >> 2) & 3);
            uintx4 v = uintx4{0, 0, 0, 0};
            if (k0 + c * CHE < p.K) v = *reinterpret_cast<const uintx4 *>(A + ctx.a_off[i] + k0 * C::ES);
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(t0 + q * 1024 + lane * 16) = v;
        }
#pragma unroll
        for (int i = 0; i < C::B_INSTR; ++i) {
            const int q = wave + i * NW;
            uintx4 v = uintx4{0, 0, 0, 0};
            if constexpr (C::B_KC) {
                const int r = 16 * q + (lane >> 2);
                const int c = (lane & 3) ^ ((r >> 2) & 3);
                if (k0 + c * CHE < p.K) v = *reinterpret_cast<const uintx4 *>(B + ctx.b_off[i] + k0 * C::ES);
            } else {
                const int k = (q * 64 + lane) >> 5;
                if (k0 + k < p.K) v = *reinterpret_cast<const uintx4 *>(B + ctx.b_off[i] + k0 * p.ldb * 2);
            }
            *reinterpret_cast<__attribute__((address_space(3))) uintx4 *>(t0 + C::A_BYTES + q * 1024 + lane * 16) = v;
        }
        __syncthreads();
        Frags<C> g0, g1;
        load_frags<C>(ctx, t0, 0, g0);
        load_frags<C>(ctx, t0, 1, g1);
        if constexpr (C::K64) {
#pragma unroll
            for (int j = 0; j < C::TN; ++j)
#pragma unroll
                for (int i = 0; i < C::TM; ++i)
                    acc[j][i] = mfma_32x32x64_f8<C::DT>(g0.b[j], g1.b[j], g0.a[i], g1.a[i], acc[j][i]);
        } else {
            mma_frags<C>(g0, acc);
            mma_frags<C>(g1, acc);
        }
        __syncthreads();                     // stage 0 is the epilogue's slab next
    }

    // Epilogue: bias, activation, bf16 conversion in registers; then each wave passes its tile
    // through a private 32-row slab (WTN*2 bytes per row, 16-byte chunks XOR-swizzled by the row)
    // in stage 0 and stores whole 128-byte lines.  See kernel_tile_direct.hpp.
    const int64_t mw = m0 + wm * C::WTM, nw = n0 + wn * C::WTN;
    const float *bias = p.bias ? p.bias + batch * p.strideBias : nullptr;
    char *Cb = p.C + batch * p.strideC * 2;
    constexpr int CPR = C::WTN / 8, PITCH = C::WTN * 2;       // 16-byte chunks and bytes per slab row
    constexpr int READS = 32 * CPR / 64;
    lds_char *slab = (lds_char *)st0 + wave * (32 * PITCH);  // NW * 32 * PITCH = 32 KiB = one stage
    float bj[TN][4][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const int64_t n = nw + 32 * j + 8 * gq + 4 * half;
            if (bias && !(C::EPI == 0 && p.bias_row) && n + 3 < p.N) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(bias + n);
#pragma unroll
                for (int e = 0; e < 4; ++e) bj[j][gq][e] = v[e];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    bj[j][gq][e] = (bias && !(C::EPI == 0 && p.bias_row) && n + e < p.N) ? bias[n + e] : 0.0f;
            }
        }
    if constexpr (C::EPI == 1) {
        float *part = reinterpret_cast<float *>(p.C);
        const int64_t slice = tile_n * C::WN + wn;
        const bool ragged = nw + C::WTN > p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = mw + 32 * i + frag_row;
            const bool live = m < p.M;
            // this lane holds columns nw + 32 j + 8 gq + 4 half + e of row m; `want` is the label's
            // offset in those terms without the 4 half (or a value no offset takes)
            const int64_t d = live ? (int64_t)p.labels[m] - nw : -1;
            const int want = d >= 0 && d < C::WTN ? (int)d - 4 * half : -1000;
            float mx = -__builtin_inff(), pick = 0.0f;
            bool hit = false;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int cofs = 32 * j + 8 * gq + e;
                        float v = acc[j][i][4 * gq + e] + bj[j][gq][e];
                        if (ragged && nw + cofs + 4 * half >= p.N) v = -__builtin_inff();
                        acc[j][i][4 * gq + e] = v;
                        mx = __builtin_fmaxf(mx, v);
                        if (want == cofs) { pick = v; hit = true; }
                    }
            mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float ref = mx == -__builtin_inff() ? 0.0f : mx;       // a slice wholly past column N
            float sum = 0.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f((acc[j][i][r] - ref) * 1.44269504088896341f);
            sum += __shfl_xor(sum, 32, 64);
            if (live && half == 0)
                *reinterpret_cast<floatx2 *>(part + 2 * (slice * p.M + m)) = floatx2{mx, sum};
            if (live && hit) p.picked[m] = pick;
        }
        return;
    }
    if constexpr (C::EPI == 2) {
        // batches: Z slabs strideC floats apart, each batch its own tiles_n * WN slices of pairs
        float *Z = reinterpret_cast<float *>(p.C) + batch * p.strideC;
        ring::floatx2 *pairs = reinterpret_cast<ring::floatx2 *>(p.picked) + batch * (p.tiles_n * C::WN) * p.M;
        const int64_t slice = tile_n * C::WN + wn;
        const int64_t left = p.N - nw;                                   // columns of this slice inside the matrix
        const float count = (float)(left >= C::WTN ? C::WTN : left > 0 ? left : 0);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t m = mw + 32 * i + frag_row;
            const bool live = m < p.M;
            float sum = 0.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float v = acc[j][i][4 * gq + e] + bj[j][gq][e];
                        acc[j][i][4 * gq + e] = v;
                        sum += (32 * j + 8 * gq + 4 * half + e < left) ? v : 0.0f;
                    }
            sum += __shfl_xor(sum, 32, 64);
            const float mean = count > 0.0f ? sum / count : 0.0f;
            float dev = 0.0f;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float d = (32 * j + 8 * gq + 4 * half + e < left) ? acc[j][i][4 * gq + e] - mean : 0.0f;
                        dev += d * d;
                    }
            dev += __shfl_xor(dev, 32, 64);
            if (live && half == 0) pairs[slice * p.M + m] = ring::floatx2{mean, dev};
            // the 32 x WTN fp32 sub-tile goes through the wave's slab (16-byte chunks XOR-swizzled by the
            // row) so that every store instruction writes whole rows of WTN * 4 contiguous bytes; plain
            // stores: the finishing kernel reads z back next, partly from the caches
            constexpr int ZCH = C::WTN / 4;                              // 16-byte chunks per slab row
            static_assert(4 * 32 * C::WTN * 4 <= C::STAGE_BYTES && C::NW <= 8, "four slabs per stage, two stages");
            lds_char *zslab = (wave < 4 ? (lds_char *)st0 : (lds_char *)st1) + (wave & 3) * (32 * C::WTN * 4);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int gq = 0; gq < 4; ++gq)
                    *reinterpret_cast<__attribute__((address_space(3))) floatx4 *>(
                        zslab + frag_row * (C::WTN * 4) + (((8 * j + 2 * gq + half) ^ (frag_row & (ZCH - 1))) << 4)) =
                        floatx4{acc[j][i][4 * gq], acc[j][i][4 * gq + 1], acc[j][i][4 * gq + 2], acc[j][i][4 * gq + 3]};
#pragma unroll
            for (int q = 0; q < 32 * ZCH / 64; ++q) {
                const int id = q * 64 + lane, row = id / ZCH, chunk = id % ZCH;
                const floatx4 v = *reinterpret_cast<const __attribute__((address_space(3))) floatx4 *>(
                    zslab + row * (C::WTN * 4) + ((chunk ^ (row & (ZCH - 1))) << 4));
                const int64_t mr = mw + 32 * i + row;
                const int c0 = 4 * chunk;
                if (mr < p.M && c0 < left) {
                    float *dst = Z + mr * p.ldc + nw + c0;
                    if (c0 + 4 <= left) {
                        *reinterpret_cast<floatx4 *>(dst) = v;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (c0 + e < left) dst[e] = v[e];
                    }
                }
            }
        }
        return;
    }
    auto slab_key = [](int row) { return CPR == 8 ? (row >> 1) & 7 : row & 15; };
    const int wkey = slab_key(frag_row);
    dispatch_act(p.act, [&](auto act_tag) {
    constexpr int ACT = decltype(act_tag)::value;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        // a bias that runs down the rows: this lane's row of the 32-row group
        const int64_t mb = mw + 32 * i + frag_row;
        const float bi = (bias && p.bias_row && mb < p.M) ? bias[mb] : 0.0f;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = apply_act_bf16out(acc[j][i][4 * gq + e] + (bj[j][gq][e] + bi), ACT);
                *reinterpret_cast<__attribute__((address_space(3))) uintx2 *>(
                    slab + frag_row * PITCH + (((4 * j + gq) ^ wkey) << 4) + 8 * half) =
                    uintx2{pack2_16<C::ODT>(y[0], y[1]), pack2_16<C::ODT>(y[2], y[3])};
            }
#pragma unroll
        for (int q = 0; q < READS; ++q) {
            const int id = q * 64 + lane, row = id / CPR, chunk = id % CPR;
            const uintx4 v = *reinterpret_cast<const __attribute__((address_space(3))) uintx4 *>(
                slab + row * PITCH + ((chunk ^ slab_key(row)) << 4));
            const int64_t m = mw + 32 * i + row, n = nw + chunk * 8;
            if (m < p.M && n < p.N) {
                char *dst = Cb + (m * p.ldc + n) * 2;
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
    }
    });
#endif
}

template <class C>
bool supports(const Problem &p)
{
    if (p.dtype != C::DT || p.a_col() || p.b_col() != C::B_KC) return false;
    if (p.K < C::BKE * C::NS || p.K % (16 / C::ES) != 0 || !vector_friendly(p)) return false;
    if (!C::B_KC && (p.N % 8 != 0)) return false;
    const int64_t a_span = p.M * p.lda * C::ES, b_span = (C::B_KC ? p.N : 32) * p.ldb * C::ES + p.N * C::ES;
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
    hipLaunchKernelGGL(gemm_ring_kernel<C>, dim3((unsigned)total), dim3(C::THREADS), 0, stream, q);
    return hipGetLastError();
}

}  // namespace ring
}  // namespace optiml

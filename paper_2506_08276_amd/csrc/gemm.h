// bf16 MFMA GEMM with fused epilogues for the encoder's four linear maps (gfx950).
#pragma once
#include "common.h"

namespace {

// C[T][N] = A[T][K] * W[N][K]^T + bias (optionally GELU), rounded to bf16.  bf16 operands, fp32 accumulation in
// MFMA 32x32x16.
// Block tile BM x BN, K-slabs of 32, WM x WN waves.  A slab row is four 16-byte chunks; chunk c of row r
// lives at chunk position c ^ ((r >> 2) & 3), so the row-wise stores and the column-of-rows MFMA operand reads
// both spread over all LDS banks.
// Software pipeline (slab s): global loads into one of four register sets at iteration s-5 (memory latency
// under load is several slabs long), LDS store into a ring of three stages in the middle of iteration s-2,
// first operand fragments read at the end of iteration s-1, MFMAs at iteration s.  One barrier per slab, and
// no wave waits on LDS right after it.  The last four iterations of a tile fetch the first four slabs of the
// block's next tile instead, so those are in registers when the epilogue ends.
// The 256x256 tile (eight waves of 128x64) halves the bytes fetched from L2 per flop compared with 128x128,
// which is what bounds the small tile.  Each output element is one fixed-order sum over K: a row's result does
// not depend on T.
// Vector-memory loads return in order, so a wait for any load is a wait for every load issued before it.  The
// kernel is written so that no wait falls behind the prefetched slabs: no register spills (a reload is a load),
// no load whose result is unused, the bias fetched ahead of the slabs and kept in LDS, per-lane values of the
// epilogue recomputed per tile instead of held in registers.
enum { EPI_BIAS = 0, EPI_BIAS_GELU = 1 };

// GELU(v) = v Phi(v) with the normal distribution function written as a logistic function of an odd polynomial,
// Phi(v) ~ 1 / (1 + 2^(-v p(v^2))), p(u) = c0 + c1 u + c2 u^2 fitted to the exact erf form (minimax over |v| <= 9):
// |error| <= 2.6e-5, below the bf16 rounding of the result wherever the result matters.  v^2 is clamped where
// Phi has saturated in fp32 (p would turn over beyond).  One hardware exponential and one reciprocal.
__device__ inline float gelu_erf(float v)
{
    const float u = fminf(v * v, 50.0f);
    const float p = fmaf(u, fmaf(u, 0.0010142733f, -0.10677579f), -2.3011213f);  // -p(u)
    return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(v * p));  // raw 2^x: overflow gives inf -> 0, underflow 0 -> v
}

constexpr int GEMM_BK = 32;

// dynamic LDS of a block: three operand stages and, per wave, the bias of its 64 output columns
template <int BM, int BN, int WM, int WN>
constexpr int gemm_smem_bytes()
{
    return 3 * (BM + BN) * GEMM_BK * (int)sizeof(bf16_t) + WM * WN * 64 * (int)sizeof(float);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(64 * WM * WN, (WM * WN <= 4) ? 2 : 1) void gemm_kernel(
    const bf16_t *__restrict__ A, const bf16_t *__restrict__ W, const float *__restrict__ bias,
    bf16_t *__restrict__ out, const int32_t *__restrict__ T_dev, int N, int K, int tiles_n, int gcols)
{
    constexpr int BK = GEMM_BK;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *As = reinterpret_cast<bf16_t *>(smem);  // [3][BM][BK]
    bf16_t *Bs = As + 3 * BM * BK;                  // [3][BN][BK]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // the same for the whole wave: a scalar register
    float *wbias = reinterpret_cast<float *>(Bs + 3 * BN * BK) + wave * 64;  // this wave's 64 bias values
    const int wm = wave / WN, wn = wave % WN;
    constexpr int NT = 64 * WM * WN;                     // threads per block
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;  // 32x32 MFMA tiles per wave
    constexpr int RPP = NT / 4;                          // rows one pass of the block's threads covers

    // Persistent blocks: the grid is one block per CU slot and every block walks over tiles, so the output stores
    // of one tile drain while the next tile's operands are already being fetched (with one block per CU nothing
    // else would hide them).  Blocks go round-robin to the 8 XCDs: block b sits on XCD b % 8.  At step j the
    // blocks of one XCD take a contiguous run of tiles (same A rows, all column tiles), so the A slab is reused out
    // of that XCD's L2 (measured: 2.3x fewer bytes fetched by the QKV GEMM than with the plain tile order).
    // When W is larger than an XCD's L2 and the output is wide (FFN1), the host splits the column tiles into groups
    // (gcols tiles each): an XCD then works with part of W only, which stays in its L2, at the price of reading A
    // once per group.
    const int T = *T_dev;
    const int n_tiles = ((T + BM - 1) / BM) * tiles_n;
    const int per_xcd = (n_tiles + 7) >> 3;
    const int blocks_per_xcd = gridDim.x >> 3;  // the host launches a multiple of 8 blocks
    constexpr int ACH = BM / RPP, BCH = BN / RPP;  // 16-byte chunks per thread and K-slab
    u32x4 ra0[ACH], rb0[BCH], ra1[ACH], rb1[BCH], ra2[ACH], rb2[BCH], ra3[ACH], rb3[BCH];
    const int lrow = tid >> 2, lc = tid & 3;
    const int soff = lrow * BK + ((lc ^ ((lrow >> 2) & 3)) << 3);  // rows RPP apart share the swizzle term

    // Operand loads are buffer loads: a descriptor per tile (scalar registers: base of the tile's BM or BN rows, size
    // of those rows, so a load can never leave the tile), one 32-bit byte offset per thread that A and W share, and a
    // scalar offset for the chunk and the K-slab.  No 64-bit vector address arithmetic and no per-thread pointers.
    const int toff = (lrow * K + lc * 8) * (int)sizeof(bf16_t);
#define GEMM_RSRC(ptr, rows)                                                                             \
    __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(ptr), 0, (rows) * K * (int)sizeof(bf16_t), 0x00020000)
#define GEMM_GLOAD(RA, RB, AP, WP, k0)                                                                   \
    _Pragma("unroll") for (int i = 0; i < ACH; ++i)                                                      \
        RA[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(AP, toff, ((RPP * i) * K + (k0)) * 2, 0)); \
    _Pragma("unroll") for (int i = 0; i < BCH; ++i)                                                      \
        RB[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(WP, toff, ((RPP * i) * K + (k0)) * 2, 0));
#define GEMM_SSTORE(RA, RB, stage)                                                                       \
    _Pragma("unroll") for (int i = 0; i < ACH; ++i)                                                      \
        *reinterpret_cast<u32x4 *>(As + (stage) * BM * BK + RPP * BK * i + soff) = RA[i];                 \
    _Pragma("unroll") for (int i = 0; i < BCH; ++i)                                                      \
        *reinterpret_cast<u32x4 *>(Bs + (stage) * BN * BK + RPP * BK * i + soff) = RB[i];


    // operand fragments: lane l reads row (l & 31) of a 32-row block, 16-byte chunk 2*ks + (l >> 5).  The block's
    // first row is a multiple of 32, so the swizzle term depends on the lane only: two offsets serve every block.
    int foff[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) foff[ks] = (lane & 31) * BK + (((ks * 2 + (lane >> 5)) ^ ((lane >> 2) & 3)) << 3);
#define GEMM_FRAGS(AF, BF, stage, ks)                                                                    \
    _Pragma("unroll") for (int mi = 0; mi < TM; ++mi)                                                    \
        AF[mi] = *reinterpret_cast<const bf16x8 *>(As + (stage) * BM * BK + (wm * (BM / WM) + mi * 32) * BK + foff[ks]); \
    _Pragma("unroll") for (int ni = 0; ni < TN; ++ni)                                                    \
        BF[ni] = *reinterpret_cast<const bf16x8 *>(Bs + (stage) * BN * BK + (wn * (BN / WN) + ni * 32) * BK + foff[ks]);
#define GEMM_MFMA(AF, BF)                                                                                \
    _Pragma("unroll") for (int mi = 0; mi < TM; ++mi)                                                    \
        _Pragma("unroll") for (int ni = 0; ni < TN; ++ni)                                                \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(BF[ni], AF[mi], acc[mi][ni], 0, 0, 0);
    // One iteration: LOAD prefetches slab kt+5 (or a slab of the next tile), the MFMAs multiply slab kt (its first
    // fragments are already in af0/bf0), STORE puts slab kt+2 into the ring while the MFMAs run, and the first
    // fragments of slab kt+1 are read.
#define GEMM_ITER(LOAD, STORE)                                                                           \
    {                                                                                                    \
        __builtin_amdgcn_sched_barrier(0);                                                               \
        LOAD                                                                                             \
        GEMM_FRAGS(af1, bf1, st_cur, 1)                                                                  \
        GEMM_MFMA(af0, bf0)                                                                              \
        STORE                                                                                            \
        GEMM_FRAGS(af0, bf0, st_nxt, 0)                                                                  \
        GEMM_MFMA(af1, bf1)                                                                              \
        GEMM_INTERLEAVE                                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                               \
        __syncthreads();                                                                                 \
        const int t_ = st_cur;                                                                           \
        st_cur = st_nxt;                                                                                 \
        st_nxt = st_nn;                                                                                  \
        st_nn = t_;                                                                                      \
    }
    // Issue order inside an iteration.  A wave issues in order, and all waves of the block run the same schedule
    // at the same time: a burst of global loads (16 cycles each in the address unit) or LDS stores fills the
    // memory pipes' queues and holds back the MFMAs behind it.  So the memory instructions are spread evenly
    // between the MFMAs: fragment reads for the second half first, one global load and one LDS store every four
    // MFMAs, the next slab's first fragments once the first half's MFMAs no longer need those registers.
#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0);
#define GEMM_INTERLEAVE                                                                                  \
    if constexpr (TM * TN == 8 && TM + TN == 6 && ACH + BCH == 4) {                                      \
        SGB(0x008, 1) SGB(0x100, 2) SGB(0x008, 1) SGB(0x020, 1) SGB(0x008, 1) SGB(0x100, 2) SGB(0x008, 1) SGB(0x200, 1) \
        SGB(0x008, 1) SGB(0x100, 2) SGB(0x008, 1) SGB(0x020, 1) SGB(0x008, 1) SGB(0x200, 1) SGB(0x008, 1)               \
        SGB(0x008, 1) SGB(0x100, 2) SGB(0x008, 1) SGB(0x020, 1) SGB(0x008, 1) SGB(0x100, 2) SGB(0x008, 1) SGB(0x200, 1) \
        SGB(0x008, 1) SGB(0x100, 2) SGB(0x008, 1) SGB(0x020, 1) SGB(0x008, 1) SGB(0x200, 1) SGB(0x008, 1)               \
    } else {                                                                                             \
        _Pragma("unroll") for (int i_ = 0; i_ < (TM + TN + 1) / 2; ++i_) { SGB(0x008, 1) SGB(0x100, 2) } \
        _Pragma("unroll") for (int i_ = 0; i_ < ACH + BCH; ++i_) { SGB(0x008, 1) SGB(0x020, 1) }         \
        _Pragma("unroll") for (int i_ = 0; i_ < ACH + BCH; ++i_) { SGB(0x008, 1) SGB(0x200, 1) }         \
        _Pragma("unroll") for (int i_ = 0; i_ < (TM + TN + 1) / 2; ++i_) { SGB(0x008, 1) SGB(0x100, 2) } \
        SGB(0x008, 2 * TM * TN)                                                                          \
    }

    // tile of this block at a step of its walk (uniform for the block); false when the walk is over.  The logical
    // order goes through the column tiles in groups of gcols: all row blocks for the first group, then for the
    // next (gcols = tiles_n: plain row-major order).  An XCD's contiguous share then lies in one group, or two.
    const int tiles_m = n_tiles / tiles_n;
#define GEMM_TILE_AT(step_, ok_, tm_, tn_)                                                               \
    {                                                                                                    \
        const int in_xcd_ = (step_) * blocks_per_xcd + (int)(blockIdx.x >> 3);                           \
        const int logical_ = (int)(blockIdx.x & 7) * per_xcd + in_xcd_;                                  \
        ok_ = in_xcd_ < per_xcd && logical_ < n_tiles;                                                   \
        if (ok_) {                                                                                       \
            const int g_ = logical_ / (tiles_m * gcols);                                                 \
            const int r_ = logical_ - g_ * tiles_m * gcols;                                              \
            const int cg_ = min(gcols, tiles_n - g_ * gcols);                                            \
            tm_ = r_ / cg_;                                                                              \
            tn_ = g_ * gcols + r_ % cg_;                                                                 \
        }                                                                                                \
    }
    bool have;
    int tile_m = 0, tile_n = 0;
    GEMM_TILE_AT(0, have, tile_m, tile_n)
    if (!have) return;
    const int KT = K / BK;  // a multiple of 4: the host checks K % (4 * BK) == 0
    // The large tile is launched for K >= 8 slabs only (the host checks): without the short-K paths the compiler
    // does not have to merge their pending loads into the waits of the long-K path.
    if constexpr (BM * BN > 128 * 128) __builtin_assume(KT >= 8);
    auto ag = GEMM_RSRC(A + (size_t)tile_m * BM * K, BM);
    auto wg = GEMM_RSRC(W + (size_t)tile_n * BN * K, BN);
    // The bias of a tile is fetched before the tile's first operand slab and put into LDS at the start of the tile:
    // a load issued in the epilogue would complete only after the next tile's prefetched slabs (loads return in
    // order), and the epilogue would wait for all of them.
    float bnext = bias[tile_n * BN + wn * (BN / WN) + lane];
    GEMM_GLOAD(ra0, rb0, ag, wg, 0)
    GEMM_GLOAD(ra1, rb1, ag, wg, BK)
    GEMM_GLOAD(ra2, rb2, ag, wg, 2 * BK)
    GEMM_GLOAD(ra3, rb3, ag, wg, 3 * BK)
  for (int step = 0;; ++step) {
    // the tile after this one; without one the prefetch at the end of the K loop re-reads this tile (in bounds, unused)
    bool have_next;
    int next_m = tile_m, next_n = tile_n;
    GEMM_TILE_AT(step + 1, have_next, next_m, next_n)
    const auto ag_next = GEMM_RSRC(A + (size_t)next_m * BM * K, BM);
    const auto wg_next = GEMM_RSRC(W + (size_t)next_n * BN * K, BN);
    // Slabs 0..3 of this tile are in the four register sets.  Steady state of the K loop at iteration 0: slabs 0 and
    // 1 in the ring, slabs 2, 3, 4 in sets 1, 2, 3, set 0 free.
    bf16x8 af0[TM], bf0[TN], af1[TM], bf1[TN];
    wbias[lane] = bnext;
    GEMM_SSTORE(ra0, rb0, 0)
    GEMM_SSTORE(ra1, rb1, 1)
    // The accumulators start at the bias instead of zero (the sum over K is added on top in the matrix pipe), so the
    // epilogue has no additions and no bias reads left: it costs as many register moves here as clearing did.  A
    // lane owns, in registers 4g..4g+3 of accumulator (mi, ni), the columns ni*32 + 8g + 4*(lane/32) + 0..3 of the
    // wave's 64; LDS serves a wave's accesses in order, so the reads see this wave's own store above.
    f32x16 acc[TM][TN];
    {
        const float *bq = wbias + 4 * (lane >> 5);
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(bq + ni * 32 + 8 * g);  // one address per half-wave: a broadcast
#pragma unroll
                for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[mi][ni][4 * g + i] = bv[i];
            }
    }
#pragma unroll
    for (int i = 0; i < ACH; ++i) { ra1[i] = ra2[i]; ra2[i] = ra3[i]; }
#pragma unroll
    for (int i = 0; i < BCH; ++i) { rb1[i] = rb2[i]; rb2[i] = rb3[i]; }
    if (KT > 4) { GEMM_GLOAD(ra3, rb3, ag, wg, 4 * BK) }
    __syncthreads();
    GEMM_FRAGS(af0, bf0, 0, 0)
    int st_cur = 0, st_nxt = 1, st_nn = 2;
    // Every load is of a slab that exists: the last group of four before the tail has one load fewer.  (A load
    // whose result nobody uses costs more than its bytes: its registers are reused at once, and that has to wait for
    // it and, as loads return in order, for every load issued before it.)
    for (int kt = 0; kt < KT - 8; kt += 4) {
        GEMM_ITER(GEMM_GLOAD(ra0, rb0, ag, wg, (kt + 5) * BK), GEMM_SSTORE(ra1, rb1, st_nn))
        GEMM_ITER(GEMM_GLOAD(ra1, rb1, ag, wg, (kt + 6) * BK), GEMM_SSTORE(ra2, rb2, st_nn))
        GEMM_ITER(GEMM_GLOAD(ra2, rb2, ag, wg, (kt + 7) * BK), GEMM_SSTORE(ra3, rb3, st_nn))
        GEMM_ITER(GEMM_GLOAD(ra3, rb3, ag, wg, (kt + 8) * BK), GEMM_SSTORE(ra0, rb0, st_nn))
    }
    if (KT >= 8) {
        GEMM_ITER(GEMM_GLOAD(ra0, rb0, ag, wg, (KT - 3) * BK), GEMM_SSTORE(ra1, rb1, st_nn))
        GEMM_ITER(GEMM_GLOAD(ra1, rb1, ag, wg, (KT - 2) * BK), GEMM_SSTORE(ra2, rb2, st_nn))
        GEMM_ITER(GEMM_GLOAD(ra2, rb2, ag, wg, (KT - 1) * BK), GEMM_SSTORE(ra3, rb3, st_nn))
        GEMM_ITER(, GEMM_SSTORE(ra0, rb0, st_nn))
    }
    // last four slabs: slabs KT-2 and KT-1 still go into the ring; the loads fetch the next tile
    bnext = bias[next_n * BN + wn * (BN / WN) + lane];
    GEMM_ITER(GEMM_GLOAD(ra0, rb0, ag_next, wg_next, 0), GEMM_SSTORE(ra1, rb1, st_nn))
    GEMM_ITER(GEMM_GLOAD(ra1, rb1, ag_next, wg_next, BK), GEMM_SSTORE(ra2, rb2, st_nn))
    GEMM_ITER(GEMM_GLOAD(ra2, rb2, ag_next, wg_next, 2 * BK), )
    GEMM_ITER(GEMM_GLOAD(ra3, rb3, ag_next, wg_next, 3 * BK), )

    // Epilogue.  The MFMAs take the W fragment as their first operand, so a 32x32 accumulator holds the transposed
    // output block: lane l owns output row l%32 and, in registers 4g..4g+3, the four adjacent columns
    // 8g + 4*(l/32) + 0..3.  Each wave passes 32 rows at a time through its own 4 KB of LDS: 8-byte stores of four
    // bf16 (unit u of a row sits at position u ^ swz(row): the 16 lanes served together hit all banks once), then
    // 16-byte reads, so that the global stores are whole 128-byte row segments per 8 lanes.
    __syncthreads();  // every wave is done with the operand stages
    constexpr int WCOLS = BN / WN;
    static_assert(WCOLS == 64, "the epilogue's staging layout is written for 64 output columns per wave");
    unsigned char *stg = smem + wave * (2 * 32 * 128);  // two slices per wave, used in turn
    const int col0 = tile_n * BN + wn * WCOLS;
    const int row0 = tile_m * BM + wm * (BM / WM);
    // What the epilogue derives from the lane is computed here, per tile, instead of occupying registers through the
    // K loop (the empty statement keeps the compiler from hoisting it).
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    const int half = lane_e >> 5, l32 = lane_e & 31;
    const int wswz = ((l32 & 7) << 1) | ((l32 >> 3) & 1);
    // write-out: a wave-wide access covers 8 rows of eight 16-byte chunks.  The output is read by a later kernel
    // only: streaming stores keep it from displacing the operand slabs in L2 (measured: 3-7% per GEMM).
    const int orow = lane_e >> 3, och = lane_e & 7;
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
        unsigned char *sl = stg + (mi & 1) * (32 * 128);  // the other slice than the previous 32 rows: their reads may still be on their way
#pragma unroll
        for (int ni = 0; ni < TN; ++ni)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                bf16x4 o4;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = acc[mi][ni][4 * g + i];  // the bias is in the sum already
                    o4[i] = (bf16_t)(EPI == EPI_BIAS_GELU ? gelu_erf(v) : v);
                }
                const int u = ni * 8 + 2 * g + half;
                *reinterpret_cast<bf16x4 *>(sl + l32 * 128 + ((u ^ wswz) << 3)) = o4;
            }
        __builtin_amdgcn_wave_barrier();  // LDS serves a wave's accesses in order: the reads below see the writes
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int lr = j * 8 + orow;
            u32x4 v = *reinterpret_cast<const u32x4 *>(sl + lr * 128 + ((och ^ orow) << 4));
            if (j & 1) v = u32x4{v[2], v[3], v[0], v[1]};  // rows 8..15 and 24..31 hold the halves of a chunk swapped
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(out + (size_t)(row0 + mi * 32 + lr) * N + col0 + och * 8));
        }
    }
    __syncthreads();  // the staging slices are operand stages again for the next tile
    if (!have_next) break;
    tile_m = next_m;
    tile_n = next_n;
    ag = ag_next;
    wg = wg_next;
  }
#undef GEMM_TILE_AT
#undef GEMM_GLOAD
#undef GEMM_RSRC
#undef GEMM_SSTORE
#undef GEMM_FRAGS
#undef GEMM_MFMA
#undef GEMM_ITER
#undef GEMM_INTERLEAVE
#undef SGB
}

}  // namespace

// Encoder forward pass for embedding recomputation (LEANN Alg. 2, the recomputation step; Sec. 3 online
// stage), written for gfx950: bf16 MFMA GEMMs with LDS-staged, swizzled tiles, an MFMA attention kernel
// working on ragged (token-packed) batches, and fp32 LayerNorm / pooling.
//
// Tokens of all chunks of a pass are packed back to back (no padding rows): chunk i owns rows
// cu[i] .. cu[i+1] of every activation matrix.  The number of valid rows T is only known on the device,
// so grids are sized for the worst case and blocks beyond T leave at once.
#include <algorithm>

#include "common.h"
#include "gemm.h"

namespace {

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ------------------------------------------------------------------ pass set-up
// lengths of the requested chunks -> exclusive prefix sum cu[0..n], cu[n] = T.  One block of 1024 threads.
__global__ __launch_bounds__(1024) void prep_kernel(const int32_t *__restrict__ lengths, const int64_t *__restrict__ ids,
                                                    int64_t first_id, int n, int64_t n_store, int seq,
                                                    int32_t *__restrict__ cu, int64_t *__restrict__ chunk_of,
                                                    int *__restrict__ err, int64_t *__restrict__ tok_count,
                                                    int64_t *__restrict__ tok_count2)
{
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (n + 1023) / 1024;
    const int beg = tid * per, end = min(n, beg + per);
    int s = 0;
    for (int i = beg; i < end; ++i) {
        int64_t id = ids ? ids[i] : first_id + i;
        int len = 0;
        if (id < 0 || id >= n_store) {
            atomicOr(err, 1);
            id = 0;
        } else {
            len = lengths[id];
            if (len < 1 || len > seq) {
                atomicOr(err, 2);
                len = 0;
            }
        }
        chunk_of[i] = id;
        cu[i] = len;  // temporarily the length
        s += len;
    }
    part[tid] = s;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        int v = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int run = tid ? part[tid - 1] : 0;
    for (int i = beg; i < end; ++i) {
        int len = cu[i];
        cu[i] = run;
        run += len;
    }
    if (tid == 1023) {
        cu[n] = part[1023];
        if (tok_count) *tok_count += part[1023];
        if (tok_count2) *tok_count2 += part[1023];
    }
}

// ------------------------------------------------------------------ embedding + LayerNorm
// one wave per (chunk, position); x[cu[i]+t] = LN(tok_emb[id] + pos_emb[t] + seg_emb) in bf16
__global__ __launch_bounds__(256) void embed_ln_kernel(const int32_t *__restrict__ tokens, const int64_t *__restrict__ chunk_of,
                                                       const int32_t *__restrict__ cu, int n, int seq, int d, int vocab,
                                                       const bf16_t *__restrict__ tok_emb, const bf16_t *__restrict__ pos_emb,
                                                       const bf16_t *__restrict__ seg_emb, const float *__restrict__ g,
                                                       const float *__restrict__ b, float eps, bf16_t *__restrict__ x,
                                                       int *__restrict__ err)
{
    const int lane = threadIdx.x & 63;
    const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int i = (int)(w / seq), t = (int)(w % seq);
    if (i >= n) return;
    const int row0 = cu[i], len = cu[i + 1] - row0;
    if (t >= len) return;
    int tok = tokens[chunk_of[i] * seq + t];
    if (tok < 0 || tok >= vocab) {
        if (lane == 0) atomicOr(err, 4);
        tok = 0;
    }
    // a lane owns 16-byte pieces (8 elements) j*64 + lane of the row, as in the residual LayerNorm below
    const int pieces = d >> 3;
    const bf16_t *te = tok_emb + (size_t)tok * d, *pe = pos_emb + (size_t)t * d;
    float v[2][8];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (j * 64 + lane < pieces) {
            const int c0 = (j * 64 + lane) * 8;
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(te + c0);
            const bf16x8 p = *reinterpret_cast<const bf16x8 *>(pe + c0);
            const bf16x8 sg = *reinterpret_cast<const bf16x8 *>(seg_emb + c0);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[j][i] = (float)a[i] + (float)p[i] + (float)sg[i];
                s += v[j][i];
            }
        }
    const float mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (j * 64 + lane < pieces) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float c = v[j][i] - mean;
                q += c * c;
            }
        }
    const float inv = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
    bf16_t *xr = x + (size_t)(row0 + t) * d;
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (j * 64 + lane < pieces) {
            const int c0 = (j * 64 + lane) * 8;
            const f32x4 g0 = *reinterpret_cast<const f32x4 *>(g + c0), g1 = *reinterpret_cast<const f32x4 *>(g + c0 + 4);
            const f32x4 b0 = *reinterpret_cast<const f32x4 *>(b + c0), b1 = *reinterpret_cast<const f32x4 *>(b + c0 + 4);
            bf16x8 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                o[i] = (bf16_t)((v[j][i] - mean) * inv * g0[i] + b0[i]);
                o[i + 4] = (bf16_t)((v[j][i + 4] - mean) * inv * g1[i] + b1[i]);
            }
            *reinterpret_cast<bf16x8 *>(xr + c0) = o;
        }
}

// ------------------------------------------------------------------ residual add + LayerNorm, in place
// x[row] = LN(x[row] + delta[row]): delta is a sublayer's output (bf16, written by the O / FFN2 GEMM), the sum, the
// statistics and the normalisation are fp32.  One wave per row, the whole row in registers before anything is
// written.  A lane owns 16-byte pieces (8 elements) j*64 + lane of the row (row length a multiple of 8, at most
// 1024).  Two-pass statistics on the registers: mean, then the biased variance of the centred values.
__global__ __launch_bounds__(256) void ln_kernel(const bf16_t *__restrict__ delta, const float *__restrict__ g,
                                                 const float *__restrict__ b, bf16_t *__restrict__ x,
                                                 const int32_t *__restrict__ T_dev, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int T = *T_dev;
    const int pieces = d >> 3;
    const int nwaves = gridDim.x * 4;
    int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= T) return;
    // a wave goes through rows row, row + nwaves, ...: the scale and shift of its pieces stay in registers, and the
    // next row's loads are issued before the current row's arithmetic
    f32x4 gg[2][2], bb[2][2];
    bf16x8 dn[2], xn[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (j * 64 + lane < pieces) {
            const int c0 = (j * 64 + lane) * 8;
            gg[j][0] = *reinterpret_cast<const f32x4 *>(g + c0);
            gg[j][1] = *reinterpret_cast<const f32x4 *>(g + c0 + 4);
            bb[j][0] = *reinterpret_cast<const f32x4 *>(b + c0);
            bb[j][1] = *reinterpret_cast<const f32x4 *>(b + c0 + 4);
            dn[j] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(delta + (size_t)row * d + c0));
            xn[j] = *reinterpret_cast<const bf16x8 *>(x + (size_t)row * d + c0);
        }
    for (; row < T; row += nwaves) {
        bf16_t *xr = x + (size_t)row * d;
        float v[2][8];
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (j * 64 + lane < pieces) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    v[j][i] = (float)xn[j][i] + (float)dn[j][i];
                    s += v[j][i];
                }
            }
        const int next = row + nwaves;
        if (next < T) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (j * 64 + lane < pieces) {
                    const int c0 = (j * 64 + lane) * 8;
                    dn[j] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(delta + (size_t)next * d + c0));
                    xn[j] = *reinterpret_cast<const bf16x8 *>(x + (size_t)next * d + c0);
                }
        }
        const float mean = wave_sum(s) / (float)d;
        float q = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (j * 64 + lane < pieces) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float c = v[j][i] - mean;
                    q += c * c;
                }
            }
        const float inv = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (j * 64 + lane < pieces) {
                bf16x8 o;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    o[i] = (bf16_t)((v[j][i] - mean) * inv * gg[j][0][i] + bb[j][0][i]);
                    o[i + 4] = (bf16_t)((v[j][i + 4] - mean) * inv * gg[j][1][i] + bb[j][1][i]);
                }
                *reinterpret_cast<bf16x8 *>(xr + (j * 64 + lane) * 8) = o;
            }
    }
}

// ------------------------------------------------------------------ attention
// One block per (chunk, head), head size 64, up to 256 keys.  K (row-major, swizzled) and V^T live in LDS.
// Each wave takes 32 query rows at a time and computes S^T = K Q^T with MFMA, so that a lane owns one
// query column: the softmax reductions run over the lane's own registers plus one exchange with lane^32.
// P^T (bf16) then feeds O^T = V^T P^T directly from registers: accumulator registers 8u..8u+7 of key tile t
// are exactly the eight k-slots of one MFMA step when V^T is read with the matching key order.
// NKT = key tiles (of 32) the block can hold: 4 for sequences up to 128 (half the registers and LDS, twice the
// blocks per CU), 8 for up to 256.
template <int NKT>
struct AttCfg {
    static constexpr int LP = NKT * 32;           // padded key capacity = V^T row pitch (bf16)
    static constexpr int KV_BYTES = (LP * 64 + 64 * LP) * (int)sizeof(bf16_t);
    static constexpr int SMEM = KV_BYTES + 4 * 16 * 128;  // plus, per wave, 16 output rows of 64 bf16
};

// V^T in LDS: row = output dimension (64 of them), LP keys per row in 16-byte groups of eight.  Inside a group of 16
// keys the order follows the MFMA operand slots of P^T (a lane of half h holds, in slots 0..7, keys 4h + 0..3 and
// 8 + 4h + 0..3): stored position 16j + 8h + slot, so that a lane's operand is one 16-byte read.  The group index is
// XORed with a function of the row: the 16 rows that one pass of a 16-byte read serves, and the (chunk, half) pairs
// that one pass of the staging stores serves, then fall into 16 different bank groups (no bank conflicts either way).
__device__ inline int vt_swizzle(int row) { return (row & 15) ^ (((row >> 4) & 3) << 1); }

template <int NKT>
__global__ __launch_bounds__(256, NKT == 4 ? 3 : 2) void attention_kernel(const bf16_t *__restrict__ qkv,
                                                                          const int32_t *__restrict__ cu,
                                                                          bf16_t *__restrict__ out, int d,
                                                                          float scale_log2e)
{
    constexpr int LP = AttCfg<NKT>::LP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *Ks = reinterpret_cast<bf16_t *>(smem);  // [LP][64], 16-byte chunks XOR-swizzled by row
    bf16_t *Vt = Ks + LP * 64;                      // [64][LP], see vt_swizzle
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // consecutive blocks are the heads of one chunk: they read adjacent 128-byte pieces of the same QKV rows at
    // about the same time
    const int H = d >> 6;
    const int c = blockIdx.x / H, h = blockIdx.x % H;
    const int t0 = cu[c], L = cu[c + 1] - t0;
    if (L <= 0) return;
    const int nkt = (L + 31) >> 5;
    const int Lp = nkt << 5;
    const size_t ld = (size_t)3 * d;
    const bf16_t *kbase = qkv + (size_t)t0 * ld + d + h * 64;
    const bf16_t *vbase = qkv + (size_t)t0 * ld + 2 * d + h * 64;
    const int half = lane >> 5, l32 = lane & 31;

    // the wave's first query block goes to registers while K and V are on their way to LDS
    bf16x8 qf[4];
    {
        const int qload = min(wave * 32 + l32, L - 1);
        const bf16_t *qp = qkv + (size_t)(t0 + qload) * ld + h * 64;
#pragma unroll
        for (int s = 0; s < 4; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + s * 16 + half * 8);
    }
    // Staging.  All global loads of the thread are issued before the first LDS store.  Keys >= L are zero.
    // V: thread (j16, hf, ch) takes the eight keys 16 j16 + 4 hf + {0..3, 8..11} of the 16-byte chunk ch (eight
    // output dimensions) and writes, per dimension, the eight keys as one 16-byte group.  Eight adjacent lanes read
    // one whole 128-byte piece of a V row.
    // K: rows as they are, 16-byte chunk ch of row key at position ch ^ ((key >> 1) & 7).
    {
        const int ch = tid & 7, hf = (tid >> 3) & 1, j16 = tid >> 4;
        const bool v_on = j16 * 16 < Lp;
        u32x4 vv[8], kk[NKT];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            const int key = j16 * 16 + 4 * hf + (r & 3) + 8 * (r >> 2);
            vv[r] = u32x4{0, 0, 0, 0};
            if (v_on && key < L) vv[r] = *reinterpret_cast<const u32x4 *>(vbase + (size_t)key * ld + ch * 8);
        }
#pragma unroll
        for (int r = 0; r < NKT; ++r) {
            const int key = r * 32 + (tid >> 3);
            kk[r] = u32x4{0, 0, 0, 0};
            if (key < L) kk[r] = *reinterpret_cast<const u32x4 *>(kbase + (size_t)key * ld + ch * 8);
        }
#pragma unroll
        for (int r = 0; r < NKT; ++r) {
            const int key = r * 32 + (tid >> 3);
            if (key < Lp) *reinterpret_cast<u32x4 *>(Ks + key * 64 + ((ch ^ ((key >> 1) & 7)) << 3)) = kk[r];
        }
        if (v_on) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {  // output dimension ch * 8 + i: element i of each of the eight key rows
                u32x4 o;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t a = vv[2 * w][i >> 1], b = vv[2 * w + 1][i >> 1];
                    o[w] = (i & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
                }
                const int row = ch * 8 + i;
                *reinterpret_cast<u32x4 *>(Vt + row * LP + (((2 * j16 + hf) ^ vt_swizzle(row)) << 3)) = o;
            }
        }
    }
    __syncthreads();

    for (int qb = wave; qb < nkt; qb += 4) {
        const int qrow = qb * 32 + l32;
        if (qb != wave) {
            const int qload = min(qrow, L - 1);
            const bf16_t *qp = qkv + (size_t)(t0 + qload) * ld + h * 64;
#pragma unroll
            for (int s = 0; s < 4; ++s) qf[s] = *reinterpret_cast<const bf16x8 *>(qp + s * 16 + half * 8);
        }
        f32x16 sc[NKT];
#pragma unroll
        for (int t = 0; t < NKT; ++t) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[t][r] = 0.f;
            if (t < nkt) {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int row = t * 32 + l32, ch = s * 2 + half;
                    bf16x8 kf = *reinterpret_cast<const bf16x8 *>(Ks + row * 64 + ((ch ^ ((row >> 1) & 7)) << 3));
                    sc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sc[t], 0, 0, 0);
                }
            }
        }
        // lane owns query column l32 and keys 32t + 8(r/4) + 4*half + r%4; only the last tile can hold keys >= L.
        // The bound is re-read per query block (the empty statement hides that it does not change): hoisted out of
        // the loop, the 128 comparison results of the unrolled tiles would be kept in scalar registers and spilled.
        int l_cmp = L - 4 * half;
        asm volatile("" : "+v"(l_cmp));
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < NKT; ++t)
            if (t < nkt) {
                if (t == nkt - 1) {
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (t * 32 + 8 * (r >> 2) + (r & 3) >= l_cmp) sc[t][r] = -INFINITY;
                }
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[t][r]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float moff = mx * scale_log2e;
        float den = 0.f;
#pragma unroll
        for (int t = 0; t < NKT; ++t)
            if (t < nkt) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = __builtin_amdgcn_exp2f(sc[t][r] * scale_log2e - moff);  // argument <= 0: no overflow, underflow to 0 is exact enough
                    sc[t][r] = p;
                    den += p;
                }
            }
        den += __shfl_xor(den, 32, 64);

        f32x16 oacc[2];
#pragma unroll
        for (int dt = 0; dt < 2; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
#pragma unroll
        for (int t = 0; t < NKT; ++t)
            if (t < nkt) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    bf16x8 pf;
#pragma unroll
                    for (int i = 0; i < 8; ++i) pf[i] = (bf16_t)sc[t][8 * u + i];
                    const int pg = 4 * t + 2 * u + half;  // the lane's group: slots 0..3 = keys 32t + 16u + 4 half + 0..3, slots 4..7 = those + 8
#pragma unroll
                    for (int dt = 0; dt < 2; ++dt) {
                        const int row = dt * 32 + l32;
                        const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(Vt + row * LP + ((pg ^ vt_swizzle(row)) << 3));
                        oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[dt], 0, 0, 0);
                    }
                }
            }
        // The lane owns query l32 and, per (dt, g), the four adjacent outputs dt*32 + 8g + 4*half + 0..3.  Sixteen
        // queries at a time go through the wave's own 2 KB of LDS (8-byte unit u of a row at position u ^ swz(row):
        // the 16 lanes served together hit all banks once), so that the global stores are 16 bytes per lane and
        // whole 128-byte lines per 8 lanes (stores of 8 bytes per lane to 32 rows cost a quarter of the kernel's time).
        const float inv = 1.0f / den;
        unsigned char *ostg = smem + AttCfg<NKT>::KV_BYTES + wave * (16 * 128);
        const int r16 = l32 & 15;
        const int wswz = ((r16 & 7) << 1) | (r16 >> 3);
        const int orow = lane >> 3, och = lane & 7;
#pragma unroll
        for (int hp = 0; hp < 2; ++hp) {
            if ((l32 >> 4) == hp) {
#pragma unroll
                for (int dt = 0; dt < 2; ++dt)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        bf16x4 o4;
#pragma unroll
                        for (int i = 0; i < 4; ++i) o4[i] = (bf16_t)(oacc[dt][4 * g + i] * inv);
                        const int u = dt * 8 + 2 * g + half;
                        *reinterpret_cast<bf16x4 *>(ostg + r16 * 128 + ((u ^ wswz) << 3)) = o4;
                    }
            }
            __builtin_amdgcn_wave_barrier();  // LDS serves a wave's accesses in order
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int lr = j * 8 + orow, q = qb * 32 + hp * 16 + lr;
                u32x4 v = *reinterpret_cast<const u32x4 *>(ostg + lr * 128 + ((och ^ orow) << 4));
                if (j & 1) v = u32x4{v[2], v[3], v[0], v[1]};  // rows 8..15 hold the halves of a chunk swapped
                if (q < L) __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(out + (size_t)(t0 + q) * d + h * 64 + och * 8));
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// ------------------------------------------------------------------ masked mean pool + L2 normalise
// One block per chunk.  Wave w sums rows w, w + 4, ... with 16-byte loads (a lane owns pieces j*64 + lane of a row, as
// in the LayerNorm kernels); the four partial sums of a column are added in wave order, so the result does not depend
// on anything but the chunk.
__global__ __launch_bounds__(256) void pool_kernel(const bf16_t *__restrict__ x, const int32_t *__restrict__ cu, int d,
                                                   float *__restrict__ out)
{
    __shared__ float part[4][1024];
    __shared__ float red[256];
    const int c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = cu[c], L = cu[c + 1] - t0;
    const int pieces = d >> 3;
    float acc[2][8];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[j][i] = 0.f;
    for (int t = wave; t < L; t += 4) {
        const bf16_t *xr = x + (size_t)(t0 + t) * d;
#pragma unroll
        for (int j = 0; j < 2; ++j)
            if (j * 64 + lane < pieces) {
                const bf16x8 r = *reinterpret_cast<const bf16x8 *>(xr + (j * 64 + lane) * 8);
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[j][i] += (float)r[i];
            }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j)
        if (j * 64 + lane < pieces) {
#pragma unroll
            for (int i = 0; i < 8; ++i) part[wave][(j * 64 + lane) * 8 + i] = acc[j][i];
        }
    __syncthreads();
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    float sq = 0.f;
    if (L > 0) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int col = tid + 256 * j;
            if (col < d) {
                v[j] = (((part[0][col] + part[1][col]) + part[2][col]) + part[3][col]) / (float)L;
                sq += v[j] * v[j];
            }
        }
    }
    red[tid] = sq;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    const float nrm = fmaxf(sqrtf(red[0]), 1e-12f);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int col = tid + 256 * j;
        if (col < d) out[(size_t)c * d + col] = v[j] / nrm;
    }
}

template <int BM, int BN, int EPI>
int launch_gemm(leann_ctx *ctx, int prof_kind, const bf16_t *A, const bf16_t *W, const float *bias, bf16_t *out,
                const int32_t *T_dev, int max_rows, int N, int K)
{
    constexpr int WM = 2, WN = BN / 64;
    constexpr int smem = gemm_smem_bytes<BM, BN, WM, WN>();
    if (N % BN || K % (4 * GEMM_BK) || (BM * BN > 128 * 128 && K < 8 * GEMM_BK)) {
        leann_set_error("GEMM shape N=%d K=%d not covered by the %dx%d tile", N, K, BM, BN);
        return LEANN_ESHAPE;
    }
    const int tiles_n = N / BN;
    // W beyond the 4 MB of L2 an XCD has is evicted between its uses; if the output is wide (so that A is small next
    // to it) the column tiles go in groups that fit (measured on FFN1: +4-5 %; on QKV, whose W fits, a loss).
    int gcols = tiles_n;
    if ((size_t)N * K * sizeof(bf16_t) > ((size_t)4 << 20) && N >= 4 * K) {
        const int groups = (int)(((size_t)N * K * sizeof(bf16_t) + ((size_t)5 << 19) - 1) / ((size_t)5 << 19));  // 2.5 MB each
        gcols = (tiles_n + groups - 1) / groups;
    }
    const int tiles = ((max_rows + BM - 1) / BM) * tiles_n;
    // persistent blocks: one per CU slot (a multiple of 8), fewer when there are fewer tiles
    const int slots = ctx->num_cus * (BM == 256 ? 1 : BM == 128 ? 2 : 4);
    const int grid = std::max(8, std::min(slots, (tiles + 7) & ~7) & ~7);
    ProfScope prof(ctx, prof_kind);
    hipLaunchKernelGGL((gemm_kernel<BM, BN, WM, WN, EPI>), dim3(grid), dim3(64 * WM * WN), smem, ctx->stream, A, W, bias,
                       out, T_dev, N, K, tiles_n, gcols);
    LEANN_HIP(hipGetLastError());
    return LEANN_OK;
}

template <int BM, int BN, int EPI>
int gemm_allow_lds()
{
    constexpr int WM = 2, WN = BN / 64;
    LEANN_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(gemm_kernel<BM, BN, WM, WN, EPI>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, gemm_smem_bytes<BM, BN, WM, WN>()));
    return LEANN_OK;
}

}  // namespace

// Kernels that use more dynamic LDS than the default limit are allowed their size on the current device.
int enc_ln_blocks_per_cu(int *out)
{
    int n = 0;
    LEANN_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void *>(ln_kernel), 256, 0));
    *out = n > 0 ? n : 1;
    return LEANN_OK;
}

int enc_init_device()
{
    LEANN_TRY((gemm_allow_lds<256, 256, EPI_BIAS>()));
    LEANN_TRY((gemm_allow_lds<256, 256, EPI_BIAS_GELU>()));
    LEANN_TRY((gemm_allow_lds<128, 128, EPI_BIAS>()));
    LEANN_TRY((gemm_allow_lds<128, 128, EPI_BIAS_GELU>()));
    LEANN_TRY((gemm_allow_lds<64, 64, EPI_BIAS>()));
    LEANN_TRY((gemm_allow_lds<64, 64, EPI_BIAS_GELU>()));
    LEANN_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(attention_kernel<8>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, AttCfg<8>::SMEM));
    return LEANN_OK;
}

int enc_forward(leann_ctx *ctx, const leann_chunks *chunks, const int64_t *ids_dev, int64_t first_id, int64_t n,
                float *out_dev, int *err_dev, int64_t *tok_count_dev)
{
    const leann_encoder_desc &e = ctx->desc;
    const int d = e.hidden, F = e.ffn, H = e.heads, seq = chunks->seq;
    if (n <= 0) return LEANN_OK;
    if (seq < 1 || seq > 256 || seq > e.max_pos) {
        leann_set_error("sequence length %d not covered (1..min(256, max_pos))", seq);
        return LEANN_ESHAPE;
    }
    int64_t per_pass = ctx->max_tokens / seq;
    if (per_pass < 1) per_pass = 1;
    if (per_pass > n) per_pass = n;
    const size_t rows = (size_t)per_pass * seq + 256;
    LEANN_TRY(ctx->x.reserve(rows * d * sizeof(bf16_t)));
    LEANN_TRY(ctx->qkv.reserve(rows * 3 * d * sizeof(bf16_t)));
    LEANN_TRY(ctx->att.reserve(rows * d * sizeof(bf16_t)));
    LEANN_TRY(ctx->delta.reserve(rows * d * sizeof(bf16_t)));
    LEANN_TRY(ctx->hid.reserve(rows * F * sizeof(bf16_t)));
    LEANN_TRY(ctx->cu.reserve((size_t)(per_pass + 1) * sizeof(int32_t)));
    LEANN_TRY(ctx->enc_ids.reserve((size_t)per_pass * sizeof(int64_t)));
    bf16_t *x = (bf16_t *)ctx->x.p, *qkv = (bf16_t *)ctx->qkv.p, *att = (bf16_t *)ctx->att.p, *hid = (bf16_t *)ctx->hid.p;
    bf16_t *delta = (bf16_t *)ctx->delta.p;  // sublayer output waiting for its residual add + LayerNorm
    int32_t *cu = (int32_t *)ctx->cu.p;
    int64_t *chunk_of = (int64_t *)ctx->enc_ids.p;
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)(d / H));
    // 256x256 block tiles for large passes and output widths that are multiples of 256 (LDS traffic per flop
    // halves); leann_set_gemm_tiles can force the small tile and move the row limit of the 64x64 tile.
    const bool wide = ctx->gemm_large_tile == 256;
    const int small_rows = ctx->gemm_small_rows;

    for (int64_t s = 0; s < n; s += per_pass) {
        const int m = (int)((n - s < per_pass) ? n - s : per_pass);
        const int max_rows = m * seq;
        // a pass of a few thousand tokens has too few 256x256 tiles for the CUs: the 128x128 tile (four times the blocks,
        // two per CU) is faster there (measured: +15 % at 32 chunks of up to 256 tokens, -6 % at 64).  Both tiles add
        // the K-slabs in the same order, so a row's result does not depend on the choice.
        const bool big = wide && max_rows > 8192;  // and, per GEMM, an output width that is a multiple of 256
        // a pass of one query's flush (a dozen chunks) does not even fill the CUs with 128x128 tiles: 64x64 tiles
        // (measured: faster up to 2048 padded rows, slower from 3072 on; leann_set_gemm_tiles moves the limit)
        const bool tiny = !big && max_rows <= small_rows && d % 64 == 0 && F % 64 == 0;
        const int32_t *T_dev = cu + m;
        {
            ProfScope prof(ctx, LEANN_PROF_ENC_OTHER);
            hipLaunchKernelGGL(prep_kernel, dim3(1), dim3(1024), 0, ctx->stream, chunks->lengths,
                               ids_dev ? ids_dev + s : nullptr, first_id + s, m, chunks->n, seq, cu, chunk_of, err_dev,
                               tok_count_dev, ctx->prof_on ? (int64_t *)ctx->prof_tokens.p : nullptr);
        }
        {
            ProfScope prof(ctx, LEANN_PROF_ENC_OTHER);
            hipLaunchKernelGGL(embed_ln_kernel, dim3((unsigned)(((int64_t)m * seq + 3) / 4)), dim3(256), 0, ctx->stream,
                               chunks->tokens, chunk_of, cu, m, seq, d, e.vocab, ctx->tok_emb, ctx->pos_emb, ctx->seg_emb,
                               ctx->emb_g, ctx->emb_b, e.ln_eps, x, err_dev);
        }
        // as many blocks as are resident at once (measured: 10 % faster than a row per wave, and than twice as
        // many blocks); their waves go through several rows each
        const int ln_grid = std::min((max_rows + 3) / 4, ctx->num_cus * ctx->ln_blocks_per_cu);
        auto layer_norm = [&](const float *g, const float *b) {
            ProfScope prof(ctx, LEANN_PROF_LAYERNORM);
            hipLaunchKernelGGL(ln_kernel, dim3(ln_grid), dim3(256), 0, ctx->stream, delta, g, b, x, T_dev, d, e.ln_eps);
        };
        for (int l = 0; l < e.layers; ++l) {
            const LayerWeights &w = ctx->layers[l];
#define LEANN_GEMM(EPI, KIND, A_, W_, B_, O_, N_, K_)                                                               \
    LEANN_TRY((big && (N_) % 256 == 0 && (K_) >= 256                                                                \
                   ? launch_gemm<256, 256, EPI>(ctx, KIND, A_, W_, B_, O_, T_dev, max_rows, N_, K_)                   \
               : tiny ? launch_gemm<64, 64, EPI>(ctx, KIND, A_, W_, B_, O_, T_dev, max_rows, N_, K_)                   \
                      : launch_gemm<128, 128, EPI>(ctx, KIND, A_, W_, B_, O_, T_dev, max_rows, N_, K_)))
            LEANN_GEMM(EPI_BIAS, LEANN_PROF_GEMM_QKV, x, w.wqkv, w.bqkv, qkv, 3 * d, d);
            {
                ProfScope prof(ctx, LEANN_PROF_ATTENTION);
                if (seq <= 128)
                    hipLaunchKernelGGL(attention_kernel<4>, dim3((unsigned)m * H), dim3(256), AttCfg<4>::SMEM, ctx->stream, qkv, cu,
                                       att, d, scale_log2e);
                else
                    hipLaunchKernelGGL(attention_kernel<8>, dim3((unsigned)m * H), dim3(256), AttCfg<8>::SMEM, ctx->stream, qkv, cu,
                                       att, d, scale_log2e);
            }
            LEANN_GEMM(EPI_BIAS, LEANN_PROF_GEMM_O, att, w.wo, w.bo, delta, d, d);
            layer_norm(w.g1, w.be1);
            LEANN_GEMM(EPI_BIAS_GELU, LEANN_PROF_GEMM_FFN1, x, w.w1, w.b1, hid, F, d);
            LEANN_GEMM(EPI_BIAS, LEANN_PROF_GEMM_FFN2, hid, w.w2, w.b2, delta, d, F);
#undef LEANN_GEMM
            layer_norm(w.g2, w.be2);
        }
        {
            ProfScope prof(ctx, LEANN_PROF_ENC_OTHER);
            hipLaunchKernelGGL(pool_kernel, dim3(m), dim3(256), 0, ctx->stream, x, cu, d, out_dev + (size_t)s * d);
        }
        LEANN_HIP(hipGetLastError());
    }
    return LEANN_OK;
}

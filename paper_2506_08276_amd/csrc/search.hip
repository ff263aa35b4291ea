// Two-level search with dynamic batching (LEANN Algorithm 2, Sec. 4.1-4.2), every stage on the device.
//
// All queries of a call advance in rounds.  In a round each active query runs hops on its own wavefront
// (traverse_kernel: read the best unvisited node of the exact queue EQ, gather its CSR neighbours, ADC-score
// the new ones out of an LDS-resident lookup table, push them into the approximate queue AQ, move the
// top re-rank fraction to the pending list P) until |P| >= batch or EQ has no unvisited node.  The pending
// lists of all queries are then packed into one list, re-embedded by the encoder in large cross-query
// batches, scored against their own query and try-inserted into EQ (score_insert_kernel).  Per query this
// is exactly the sequential algorithm; batching across queries changes no value because the encoder's
// output for a chunk does not depend on the rest of the batch.
#include <algorithm>
#include <vector>

#include "common.h"

namespace {

constexpr int KSUB = 256;

struct SearchState {
    float *eq_score;      // [G][ef]
    uint32_t *eq_id;      // [G][ef]
    uint8_t *eq_vis;      // [G][ef]
    int32_t *eq_n;        // [G]
    float *aq_score;      // [G][aqcap]
    uint32_t *aq_id;      // [G][aqcap]
    int32_t *aq_n;        // [G]
    uint32_t *seen;       // [G][words]
    uint32_t *pend;       // [G][pcap]
    int32_t *n_pend;      // [G]
    int32_t *src;         // [G][pcap]  >= 0: row of the encoder output; -1 .. -2^30: -(cache row + 1); below: -(2^30 + memo row + 1)
    int32_t *owner;       // [N] smallest pending entry (q * pcap + j) that asked for the chunk this round, else INT_MAX
    int32_t *memo_slot;   // [N] row of the call's embedding memo that holds the chunk, -1: none; NULL: memo off
    const float *memo_emb;  // [memo rows][d]
    int32_t *done;        // [G]
    int32_t *enc_off;     // [G + 1]
    int64_t *enc_ids;     // [G * pcap]
    long long *counters;  // see CTR_*
    const float *lut;     // [G][m_sub][256]
    int64_t words;
    int32_t ef, aqcap, pcap;
};

enum { CTR_HOPS = 0, CTR_ADC, CTR_RECOMP, CTR_FLUSH, CTR_PENDING, CTR_NENC, CTR_ERR, CTR_TOKENS, CTR_MAXDEG, CTR_HITS, CTR_MEMO_HITS, CTR_COUNT };
constexpr int MEMO_SRC_BASE = 1 << 30;
enum { ERR_BAD_NEIGHBOUR = 1, ERR_AQ_OVERFLOW = 2, ERR_P_OVERFLOW = 4, ERR_BAD_SLOT = 8 };

__device__ inline bool better(float sa, uint32_t ia, float sb, uint32_t ib) { return sa > sb || (sa == sb && ia < ib); }

// wave-wide arg-best under (score desc, id asc); pos < 0 marks "nothing".  Result is uniform.
__device__ inline void wave_best(float &s, uint32_t &id, int &pos)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float s2 = __shfl_xor(s, o, 64);
        uint32_t id2 = __shfl_xor(id, o, 64);
        int p2 = __shfl_xor(pos, o, 64);
        if (p2 >= 0 && (pos < 0 || better(s2, id2, s, id))) {
            s = s2;
            id = id2;
            pos = p2;
        }
    }
}

// wave-wide arg-worst under the same order.
__device__ inline void wave_worst(float &s, uint32_t &id, int &pos)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float s2 = __shfl_xor(s, o, 64);
        uint32_t id2 = __shfl_xor(id, o, 64);
        int p2 = __shfl_xor(pos, o, 64);
        if (p2 >= 0 && (pos < 0 || better(s, id, s2, id2))) {
            s = s2;
            id = id2;
            pos = p2;
        }
    }
}

__global__ void maxdeg_kernel(const uint64_t *__restrict__ row_ptr, int64_t n, long long *__restrict__ counters)
{
    long long best = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        best = max(best, (long long)(row_ptr[i + 1] - row_ptr[i]));
    atomicMax(&counters[CTR_MAXDEG], best);
}

__global__ void init_kernel(SearchState s, int g, uint32_t entry)
{
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= g) return;
    s.eq_n[q] = 0;
    s.aq_n[q] = 0;
    s.done[q] = 0;
    s.n_pend[q] = 1;  // the entry point's exact score is the first flush
    s.pend[(size_t)q * s.pcap] = entry;
    s.seen[(size_t)q * s.words + (entry >> 5)] = 1u << (entry & 31);
}

// One wavefront per query.  Dynamic LDS: lookup table [m_sub][256] fp32, then EQ score/id/visited copies.
__global__ __launch_bounds__(64) void traverse_kernel(SearchState s, const uint64_t *__restrict__ row_ptr,
                                                      const uint32_t *__restrict__ col_idx, int64_t n,
                                                      const uint8_t *__restrict__ codes, int m_sub, float alpha, int batch)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *tab = reinterpret_cast<float *>(smem);
    float *eqs = tab + m_sub * KSUB;
    uint32_t *eqi = reinterpret_cast<uint32_t *>(eqs + s.ef);
    uint8_t *eqv = reinterpret_cast<uint8_t *>(eqi + s.ef);
    const int q = blockIdx.x, lane = threadIdx.x;
    if (s.done[q]) return;
    const int n_eq = s.eq_n[q];
    int n_aq = s.aq_n[q], n_pend = s.n_pend[q];
    int any = 0;
    for (int i = lane; i < n_eq; i += 64) {
        eqs[i] = s.eq_score[(size_t)q * s.ef + i];
        eqi[i] = s.eq_id[(size_t)q * s.ef + i];
        uint8_t v = s.eq_vis[(size_t)q * s.ef + i];
        eqv[i] = v;
        any |= !v;
    }
    if (__ballot(any) == 0ull) {  // nothing to expand: wait for the flush, or finished
        if (lane == 0 && n_pend == 0) s.done[q] = 1;
        return;
    }
    {
        const float4 *src = reinterpret_cast<const float4 *>(s.lut + (size_t)q * m_sub * KSUB);
        for (int i = lane; i < m_sub * KSUB / 4; i += 64) reinterpret_cast<float4 *>(tab)[i] = src[i];
    }
    __syncthreads();
    float *aqs = s.aq_score + (size_t)q * s.aqcap;
    uint32_t *aqi = s.aq_id + (size_t)q * s.aqcap;
    uint32_t *seen = s.seen + (size_t)q * s.words;
    uint32_t *pend = s.pend + (size_t)q * s.pcap;
    int hops = 0, adc = 0, err = 0;
    while (n_pend < batch) {
        // Alg. 2: u = the best node of EQ that has not been expanded yet; it is marked visited
        float bs = -INFINITY;
        uint32_t bid = 0xffffffffu;
        int bpos = -1;
        for (int i = lane; i < n_eq; i += 64)
            if (!eqv[i] && (bpos < 0 || better(eqs[i], eqi[i], bs, bid))) {
                bs = eqs[i];
                bid = eqi[i];
                bpos = i;
            }
        wave_best(bs, bid, bpos);
        if (bpos < 0) break;
        if (lane == 0) eqv[bpos] = 1;
        ++hops;
        const uint64_t beg = row_ptr[bid], end = row_ptr[bid + 1];
        int n_new = 0;
        for (uint64_t base = beg; base < end; base += 64) {
            const uint64_t e = base + lane;
            bool is_new = false;
            uint32_t v = 0;
            if (e < end) {
                v = col_idx[e];
                if (v >= n) {
                    err |= ERR_BAD_NEIGHBOUR;
                } else {
                    const uint32_t bit = 1u << (v & 31);
                    is_new = !(atomicOr(&seen[v >> 5], bit) & bit);
                }
            }
            float sc = 0.f;
            if (is_new) {  // ADC: table entries summed in subspace order
                const uint8_t *code = codes + (size_t)v * m_sub;
                if ((m_sub & 15) == 0) {
                    for (int m0 = 0; m0 < m_sub; m0 += 16) {
                        const uint4 w = *reinterpret_cast<const uint4 *>(code + m0);
                        const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                        for (int i = 0; i < 16; ++i) sc += tab[(m0 + i) * KSUB + ((ww[i >> 2] >> (8 * (i & 3))) & 255u)];
                    }
                } else {
                    for (int m = 0; m < m_sub; ++m) sc += tab[m * KSUB + code[m]];
                }
            }
            const unsigned long long mask = __ballot(is_new);
            const int pos = n_aq + __popcll(mask & ((1ull << lane) - 1ull));
            if (is_new) {
                if (pos < s.aqcap) {
                    aqs[pos] = sc;
                    aqi[pos] = v;
                } else {
                    err |= ERR_AQ_OVERFLOW;
                }
            }
            const int cnt = __popcll(mask);
            n_aq = min(n_aq + cnt, s.aqcap);
            n_new += cnt;
        }
        adc += n_new;
        __syncthreads();  // single-wave block: orders this wave's AQ stores before the scans below
        // move the r best entries of AQ to the pending list
        const int r = (int)ceilf(alpha * (float)n_new);
        for (int t = 0; t < r && n_aq > 0; ++t) {
            float ps = -INFINITY;
            uint32_t pid = 0xffffffffu;
            int ppos = -1;
            for (int i = lane; i < n_aq; i += 64) {
                const float x = aqs[i];
                const uint32_t id = aqi[i];
                if (ppos < 0 || better(x, id, ps, pid)) {
                    ps = x;
                    pid = id;
                    ppos = i;
                }
            }
            wave_best(ps, pid, ppos);
            if (lane == 0) {
                if (n_pend < s.pcap) pend[n_pend] = pid;
                aqs[ppos] = aqs[n_aq - 1];
                aqi[ppos] = aqi[n_aq - 1];
            }
            if (n_pend >= s.pcap) err |= ERR_P_OVERFLOW;
            n_pend = min(n_pend + 1, s.pcap);
            --n_aq;
            __syncthreads();
        }
    }
    for (int i = lane; i < n_eq; i += 64) s.eq_vis[(size_t)q * s.ef + i] = eqv[i];
    const unsigned long long anyerr = __ballot(err != 0);
    if (anyerr) {
        int e = err;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) e |= __shfl_xor(e, o, 64);
        if (lane == 0) atomicOr((unsigned long long *)&s.counters[CTR_ERR], (unsigned long long)e);
    }
    if (lane == 0) {
        s.aq_n[q] = n_aq;
        s.n_pend[q] = n_pend;
        if (n_pend == 0) s.done[q] = 1;  // left the loop with no unvisited node and nothing pending
        atomicAdd((unsigned long long *)&s.counters[CTR_HOPS], (unsigned long long)hops);
        atomicAdd((unsigned long long *)&s.counters[CTR_ADC], (unsigned long long)adc);
    }
}

// Chunks that several queries ask for in the same round are encoded once: the pending entry with the smallest
// index (q * pcap + j) owns the chunk, the others read the owner's row.  The encoder's output for a chunk does
// not depend on its batch, so every query still sees exactly the scores it would compute alone.
constexpr int NO_OWNER = 0x7f7f7f7f;  // the fill byte 0x7f makes hipMemsetAsync usable

// slot_of entries >= cache_rows would send score_insert_kernel outside the stored table: they are reported
// (ERR_BAD_SLOT) and the host ends the search before anything reads through them.
__global__ __launch_bounds__(64) void claim_kernel(SearchState s, const int32_t *__restrict__ slot_of, int64_t cache_rows)
{
    const int q = blockIdx.x;
    const int np = s.n_pend[q];
    int hits = 0, memo_hits = 0;
    bool bad = false;
    for (int j = threadIdx.x; j < np; j += 64) {
        const uint32_t c = s.pend[(size_t)q * s.pcap + j];
        if (slot_of && slot_of[c] >= 0) {
            bad |= slot_of[c] >= cache_rows;
            ++hits;
            continue;
        }
        if (s.memo_slot && s.memo_slot[c] >= 0) {  // encoded earlier in this call
            ++memo_hits;
            continue;
        }
        atomicMin(&s.owner[c], q * s.pcap + j);
    }
    if (bad) atomicOr((unsigned long long *)&s.counters[CTR_ERR], (unsigned long long)ERR_BAD_SLOT);
    if (s.memo_slot) {
        for (int o = 32; o; o >>= 1) memo_hits += __shfl_xor(memo_hits, o);
        if (threadIdx.x == 0 && memo_hits)
            atomicAdd((unsigned long long *)&s.counters[CTR_MEMO_HITS], (unsigned long long)memo_hits);
    }
    if (slot_of) {
        for (int o = 32; o; o >>= 1) hits += __shfl_xor(hits, o);
        if (threadIdx.x == 0 && hits) atomicAdd((unsigned long long *)&s.counters[CTR_HITS], (unsigned long long)hits);
    }
}

// Pack the round: encoder input list (one entry per owned chunk, in entry order), source rows of the owners and
// of the entries served by the stored-embedding table, and the round's totals.  One block of 1024 threads.
__global__ __launch_bounds__(1024) void collect_kernel(SearchState s, int g, const int32_t *__restrict__ slot_of)
{
    __shared__ int part[1024];
    const int tid = threadIdx.x;
    const int per = (g + 1023) / 1024;
    const int beg = tid * per, end = min(g, beg + per);
    int need = 0, pending = 0;
    for (int q = beg; q < end; ++q) {
        const int np = s.n_pend[q];
        pending += np;
        for (int j = 0; j < np; ++j) need += s.owner[s.pend[(size_t)q * s.pcap + j]] == q * s.pcap + j;
    }
    part[tid] = need;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        int v = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    int run = tid ? part[tid - 1] : 0;
    for (int q = beg; q < end; ++q) {
        s.enc_off[q] = run;
        const int np = s.n_pend[q];
        for (int j = 0; j < np; ++j) {
            const int e = q * s.pcap + j;
            const uint32_t c = s.pend[e];
            const int slot = slot_of ? slot_of[c] : -1;
            const int mslot = (slot < 0 && s.memo_slot) ? s.memo_slot[c] : -1;
            if (slot >= 0) {
                s.src[e] = -(slot + 1);
            } else if (mslot >= 0) {
                s.src[e] = -(MEMO_SRC_BASE + mslot + 1);
            } else if (s.owner[c] == e) {
                s.enc_ids[run] = c;
                s.src[e] = run++;
            }
        }
    }
    if (tid == 1023) {
        s.enc_off[g] = part[1023];
        s.counters[CTR_NENC] = part[1023];
    }
    if (pending) atomicAdd((unsigned long long *)&s.counters[CTR_PENDING], (unsigned long long)pending);
}

// Entries that do not own their chunk take the owner's row.
__global__ __launch_bounds__(64) void resolve_kernel(SearchState s, const int32_t *__restrict__ slot_of)
{
    const int q = blockIdx.x;
    const int np = s.n_pend[q];
    for (int j = threadIdx.x; j < np; j += 64) {
        const int e = q * s.pcap + j;
        const uint32_t c = s.pend[e];
        if (slot_of && slot_of[c] >= 0) continue;
        if (s.memo_slot && s.memo_slot[c] >= 0) continue;
        const int o = s.owner[c];
        if (o != e) s.src[e] = s.src[o];
    }
}

// Exact scores of the pending chunks and try-insert into EQ, in pending order.  One wavefront per query.
__global__ __launch_bounds__(64) void score_insert_kernel(SearchState s, const float *__restrict__ queries, int d,
                                                          const float *__restrict__ enc_emb,
                                                          const float *__restrict__ cache_emb)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *eqs = reinterpret_cast<float *>(smem);
    uint32_t *eqi = reinterpret_cast<uint32_t *>(eqs + s.ef);
    uint8_t *eqv = reinterpret_cast<uint8_t *>(eqi + s.ef);
    const int q = blockIdx.x, lane = threadIdx.x;
    const int np = s.n_pend[q];
    if (np == 0) return;
    int n_eq = s.eq_n[q];
    for (int i = lane; i < n_eq; i += 64) {
        eqs[i] = s.eq_score[(size_t)q * s.ef + i];
        eqi[i] = s.eq_id[(size_t)q * s.ef + i];
        eqv[i] = s.eq_vis[(size_t)q * s.ef + i];
    }
    float qv[16];
    const int per = (d + 63) >> 6;
#pragma unroll
    for (int j = 0; j < 16; ++j) qv[j] = (j < per && j * 64 + lane < d) ? queries[(size_t)q * d + j * 64 + lane] : 0.f;
    __syncthreads();
    for (int c = 0; c < np; ++c) {
        const int src = s.src[(size_t)q * s.pcap + c];
        const uint32_t id = s.pend[(size_t)q * s.pcap + c];
        const float *e = src >= 0                ? enc_emb + (size_t)src * d
                         : src >= -MEMO_SRC_BASE ? cache_emb + (size_t)(-src - 1) * d
                                                 : s.memo_emb + (size_t)(-(src + MEMO_SRC_BASE) - 1) * d;
        float acc = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j)
            if (j < per && j * 64 + lane < d) acc += qv[j] * e[j * 64 + lane];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
        if (n_eq < s.ef) {
            if (lane == 0) {
                eqs[n_eq] = acc;
                eqi[n_eq] = id;
                eqv[n_eq] = 0;
            }
            ++n_eq;
        } else {  // EQ full: the candidate must beat the tail
            float ws = 0.f;
            uint32_t wid = 0;
            int wpos = -1;
            for (int i = lane; i < n_eq; i += 64)
                if (wpos < 0 || better(ws, wid, eqs[i], eqi[i])) {
                    ws = eqs[i];
                    wid = eqi[i];
                    wpos = i;
                }
            wave_worst(ws, wid, wpos);
            if (lane == 0 && better(acc, id, ws, wid)) {
                eqs[wpos] = acc;
                eqi[wpos] = id;
                eqv[wpos] = 0;
            }
        }
        __syncthreads();
    }
    for (int i = lane; i < n_eq; i += 64) {
        s.eq_score[(size_t)q * s.ef + i] = eqs[i];
        s.eq_id[(size_t)q * s.ef + i] = eqi[i];
        s.eq_vis[(size_t)q * s.ef + i] = eqv[i];
    }
    for (int j = lane; j < np; j += 64) s.owner[s.pend[(size_t)q * s.pcap + j]] = NO_OWNER;  // free for the next round
    if (lane == 0) {
        s.eq_n[q] = n_eq;
        s.n_pend[q] = 0;
        atomicAdd((unsigned long long *)&s.counters[CTR_RECOMP], (unsigned long long)np);
        atomicAdd((unsigned long long *)&s.counters[CTR_FLUSH], 1ull);
    }
}

// The call's embedding memo: rows the encoder produced in this round are kept (while there is room) so that a later
// round of the same call reads them instead of encoding the chunk again.  One wavefront per encoded chunk.
__global__ __launch_bounds__(256) void memo_store_kernel(const float *__restrict__ enc_emb, const int64_t *__restrict__ enc_ids,
                                                         int n_enc, int d, int64_t base, int64_t cap,
                                                         float *__restrict__ memo_emb, int32_t *__restrict__ memo_slot)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (i >= n_enc || base + i >= cap) return;
    const float *srcp = enc_emb + (size_t)i * d;
    float *dst = memo_emb + (size_t)(base + i) * d;
    for (int c = lane; c < d; c += 64) dst[c] = srcp[c];
    if (lane == 0) memo_slot[enc_ids[i]] = (int32_t)(base + i);
}

// Exact scores of the add buffer (App. B "Batched Add Operation": buffered chunks are scanned, not traversed):
// out[q][r] = <queries[q], buf[r]>.  One wavefront per (query, buffer row).
__global__ __launch_bounds__(256) void buffer_score_kernel(const float *__restrict__ queries, const float *__restrict__ buf,
                                                           int nb, int d, float *__restrict__ out)
{
    const int q = blockIdx.y, r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= nb) return;
    const float *qv = queries + (size_t)q * d, *e = buf + (size_t)r * d;
    float acc = 0.f;
    for (int i = lane; i < d; i += 64) acc += qv[i] * e[i];
    for (int o = 32; o; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) out[(size_t)q * nb + r] = acc;
}

// Output stage: the k best of (EQ without soft-deleted nodes) united with the scored add buffer, under
// (score desc, id asc); padded with id -1 / score -inf.  One wavefront per query; position p < n_eq is an EQ
// entry, p >= n_eq a buffer row.  Ids are unique over both, so "strictly after the last one emitted" selects the
// next.
__global__ __launch_bounds__(64) void finalize_kernel(SearchState s, int k, const uint32_t *__restrict__ deleted_bits,
                                                      const float *__restrict__ buf_scores,
                                                      const uint32_t *__restrict__ buf_ids, int nb,
                                                      int64_t *__restrict__ out_ids, float *__restrict__ out_scores)
{
    const int q = blockIdx.x, lane = threadIdx.x;
    const int n_eq = s.eq_n[q];
    const float *eqs = s.eq_score + (size_t)q * s.ef;
    const uint32_t *eqi = s.eq_id + (size_t)q * s.ef;
    const float *bsc = buf_scores + (size_t)q * nb;
    float last_s = INFINITY;
    uint32_t last_id = 0;
    bool have_last = false, exhausted = false;
    for (int j = 0; j < k; ++j) {
        float bs = -INFINITY;
        uint32_t bid = 0xffffffffu;
        int bpos = -1;
        if (!exhausted)
            for (int i = lane; i < n_eq + nb; i += 64) {
                float x;
                uint32_t id;
                if (i < n_eq) {
                    x = eqs[i];
                    id = eqi[i];
                    if (deleted_bits && (deleted_bits[id >> 5] >> (id & 31) & 1u)) continue;
                } else {
                    x = bsc[i - n_eq];
                    id = buf_ids[i - n_eq];
                }
                if (have_last && !better(last_s, last_id, x, id)) continue;  // already emitted
                if (bpos < 0 || better(x, id, bs, bid)) {
                    bs = x;
                    bid = id;
                    bpos = i;
                }
            }
        wave_best(bs, bid, bpos);
        if (lane == 0) {
            out_ids[(size_t)q * k + j] = bpos >= 0 ? (int64_t)bid : -1;
            out_scores[(size_t)q * k + j] = bpos >= 0 ? bs : -INFINITY;
        }
        if (bpos < 0) exhausted = true;
        have_last = true;
        last_s = bs;
        last_id = bid;
    }
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

int search_init_device()
{
    LEANN_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(traverse_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    return LEANN_OK;
}

int search_run(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_graph *graph, const leann_pq *pq,
               const leann_chunks *chunks, const leann_emb_cache *cache, const leann_updates *upd, int32_t ef, int32_t k,
               float alpha, int32_t batch, int64_t *out_ids_dev, float *out_scores_dev, leann_search_stats *stats)
{
    const int d = ctx->desc.hidden, m_sub = pq->m_sub;
    const int64_t n = graph->n;
    hipStream_t st = ctx->stream;
    LEANN_TRY(ctx->s_misc.reserve(CTR_COUNT * sizeof(long long)));
    long long *counters = (long long *)ctx->s_misc.p;
    LEANN_HIP(hipMemsetAsync(counters, 0, CTR_COUNT * sizeof(long long), st));
    LEANN_TRY(ctx->meta.reserve(256));
    int *enc_err = (int *)ctx->meta.p;
    LEANN_HIP(hipMemsetAsync(enc_err, 0, sizeof(int), st));
    hipLaunchKernelGGL(maxdeg_kernel, dim3(256), dim3(256), 0, st, graph->row_ptr, n, counters);
    long long h_ctr[CTR_COUNT];
    LEANN_HIP(hipMemcpyAsync(h_ctr, counters, sizeof(h_ctr), hipMemcpyDeviceToHost, st));
    LEANN_HIP(hipStreamSynchronize(st));
    const long long maxdeg = h_ctr[CTR_MAXDEG];

    // capacities
    const int64_t rmax = (int64_t)ceilf(alpha * (float)maxdeg);
    int64_t pcap64 = std::min<int64_t>((int64_t)batch - 1 + rmax, n) + 1;
    const int32_t pcap = (int32_t)std::max<int64_t>(pcap64, 2);
    const int32_t aqcap = (int32_t)std::max<int64_t>(1, std::min<int64_t>(n, ctx->aq_capacity > 0 ? ctx->aq_capacity : 32768));
    const int64_t words = (n + 31) / 32;
    // queries in flight: bounded by a 4 GiB budget for pending embeddings and for the visited bitmaps
    const size_t budget = (size_t)4 << 30;
    int64_t g_max = std::min<int64_t>(nq, 4096);
    g_max = std::min<int64_t>(g_max, std::max<int64_t>(1, (int64_t)(budget / ((size_t)pcap * d * sizeof(float)))));
    g_max = std::min<int64_t>(g_max, std::max<int64_t>(1, (int64_t)(budget / ((size_t)words * 4))));
    const int G = (int)g_max;

    // carve the state out of one allocation
    size_t off = 0;
    auto carve = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    const size_t o_eqs = carve((size_t)G * ef * 4), o_eqi = carve((size_t)G * ef * 4), o_eqv = carve((size_t)G * ef);
    const size_t o_eqn = carve((size_t)G * 4), o_aqs = carve((size_t)G * aqcap * 4), o_aqi = carve((size_t)G * aqcap * 4);
    const size_t o_aqn = carve((size_t)G * 4), o_pend = carve((size_t)G * pcap * 4), o_np = carve((size_t)G * 4);
    const size_t o_src = carve((size_t)G * pcap * 4), o_done = carve((size_t)G * 4), o_eoff = carve((size_t)(G + 1) * 4);
    const size_t o_eids = carve((size_t)G * pcap * 8);
    LEANN_TRY(ctx->s_state.reserve(off));
    LEANN_TRY(ctx->s_seen.reserve((size_t)G * words * 4));
    LEANN_TRY(ctx->s_lut.reserve((size_t)G * m_sub * KSUB * sizeof(float)));
    LEANN_TRY(ctx->s_emb.reserve((size_t)G * pcap * d * sizeof(float)));
    LEANN_TRY(ctx->s_owner.reserve((size_t)n * sizeof(int32_t)));
    LEANN_HIP(hipMemsetAsync(ctx->s_owner.p, 0x7f, (size_t)n * sizeof(int32_t), st));
    // per-call embedding memo (leann_set_call_memo): empty at the start of every call
    const int64_t memo_cap = std::min<int64_t>(ctx->memo_rows, MEMO_SRC_BASE - 1);
    int64_t memo_n = 0;
    if (memo_cap > 0) {
        LEANN_TRY(ctx->s_memo_slot.reserve((size_t)n * sizeof(int32_t)));
        LEANN_TRY(ctx->s_memo_emb.reserve((size_t)memo_cap * d * sizeof(float)));
        LEANN_HIP(hipMemsetAsync(ctx->s_memo_slot.p, 0xff, (size_t)n * sizeof(int32_t), st));
    }
    char *base = (char *)ctx->s_state.p;
    SearchState s;
    s.eq_score = (float *)(base + o_eqs);
    s.eq_id = (uint32_t *)(base + o_eqi);
    s.eq_vis = (uint8_t *)(base + o_eqv);
    s.eq_n = (int32_t *)(base + o_eqn);
    s.aq_score = (float *)(base + o_aqs);
    s.aq_id = (uint32_t *)(base + o_aqi);
    s.aq_n = (int32_t *)(base + o_aqn);
    s.seen = (uint32_t *)ctx->s_seen.p;
    s.pend = (uint32_t *)(base + o_pend);
    s.n_pend = (int32_t *)(base + o_np);
    s.src = (int32_t *)(base + o_src);
    s.done = (int32_t *)(base + o_done);
    s.owner = (int32_t *)ctx->s_owner.p;
    s.memo_slot = memo_cap > 0 ? (int32_t *)ctx->s_memo_slot.p : nullptr;
    s.memo_emb = memo_cap > 0 ? (const float *)ctx->s_memo_emb.p : nullptr;
    s.enc_off = (int32_t *)(base + o_eoff);
    s.enc_ids = (int64_t *)(base + o_eids);
    s.counters = counters;
    s.lut = (const float *)ctx->s_lut.p;
    s.words = words;
    s.ef = ef;
    s.aqcap = aqcap;
    s.pcap = pcap;

    const int trav_smem = m_sub * KSUB * (int)sizeof(float) + ef * 9 + 16;
    const int eq_smem = ef * 9 + 16;
    if (trav_smem > 150 * 1024) {
        leann_set_error("lookup table + queue of %d bytes exceed the LDS budget", trav_smem);
        return LEANN_ESHAPE;
    }

    struct Events : std::vector<hipEvent_t> {  // destroyed on every way out of this function
        ~Events()
        {
            for (hipEvent_t e : *this) (void)hipEventDestroy(e);
        }
    } evs;
    auto mark = [&]() -> int {
        hipEvent_t e;
        LEANN_HIP(hipEventCreate(&e));
        LEANN_HIP(hipEventRecord(e, st));
        evs.push_back(e);
        return LEANN_OK;
    };
    int rc = LEANN_OK;
    int64_t rounds = 0, encoded = 0;
    LEANN_TRY(mark());  // evs[0]: start
    for (int64_t q0 = 0; q0 < nq && rc == LEANN_OK; q0 += G) {
        const int g = (int)std::min<int64_t>(G, nq - q0);
        const float *qg = queries_dev + (size_t)q0 * d;
        LEANN_HIP(hipMemsetAsync(s.seen, 0, (size_t)g * words * 4, st));
        hipLaunchKernelGGL(init_kernel, dim3((g + 255) / 256), dim3(256), 0, st, s, g, graph->entry);
        LEANN_TRY(pq_build_lut(ctx, qg, g, pq, (float *)ctx->s_lut.p));
        for (;;) {
            LEANN_TRY(mark());
            {
                ProfScope prof(ctx, LEANN_PROF_TRAVERSE);
                hipLaunchKernelGGL(traverse_kernel, dim3(g), dim3(64), trav_smem, st, s, graph->row_ptr, graph->col_idx,
                                   n, pq->codes, m_sub, alpha, batch);
            }
            LEANN_HIP(hipMemsetAsync(&counters[CTR_PENDING], 0, 2 * sizeof(long long), st));
            {
                ProfScope prof(ctx, LEANN_PROF_COLLECT);
                const int32_t *slot_of = cache ? cache->slot_of : nullptr;
                hipLaunchKernelGGL(claim_kernel, dim3(g), dim3(64), 0, st, s, slot_of, cache ? cache->rows : 0);
                hipLaunchKernelGGL(collect_kernel, dim3(1), dim3(1024), 0, st, s, g, slot_of);
                hipLaunchKernelGGL(resolve_kernel, dim3(g), dim3(64), 0, st, s, slot_of);
            }
            LEANN_HIP(hipMemcpyAsync(h_ctr, counters, sizeof(h_ctr), hipMemcpyDeviceToHost, st));
            LEANN_TRY(mark());
            LEANN_HIP(hipStreamSynchronize(st));
            if (h_ctr[CTR_ERR]) {
                rc = (h_ctr[CTR_ERR] & (ERR_BAD_NEIGHBOUR | ERR_BAD_SLOT)) ? LEANN_EINVAL : LEANN_ECAPACITY;
                leann_set_error((h_ctr[CTR_ERR] & ERR_BAD_NEIGHBOUR) ? "graph holds a neighbour id >= n"
                                : (h_ctr[CTR_ERR] & ERR_BAD_SLOT) ? "embedding cache: slot_of holds a row >= rows"
                                : "a per-query queue outgrew its capacity (see leann_set_limits)");
                break;
            }
            if (h_ctr[CTR_PENDING] == 0) {
                for (int i = 0; i < 2; ++i) {
                    (void)hipEventDestroy(evs.back());
                    evs.pop_back();
                }
                break;
            }
            const int64_t n_enc = h_ctr[CTR_NENC];
            if (n_enc > 0) {
                rc = enc_forward(ctx, chunks, s.enc_ids, 0, n_enc, (float *)ctx->s_emb.p, enc_err,
                                 (int64_t *)&counters[CTR_TOKENS]);
                if (rc != LEANN_OK) break;
                encoded += n_enc;
                if (memo_cap > 0 && memo_n < memo_cap) {
                    hipLaunchKernelGGL(memo_store_kernel, dim3((unsigned)((n_enc + 3) / 4)), dim3(256), 0, st,
                                       (const float *)ctx->s_emb.p, s.enc_ids, (int)n_enc, d, memo_n, memo_cap,
                                       (float *)ctx->s_memo_emb.p, s.memo_slot);
                    memo_n = std::min<int64_t>(memo_cap, memo_n + n_enc);
                }
            }
            {
                ProfScope prof(ctx, LEANN_PROF_SCORE_INSERT);
                hipLaunchKernelGGL(score_insert_kernel, dim3(g), dim3(64), eq_smem, st, s, qg, d,
                                   (const float *)ctx->s_emb.p, cache ? cache->emb : nullptr);
            }
            ++rounds;
        }
        if (rc != LEANN_OK) break;
        const int nb = upd ? (int)upd->buffer_n : 0;
        const float *buf_scores = nullptr;
        if (nb > 0) {
            if ((size_t)g * nb * sizeof(float) > ((size_t)4 << 30)) {
                leann_set_error("leann_search: %d queries x %d buffered rows exceed the 4 GiB score workspace", g, nb);
                rc = LEANN_ECAPACITY;
                break;
            }
            LEANN_TRY(ctx->s_buf.reserve((size_t)g * nb * sizeof(float)));
            buf_scores = (const float *)ctx->s_buf.p;
            hipLaunchKernelGGL(buffer_score_kernel, dim3((nb + 3) / 4, g), dim3(256), 0, st, queries_dev + (size_t)q0 * d,
                               upd->buffer_emb, nb, d, (float *)ctx->s_buf.p);
        }
        hipLaunchKernelGGL(finalize_kernel, dim3(g), dim3(64), 0, st, s, k, upd ? upd->deleted_bits : nullptr, buf_scores,
                           upd ? upd->buffer_ids : nullptr, nb, out_ids_dev + (size_t)q0 * k,
                           out_scores_dev + (size_t)q0 * k);
    }
    if (rc == LEANN_OK) rc = mark();
    int h_enc_err = 0;
    if (rc == LEANN_OK) {
        LEANN_HIP(hipMemcpyAsync(h_ctr, counters, sizeof(h_ctr), hipMemcpyDeviceToHost, st));
        LEANN_HIP(hipMemcpyAsync(&h_enc_err, enc_err, sizeof(int), hipMemcpyDeviceToHost, st));
    }
    hipError_t sync_rc = hipStreamSynchronize(st);
    if (rc == LEANN_OK && sync_rc != hipSuccess) {
        leann_set_error("search kernels failed: %s", hipGetErrorString(sync_rc));
        rc = LEANN_EDEVICE;
    }
    if (rc == LEANN_OK && h_enc_err) {
        leann_set_error("chunk store holds a token id or length outside its range (flags %d)", h_enc_err);
        rc = LEANN_EINVAL;
    }
    if (rc == LEANN_OK && stats) {
        stats->hops = h_ctr[CTR_HOPS];
        stats->adc_candidates = h_ctr[CTR_ADC];
        stats->recomputed_chunks = h_ctr[CTR_RECOMP];
        stats->cache_hits = h_ctr[CTR_HITS];
        stats->memo_hits = h_ctr[CTR_MEMO_HITS];
        stats->encoded_chunks = encoded;
        stats->encoded_tokens = h_ctr[CTR_TOKENS];
        stats->flushes = h_ctr[CTR_FLUSH];
        stats->rounds = rounds;
        float total = 0.f, trav = 0.f;
        (void)hipEventElapsedTime(&total, evs.front(), evs.back());
        // events come in (round start, after collect) pairs between the first and the last one
        for (size_t i = 1; i + 1 < evs.size(); i += 2) {
            float t = 0.f;
            (void)hipEventElapsedTime(&t, evs[i], evs[i + 1]);
            trav += t;
        }
        stats->total_ms = total;
        stats->traverse_ms = trav;
        stats->encoder_ms = total - trav;
    }
    return rc;
}

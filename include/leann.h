/*
 * libleann -- C ABI of the MI355X (gfx950) implementation of LEANN's search hot
 * path (arXiv 2506.08276): the recompute-and-score loop of best-first
 * proximity-graph search.
 *
 * Conventions that hold for every call
 *   - "dev" pointers are device (HBM) addresses on the context's GPU, "host"
 *     pointers are ordinary host memory.  All buffers are caller-owned and
 *     only borrowed for the duration of the call; the library owns the opaque
 *     handles (leann_ctx, leann_pq) and its internal workspaces.
 *   - Work is enqueued on the HIP stream given to leann_create.  Calls that
 *     write host memory or return counts synchronise that stream; the others
 *     return as soon as the work is enqueued.
 *   - Every function returns LEANN_OK (0) or a negative status; on error no
 *     output buffer has been written.  leann_last_error() gives a message for
 *     the calling thread.  Nothing is printed and nothing aborts.
 *   - Arrays are row-major.  Scores are inner-product similarities: larger is
 *     closer.  Every ranking uses the total order (score descending, id
 *     ascending).
 */
#ifndef LEANN_H
#define LEANN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    LEANN_OK = 0,
    LEANN_EINVAL = -1,    /* bad argument value (k > ef, ratio outside (0,1], null pointer, ...) */
    LEANN_ENOMEM = -2,    /* device or host allocation failed */
    LEANN_EDEVICE = -3,   /* a HIP call failed */
    LEANN_ESHAPE = -4,    /* shape the kernels do not cover (see leann_create) or inconsistent sizes */
    LEANN_ECAPACITY = -5  /* a per-query queue outgrew its capacity */
};

enum { LEANN_F32 = 0, LEANN_BF16 = 1 };

typedef struct leann_ctx leann_ctx;
typedef struct leann_pq leann_pq;

/* Encoder shape.  The paper fixes a BERT-style encoder of 110 M parameters with
 * 768-d output over 256-token chunks (Sec. 7 set-up); the layer equations are the
 * standard post-LN ones, see leann_embed. */
typedef struct {
    int32_t layers, hidden, heads, ffn, vocab, max_pos;
    float ln_eps;
} leann_encoder_desc;

/* Pruned proximity graph in CSR form, 4-byte neighbour ids (Sec. 5, "Space(G1)").
 * row_ptr[n+1] and col_idx[row_ptr[n]] are device pointers; entry is the fixed
 * entry point p of Algorithm 2. */
typedef struct {
    const uint64_t *row_ptr;
    const uint32_t *col_idx;
    int64_t n;
    uint32_t entry;
} leann_graph;

/* Raw chunk store as token ids: tokens[n][seq] (PAD beyond the valid length,
 * content ignored) and lengths[n] in [1, seq]; device pointers. */
typedef struct {
    const int32_t *tokens;
    const int32_t *lengths;
    int64_t n;
    int32_t seq;
} leann_chunks;

/* Optional table of stored exact embeddings (the paper's embedding cache for
 * frequently visited nodes, Sec. 3 / App. D "Relaxing Disk Constraint").
 * slot_of[n] gives the row of emb for a node, or -1 when the node must be
 * recomputed; emb[rows][d] fp32.  Device pointers.  NULL = recompute everything. */
typedef struct {
    const int32_t *slot_of;
    const float *emb;
    int64_t rows;
} leann_emb_cache;

/* Pending index updates seen by the output stage of a search (App. B "Soft
 * Deletion Strategy", "Batched Add Operation"):
 *   deleted_bits: bit (v & 31) of word (v >> 5) set = node v is soft-deleted; (n + 31) / 32
 *     words.  Deleted nodes are traversed as before (their adjacency lists stay); the exact
 *     queue is filtered by the flag before the k best active entries are returned.
 *   buffer_emb fp32[buffer_n][hidden], buffer_ids[buffer_n]: embeddings of added chunks that
 *     are not inserted into the graph yet.  Every one is scored exactly (<q, e>) and merged
 *     with the graph's result under (score descending, id ascending).
 * Device pointers, borrowed for the call; either part may be absent (NULL / 0). */
typedef struct {
    const uint32_t *deleted_bits;
    const float *buffer_emb;
    const uint32_t *buffer_ids;
    int64_t buffer_n;
} leann_updates;

/* Per-call totals over all queries of a leann_search call. */
typedef struct {
    int64_t hops;              /* exploration steps (Alg. 2: taking the best unvisited node of EQ) */
    int64_t adc_candidates;    /* neighbours scored with PQ */
    int64_t recomputed_chunks; /* exact scores taken (sum over queries, entry point included) */
    int64_t encoded_chunks;    /* chunks actually sent through the encoder (after sharing within a round) */
    int64_t encoded_tokens;    /* valid tokens of those chunks */
    int64_t flushes;           /* per-query batch flushes */
    int64_t rounds;            /* traverse -> encode -> insert rounds over the whole query set */
    int64_t cache_hits;        /* exact scores served by the stored-embedding table (part of recomputed_chunks) */
    int64_t memo_hits;         /* exact scores served by the call's embedding memo (leann_set_call_memo; part of recomputed_chunks) */
    float encoder_ms, traverse_ms, total_ms; /* device time (HIP events) */
} leann_search_stats;

/* Message of the last error on the calling thread.  ctx is accepted for symmetry with the other calls and may be
 * NULL (leann_create fails before a context exists); the string is per thread, not per context. */
const char *leann_last_error(const leann_ctx *ctx);

/*
 * Create a context holding the encoder weights.
 *   weights_dev: packed parameters on the device, dtype LEANN_F32 or LEANN_BF16
 *   (every value in that one type), in this order, linear maps stored [out][in]:
 *     tok_emb[vocab][d], pos_emb[max_pos][d], seg_emb[d], emb_ln_g[d], emb_ln_b[d],
 *     per layer: Wqkv[3d][d] (query rows, key rows, value rows), bqkv[3d], Wo[d][d], bo[d],
 *                ln1_g[d], ln1_b[d], W1[F][d], b1[F], W2[d][F], b2[d], ln2_g[d], ln2_b[d].
 *   The library keeps its own copy (matrices and embedding tables in bf16, the
 *   rest in fp32); the caller may free weights_dev after the call returns.
 *   Shapes covered: hidden/heads == 64, hidden % 128 == 0, ffn % 128 == 0,
 *   sequence length <= 256; anything else is LEANN_ESHAPE.
 *   device: HIP device ordinal; hip_stream: a hipStream_t (NULL = default stream).
 */
int leann_create(leann_ctx **out, const leann_encoder_desc *desc, const void *weights_dev, int weight_dtype,
                 int device, void *hip_stream);
void leann_destroy(leann_ctx *ctx);

/*
 * Embedding recomputation (Alg. 2, the recomputation step; Sec. 3 online stage).
 * For each requested chunk: x = LN(tok_emb[id_t] + pos_emb[t] + seg_emb), t < L;
 * per layer  x = LN(x + MHA(x) Wo + bo),  x = LN(x + GELU(x W1 + b1) W2 + b2)
 * with softmax over the L valid keys only; e = mean_t x_t;  e <- e / max(|e|, 1e-12).
 * bf16 matrix products with fp32 accumulation; softmax, LayerNorm and pooling in fp32.
 *   ids_dev: int64[n_ids] chunk numbers (device), NULL = chunks 0..n_ids-1.
 *   out_emb_dev: fp32[n_ids][hidden].
 * A chunk's embedding does not depend on which other chunks share the call.
 * Errors: token id outside [0, vocab), length outside [1, seq], id outside [0, n) -> LEANN_EINVAL.
 */
int leann_embed(leann_ctx *ctx, const leann_chunks *chunks, const int64_t *ids_dev, int64_t n_ids,
                float *out_emb_dev);

/*
 * Build the PQ table of the offline stage (Sec. 3: the index keeps a small PQ table of all embeddings).
 * Splits d into m_sub contiguous sub-vectors; per subspace runs `iters` Lloyd
 * iterations with 256 centroids on min(n, 65536) rows chosen by a seeded
 * permutation (splitmix64 Fisher-Yates; the first 256 rows of it are the initial
 * centroids; an empty cluster keeps its centroid; ties go to the lowest index),
 * then encodes all n rows.  emb_dev: fp32[n][d].  d/m_sub <= 32.
 */
int leann_build_pq(leann_ctx *ctx, const float *emb_dev, int64_t n, int32_t d, int32_t m_sub, int32_t iters,
                   uint64_t seed, leann_pq **out);
/* The PQ table is one of the two things the index stores (Sec. 3 "Storage composition": graph + PQ codes); the
 * calls below move it between the library and the caller.
 * Copy codebook fp32[m_sub][256][d/m_sub] and codes u8[n][m_sub] to host buffers (either may be NULL). */
int leann_pq_export(leann_ctx *ctx, const leann_pq *pq, float *codebook_host, uint8_t *codes_host);
/* Make a PQ table from host copies of a codebook and codes. */
int leann_pq_import(leann_ctx *ctx, const float *codebook_host, const uint8_t *codes_host, int64_t n, int32_t d,
                    int32_t m_sub, leann_pq **out);
/* Wrap a device-resident code table without copying it: codes_dev u8[n][m_sub] stays caller-owned and must
 * outlive the handle; the codebook is copied from the host. */
int leann_pq_wrap(leann_ctx *ctx, const float *codebook_host, const uint8_t *codes_dev, int64_t n, int32_t d,
                  int32_t m_sub, leann_pq **out);
int leann_pq_info(const leann_pq *pq, int64_t *n, int32_t *d, int32_t *m_sub);
void leann_pq_free(leann_pq *pq);

/*
 * Approximate scores (Alg. 2, the step that ranks a hop's new neighbours by their PQ distance to
 * the query before they enter AQ), product quantisation's asymmetric distance: for each query a lookup table
 * lut[m][c] = -|q_m - codebook[m][c]|^2 is built (sub-vector summed in index order)
 * and out[i][j] = sum_m lut[m][codes[cand[i][j]][m]] in the fixed order m = 0..m_sub-1,
 * fp32: the negated squared distance between q and the decoded vector (larger is closer).
 *   queries_dev fp32[nq][d]; cand_ids_dev u32[nq][nc]; out_dev fp32[nq][nc].
 * Candidate ids >= n are an error (LEANN_EINVAL, reported after the kernel ran; out_dev
 * then holds -inf at those positions).
 */
int leann_adc(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_pq *pq,
              const uint32_t *cand_ids_dev, int32_t nc, float *out_dev);

/*
 * leann_adc for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same kernels and same results as leann_adc; the
 * per-query lookup tables live in a fixed array inside the library (4 MiB + 256 bytes per GPU, held
 * until the process ends) instead of a grown workspace.  The call allocates nothing, records no
 * memset and does not synchronise: the work is enqueued on the context's stream.
 *   Limits: nq <= 128 and m_sub <= 32; anything larger -> LEANN_ECAPACITY, nothing enqueued.
 *   A candidate id >= n is not reported through the status (that would need a synchronisation):
 *   out_dev holds -inf at its position.
 *   All calls on one GPU share the array: calls that overlap on one GPU (different streams or
 *   contexts) race; calls on one stream are ordered and safe.
 */
int leann_adc_noalloc(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_pq *pq,
                      const uint32_t *cand_ids_dev, int32_t nc, float *out_dev);

/*
 * Two-level search with dynamic batching (Algorithm 2, Sec. 4.1-4.2) for nq
 * independent queries, all stages on the device.
 * Per query: EQ (exact queue, size ef) starts with the entry point's exact score.
 * Each hop reads the best unvisited node u of EQ, marks it visited, ADC-scores the
 * neighbours of u that have no ADC score yet and pushes them into AQ, then moves the
 * r = ceil(rerank_ratio * number of those new neighbours) best entries of AQ (fp32
 * product; AQ holds every ADC-scored node not yet recomputed) to the pending list P.
 * When |P| >= batch, or EQ has no unvisited node, the chunks in P are re-embedded,
 * scored by inner product with the query and try-inserted into EQ in P's order
 * (insert when EQ is not full or the score beats EQ's worst entry, which is evicted).
 * The search ends when EQ has no unvisited node and P is empty; the k best of EQ
 * are returned, padded with id -1 / score -inf.
 * A query's result does not depend on nq or on the other queries of the call:
 * the encoder batches across queries, never changing a chunk's embedding.
 *   queries_dev fp32[nq][hidden]; out_ids_dev int64[nq][k]; out_scores_dev fp32[nq][k];
 *   cache: optional stored embeddings (NULL = none; a slot_of entry >= rows -> LEANN_EINVAL);
 *   stats_host: optional totals.
 * Errors: k < 1, k > ef, ef > 1024, rerank_ratio outside (0,1], batch < 1, entry >= n,
 * graph/chunk/PQ sizes that disagree -> LEANN_EINVAL / LEANN_ESHAPE; a neighbour id >= n
 * or a per-query queue overflow -> LEANN_EINVAL / LEANN_ECAPACITY after the run
 * (outputs then undefined).  Synchronises the stream before returning.
 */
int leann_search(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_graph *graph,
                 const leann_pq *pq, const leann_chunks *chunks, const leann_emb_cache *cache, int32_t ef,
                 int32_t k, float rerank_ratio, int32_t batch, int64_t *out_ids_dev, float *out_scores_dev,
                 leann_search_stats *stats_host);

/* leann_search with pending updates (see leann_updates); updates == NULL is leann_search.
 * Errors as leann_search, plus LEANN_EINVAL for a buffer with null pointers or more than
 * 2^24 rows. */
int leann_search_updates(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_graph *graph,
                         const leann_pq *pq, const leann_chunks *chunks, const leann_emb_cache *cache,
                         const leann_updates *updates, int32_t ef, int32_t k, float rerank_ratio, int32_t batch,
                         int64_t *out_ids_dev, float *out_scores_dev, leann_search_stats *stats_host);

/*
 * Index graph construction by insertion (Algorithm 3 with the node-insertion listing of
 * the update appendix).  Nodes enter in id order.  For node v: W = best-first search
 * (Algorithm 1, exact similarities <e_v, e_x> from emb, queue length efC, start at node 0)
 * on the graph built so far; neighbours = RNG selection from W (walk by descending
 * similarity, keep x unless a kept y has <e_x, e_y> > <e_x, e_v>), at most M for nodes
 * flagged in is_hub (NULL: every node), m for the others; edges are added in both
 * directions, and a neighbour whose list exceeds M is shrunk to M with the same rule.
 * Total order (similarity descending, id ascending).
 * batch > 1: the nodes of a batch search the graph as it was before the batch (one
 * wavefront each), then their edges are committed in id order and every node that
 * received edges is shrunk once; batch k holds min(batch, max(1, inserted / ramp)) nodes.
 * batch = 1 is the sequential listing.
 *   emb_dev fp32[n][d] (device); is_hub_dev uint8[n] or NULL (device);
 *   row_ptr_dev uint64[n + 1], col_idx_dev uint32 with room for n * M entries (device,
 *   caller-owned); n_edges_host receives the edge count.  Scratch is allocated and freed
 *   inside the call (n * (M + batch) * 4 + batch * n * 2 bytes).  Synchronises the stream.
 * Errors: efC outside 1..256, M outside 1..64, m outside 1..M, batch outside 1..1024,
 * ramp < 1, n >= 2^31 -> LEANN_EINVAL.
 */
int leann_build_graph(leann_ctx *ctx, const float *emb_dev, int64_t n, int32_t d, const uint8_t *is_hub_dev,
                      int32_t efC, int32_t M, int32_t m, int32_t batch, int32_t ramp, uint64_t *row_ptr_dev,
                      uint32_t *col_idx_dev, int64_t *n_edges_host);

/* Algorithm 3's set V* of highest-degree nodes: is_hub_dev[v] = 1 for the
 * ceil(beta * n) nodes of largest out-degree in the CSR graph (ties: lower id), else 0.
 * Degrees above 4096 -> LEANN_ECAPACITY. */
int leann_top_degree(leann_ctx *ctx, const uint64_t *row_ptr_dev, int64_t n, double beta, uint8_t *is_hub_dev);

/* Tuning knobs (all optional): largest number of tokens one encoder pass holds
 * (workspace size), and the per-query capacity of the approximate queue. */
int leann_set_limits(leann_ctx *ctx, int64_t max_tokens_per_pass, int32_t aq_capacity);
/* Per-call embedding memo (off by default; an option for throughput with many queries per call): with max_rows > 0
 * a leann_search call keeps up to max_rows embeddings that its own encoder passes produced (max_rows * hidden * 4 bytes
 * of device memory plus 4 bytes per node) and serves a later request for the same chunk, by any query of the same call,
 * from there instead of encoding it again.  The memo is empty at the start of every call: nothing computed in one call
 * is reused in another, and nothing is stored with the index.  A chunk's embedding does not depend on its batch, so
 * ids, scores and every per-query count are unchanged; encoded_chunks drops and memo_hits counts the requests served.
 * Without it, requests for one chunk are merged only within a round.  max_rows = 0 turns it off and frees its memory. */
int leann_set_call_memo(leann_ctx *ctx, int64_t max_rows);
/* GEMM tile choice of the encoder (a tuning and test aid; results do not depend on it, every tile adds the K-slabs
 * in the same order): large_tile 256 (default) or 128 = block tile for passes of more than 8192 padded rows
 * (0 leaves it); small_rows = passes of at most this many padded rows use 64x64 tiles (default 2048). */
int leann_set_gemm_tiles(leann_ctx *ctx, int32_t large_tile, int32_t small_rows);

/*
 * Per-kernel device timing for the benchmark: between leann_profile_begin and leann_profile_end every kernel
 * the library launches on this context is bracketed by HIP events on the context's stream.  ms[i] / launches[i]
 * give summed duration and launch count per kernel family; tokens = valid tokens that went through the encoder,
 * so that the GEMM work is tokens * layers * 2 * (4*hidden^2 + 2*hidden*ffn) flops.  leann_profile_end
 * synchronises the stream.
 */
enum {
    LEANN_PROF_GEMM_QKV = 0, LEANN_PROF_GEMM_O, LEANN_PROF_GEMM_FFN1, LEANN_PROF_GEMM_FFN2, LEANN_PROF_ATTENTION,
    LEANN_PROF_LAYERNORM, LEANN_PROF_ENC_OTHER, LEANN_PROF_TRAVERSE, LEANN_PROF_COLLECT, LEANN_PROF_SCORE_INSERT,
    LEANN_PROF_LUT, LEANN_PROF_ADC, LEANN_PROF_KINDS
};
typedef struct {
    double ms[LEANN_PROF_KINDS];
    int64_t launches[LEANN_PROF_KINDS];
    int64_t tokens;
} leann_profile;
int leann_profile_begin(leann_ctx *ctx);
int leann_profile_end(leann_ctx *ctx, leann_profile *out_host);

/*
 * Measured denominator for the encoder's roofline (benchmark hook, not on the search path): the rate this GPU
 * sustains on nothing but independent bf16 MFMA 32x32x16 instructions (8 accumulators per wave, the GEMM's wave
 * tile), `launches` launches of blocks_per_cu (1 or 2) blocks of four waves per compute unit, `iters` rounds each.
 * operand_kind: 0 zeros, 1 values near one, 2 random sign / exponent in [2^-4, 2) / mantissa.
 * tflops_host receives TFLOP/s over the timed launches (HIP events on the context's stream, after three warm-up
 * launches), ms_host (optional) the average launch duration.  Allocates and frees its buffers; synchronises.
 */
int leann_bench_mfma(leann_ctx *ctx, int32_t operand_kind, int32_t blocks_per_cu, int32_t iters, int32_t launches,
                     double *tflops_host, double *ms_host);

/*
 * Measured ceiling of the ADC scorer's access pattern (benchmark hook): 67 108 864 gathers per launch of uniformly
 * random 32-byte rows from table_dev (u8[table_rows][32], device, caller-owned), nothing else.  rows_per_s_host
 * receives rows per second over `launches` timed launches after one warm-up launch, ms_host (optional) the average
 * launch duration.  Allocates and frees 0.27 GB of ids; synchronises.
 */
int leann_bench_gather(leann_ctx *ctx, const uint8_t *table_dev, int64_t table_rows, int32_t launches,
                       double *rows_per_s_host, double *ms_host);

/*
 * Measured ceiling of the GEMM's operand feed (benchmark hook): one block of eight waves per compute unit does nothing
 * but the GEMM's operand loads (16 bytes per lane, 64-byte row pieces of 1536-byte rows, eight in flight per lane) over
 * a panel of panel_rows rows allocated inside the call: a panel of a few MB is served by the L2, a large one by memory.
 * bytes_per_s_host receives the rate over `launches` timed launches after one warm-up launch.  Synchronises.
 */
int leann_bench_l1pull(leann_ctx *ctx, int64_t panel_rows, int32_t launches, double *bytes_per_s_host, double *ms_host);

#ifdef __cplusplus
}
#endif
#endif /* LEANN_H */

// C ABI of libleann: context life cycle, argument checks, and the embed / search entry points.
#include <stdarg.h>
#include <stdio.h>

#include "common.h"

static thread_local char g_err[512] = "";

void leann_set_error(const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int DevBuf::reserve(size_t need)
{
    if (need <= bytes) return LEANN_OK;
    if (p) {
        (void)hipFree(p);
        p = nullptr;
        bytes = 0;
    }
    hipError_t e = hipMalloc(&p, need);
    if (e != hipSuccess) {
        p = nullptr;
        leann_set_error("device allocation of %zu bytes failed: %s", need, hipGetErrorString(e));
        (void)hipGetLastError();
        return LEANN_ENOMEM;
    }
    bytes = need;
    return LEANN_OK;
}

void DevBuf::release()
{
    if (p) (void)hipFree(p);
    p = nullptr;
    bytes = 0;
}

ProfScope::ProfScope(leann_ctx *c, int kind) : ctx(c)
{
    if (!c->prof_on) return;
    hipEvent_t a = nullptr;
    for (hipEvent_t *e : {&a, &b}) {
        if (!c->prof_pool.empty()) {
            *e = c->prof_pool.back();
            c->prof_pool.pop_back();
        } else if (hipEventCreate(e) != hipSuccess) {
            *e = nullptr;
        }
    }
    if (!a || !b) {
        b = nullptr;
        return;
    }
    (void)hipEventRecord(a, c->stream);
    c->prof_spans.push_back({kind, a, b});
}

ProfScope::~ProfScope()
{
    if (b) (void)hipEventRecord(b, ctx->stream);
}

namespace {

__global__ void f32_to_bf16_kernel(const float *__restrict__ in, bf16_t *__restrict__ out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        out[i] = (bf16_t)in[i];
}
__global__ void bf16_to_f32_kernel(const bf16_t *__restrict__ in, float *__restrict__ out, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        out[i] = (float)in[i];
}

size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// copies `count` packed source elements starting at element `src_off` into an own bf16 / fp32 buffer; a failed
// copy is remembered in *status (the first one wins)
void to_bf16(hipError_t *status, leann_ctx *ctx, const void *src, int dtype, size_t src_off, size_t count, bf16_t *dst)
{
    const unsigned grid = (unsigned)std::min<size_t>((count + 255) / 256, 4096);
    if (dtype == LEANN_F32)
        hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(grid), dim3(256), 0, ctx->stream, (const float *)src + src_off, dst,
                           count);
    else
    {
        const hipError_t e = hipMemcpyAsync(dst, (const bf16_t *)src + src_off, count * sizeof(bf16_t),
                                            hipMemcpyDeviceToDevice, ctx->stream);
        if (*status == hipSuccess) *status = e;
    }
}
void to_f32(hipError_t *status, leann_ctx *ctx, const void *src, int dtype, size_t src_off, size_t count, float *dst)
{
    const unsigned grid = (unsigned)std::min<size_t>((count + 255) / 256, 4096);
    if (dtype == LEANN_BF16)
        hipLaunchKernelGGL(bf16_to_f32_kernel, dim3(grid), dim3(256), 0, ctx->stream, (const bf16_t *)src + src_off, dst,
                           count);
    else
    {
        const hipError_t e = hipMemcpyAsync(dst, (const float *)src + src_off, count * sizeof(float),
                                            hipMemcpyDeviceToDevice, ctx->stream);
        if (*status == hipSuccess) *status = e;
    }
}

}  // namespace

extern "C" {

const char *leann_last_error(const leann_ctx *) { return g_err; }

int leann_create(leann_ctx **out, const leann_encoder_desc *desc, const void *weights_dev, int weight_dtype, int device,
                 void *hip_stream)
{
    if (!out || !desc || !weights_dev || (weight_dtype != LEANN_F32 && weight_dtype != LEANN_BF16)) {
        leann_set_error("leann_create: null argument or unknown weight dtype");
        return LEANN_EINVAL;
    }
    const leann_encoder_desc &e = *desc;
    if (e.layers < 0 || e.hidden < 1 || e.heads < 1 || e.ffn < 1 || e.vocab < 1 || e.max_pos < 1 || !(e.ln_eps >= 0.f)) {
        leann_set_error("leann_create: non-positive encoder dimension");
        return LEANN_EINVAL;
    }
    if (e.hidden % e.heads || e.hidden / e.heads != 64 || e.hidden % 128 || e.ffn % 128 || e.hidden > 1024) {
        leann_set_error("encoder shape not covered: need hidden/heads == 64, hidden %% 128 == 0 (<= 1024), ffn %% 128 == 0");
        return LEANN_ESHAPE;
    }
    int ndev = 0;
    LEANN_HIP(hipGetDeviceCount(&ndev));
    if (device < 0 || device >= ndev) {
        leann_set_error("leann_create: device %d of %d", device, ndev);
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(device));
    LEANN_TRY(enc_init_device());
    LEANN_TRY(pq_init_device());
    LEANN_TRY(search_init_device());
    leann_ctx *ctx = new leann_ctx();
    ctx->desc = e;
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, device) == hipSuccess && prop.multiProcessorCount >= 8)
            ctx->num_cus = prop.multiProcessorCount;
    }
    if (enc_ln_blocks_per_cu(&ctx->ln_blocks_per_cu) != LEANN_OK) {
        leann_destroy(ctx);
        return LEANN_EDEVICE;
    }
    const size_t d = e.hidden, F = e.ffn, L = e.layers;
    const size_t n_emb = ((size_t)e.vocab + e.max_pos + 1) * d;
    size_t bf_bytes = up256(e.vocab * d * 2) + up256(e.max_pos * d * 2) + up256(d * 2) +
                      L * (up256(3 * d * d * 2) + up256(d * d * 2) + 2 * up256(F * d * 2));
    size_t f_bytes = 2 * up256(d * 4) + L * (up256(3 * d * 4) + 6 * up256(d * 4) + up256(F * 4));
    if (ctx->w_bf16.reserve(bf_bytes) != LEANN_OK || ctx->w_f32.reserve(f_bytes) != LEANN_OK) {
        leann_destroy(ctx);
        return LEANN_ENOMEM;
    }
    char *pb = (char *)ctx->w_bf16.p, *pf = (char *)ctx->w_f32.p;
    size_t so = 0;  // element offset in the packed source
    hipError_t copy_rc = hipSuccess;
    auto mat = [&](size_t count) {
        bf16_t *dst = (bf16_t *)pb;
        to_bf16(&copy_rc, ctx, weights_dev, weight_dtype, so, count, dst);
        pb += up256(count * 2);
        so += count;
        return (const bf16_t *)dst;
    };
    auto vec = [&](size_t count) {
        float *dst = (float *)pf;
        to_f32(&copy_rc, ctx, weights_dev, weight_dtype, so, count, dst);
        pf += up256(count * 4);
        so += count;
        return (const float *)dst;
    };
    ctx->tok_emb = mat((size_t)e.vocab * d);
    ctx->pos_emb = mat((size_t)e.max_pos * d);
    ctx->seg_emb = mat(d);
    ctx->emb_g = vec(d);
    ctx->emb_b = vec(d);
    (void)n_emb;
    ctx->layers.resize(L);
    for (size_t l = 0; l < L; ++l) {
        LayerWeights &w = ctx->layers[l];
        w.wqkv = mat(3 * d * d);
        w.bqkv = vec(3 * d);
        w.wo = mat(d * d);
        w.bo = vec(d);
        w.g1 = vec(d);
        w.be1 = vec(d);
        w.w1 = mat(F * d);
        w.b1 = vec(F);
        w.w2 = mat(d * F);
        w.b2 = vec(d);
        w.g2 = vec(d);
        w.be2 = vec(d);
    }
    hipError_t rc = hipGetLastError();
    if (rc == hipSuccess) rc = copy_rc;
    if (rc == hipSuccess) rc = hipStreamSynchronize(ctx->stream);
    if (rc != hipSuccess) {
        leann_set_error("copying the weights failed: %s", hipGetErrorString(rc));
        leann_destroy(ctx);
        return LEANN_EDEVICE;
    }
    *out = ctx;
    return LEANN_OK;
}

void leann_destroy(leann_ctx *ctx)
{
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    DevBuf *bufs[] = {&ctx->w_bf16, &ctx->w_f32, &ctx->x, &ctx->qkv, &ctx->att, &ctx->delta, &ctx->hid, &ctx->cu,
                      &ctx->len, &ctx->meta, &ctx->enc_ids, &ctx->s_state, &ctx->s_emb, &ctx->s_lut, &ctx->s_seen,
                      &ctx->s_misc, &ctx->s_owner, &ctx->s_buf, &ctx->s_memo_slot, &ctx->s_memo_emb};
    for (DevBuf *b : bufs) b->release();
    ctx->prof_tokens.release();
    for (auto &sp : ctx->prof_spans) {
        (void)hipEventDestroy(sp.a);
        (void)hipEventDestroy(sp.b);
    }
    for (hipEvent_t e : ctx->prof_pool) (void)hipEventDestroy(e);
    delete ctx;
}

int leann_set_limits(leann_ctx *ctx, int64_t max_tokens_per_pass, int32_t aq_capacity)
{
    if (!ctx || max_tokens_per_pass < 0 || aq_capacity < 0) {
        leann_set_error("leann_set_limits: null context or negative limit");
        return LEANN_EINVAL;
    }
    if (max_tokens_per_pass > 0) ctx->max_tokens = std::min<int64_t>(max_tokens_per_pass, (int64_t)1 << 22);
    if (aq_capacity > 0) ctx->aq_capacity = aq_capacity;
    return LEANN_OK;
}

int leann_set_gemm_tiles(leann_ctx *ctx, int32_t large_tile, int32_t small_rows)
{
    if (!ctx || (large_tile != 0 && large_tile != 128 && large_tile != 256) || small_rows < 0) {
        leann_set_error("leann_set_gemm_tiles: null context, a large tile other than 128 / 256, or a negative row limit");
        return LEANN_EINVAL;
    }
    if (large_tile) ctx->gemm_large_tile = large_tile;
    ctx->gemm_small_rows = small_rows;
    return LEANN_OK;
}

int leann_set_call_memo(leann_ctx *ctx, int64_t max_rows)
{
    if (!ctx || max_rows < 0) {
        leann_set_error("leann_set_call_memo: null context or negative row count");
        return LEANN_EINVAL;
    }
    ctx->memo_rows = max_rows;
    if (max_rows == 0) {
        ctx->s_memo_slot.release();
        ctx->s_memo_emb.release();
    }
    return LEANN_OK;
}

int leann_profile_begin(leann_ctx *ctx)
{
    if (!ctx) {
        leann_set_error("leann_profile_begin: null context");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    LEANN_TRY(ctx->prof_tokens.reserve(sizeof(int64_t)));
    LEANN_HIP(hipMemsetAsync(ctx->prof_tokens.p, 0, sizeof(int64_t), ctx->stream));
    for (auto &sp : ctx->prof_spans) {
        ctx->prof_pool.push_back(sp.a);
        ctx->prof_pool.push_back(sp.b);
    }
    ctx->prof_spans.clear();
    ctx->prof_on = true;
    return LEANN_OK;
}

int leann_profile_end(leann_ctx *ctx, leann_profile *out_host)
{
    if (!ctx || !out_host) {
        leann_set_error("leann_profile_end: null argument");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    ctx->prof_on = false;
    *out_host = leann_profile{};
    LEANN_HIP(hipStreamSynchronize(ctx->stream));
    if (ctx->prof_tokens.p)
        LEANN_HIP(hipMemcpy(&out_host->tokens, ctx->prof_tokens.p, sizeof(int64_t), hipMemcpyDeviceToHost));
    for (auto &sp : ctx->prof_spans) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, sp.a, sp.b) == hipSuccess) {
            out_host->ms[sp.kind] += t;
            out_host->launches[sp.kind] += 1;
        }
        ctx->prof_pool.push_back(sp.a);
        ctx->prof_pool.push_back(sp.b);
    }
    ctx->prof_spans.clear();
    return LEANN_OK;
}

static int check_chunks(const leann_ctx *ctx, const leann_chunks *chunks)
{
    if (!chunks || !chunks->tokens || !chunks->lengths || chunks->n < 1) {
        leann_set_error("chunk store: null pointer or no chunks");
        return LEANN_EINVAL;
    }
    if (chunks->seq < 1 || chunks->seq > 256 || chunks->seq > ctx->desc.max_pos) {
        leann_set_error("chunk store: sequence length %d not covered (1..min(256, max_pos))", chunks->seq);
        return LEANN_ESHAPE;
    }
    return LEANN_OK;
}

int leann_embed(leann_ctx *ctx, const leann_chunks *chunks, const int64_t *ids_dev, int64_t n_ids, float *out_emb_dev)
{
    if (!ctx || n_ids < 0 || (n_ids > 0 && !out_emb_dev)) {
        leann_set_error("leann_embed: null argument or negative count");
        return LEANN_EINVAL;
    }
    LEANN_TRY(check_chunks(ctx, chunks));
    if (!ids_dev && n_ids > chunks->n) {
        leann_set_error("leann_embed: %lld chunks requested, the store holds %lld", (long long)n_ids, (long long)chunks->n);
        return LEANN_EINVAL;
    }
    if (n_ids == 0) return LEANN_OK;
    LEANN_HIP(hipSetDevice(ctx->device));
    LEANN_TRY(ctx->meta.reserve(256));
    int *err = (int *)ctx->meta.p;
    LEANN_HIP(hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
    LEANN_TRY(enc_forward(ctx, chunks, ids_dev, 0, n_ids, out_emb_dev, err, nullptr));
    int herr = 0;
    LEANN_HIP(hipMemcpyAsync(&herr, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    LEANN_HIP(hipStreamSynchronize(ctx->stream));
    if (herr) {
        leann_set_error("leann_embed: %s%s%s", (herr & 1) ? "chunk id outside the store; " : "",
                        (herr & 2) ? "length outside [1, seq]; " : "", (herr & 4) ? "token id outside [0, vocab)" : "");
        return LEANN_EINVAL;
    }
    return LEANN_OK;
}

int leann_search(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_graph *graph, const leann_pq *pq,
                 const leann_chunks *chunks, const leann_emb_cache *cache, int32_t ef, int32_t k, float rerank_ratio,
                 int32_t batch, int64_t *out_ids_dev, float *out_scores_dev, leann_search_stats *stats_host)
{
    return leann_search_updates(ctx, queries_dev, nq, graph, pq, chunks, cache, nullptr, ef, k, rerank_ratio, batch,
                                out_ids_dev, out_scores_dev, stats_host);
}

int leann_search_updates(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_graph *graph,
                         const leann_pq *pq, const leann_chunks *chunks, const leann_emb_cache *cache,
                         const leann_updates *updates, int32_t ef, int32_t k, float rerank_ratio, int32_t batch,
                         int64_t *out_ids_dev, float *out_scores_dev, leann_search_stats *stats_host)
{
    if (!ctx || !graph || !pq || nq < 0 || (nq > 0 && (!queries_dev || !out_ids_dev || !out_scores_dev))) {
        leann_set_error("leann_search: null argument or negative query count");
        return LEANN_EINVAL;
    }
    LEANN_TRY(check_chunks(ctx, chunks));
    if (!graph->row_ptr || !graph->col_idx || graph->n < 1 || graph->entry >= (uint64_t)graph->n) {
        leann_set_error("leann_search: graph pointers null, empty graph or entry point outside it");
        return LEANN_EINVAL;
    }
    if (k < 1 || k > ef || ef > 1024 || !(rerank_ratio > 0.f) || rerank_ratio > 1.f || batch < 1) {
        leann_set_error("leann_search: need 1 <= k <= ef <= 1024, 0 < rerank_ratio <= 1, batch >= 1");
        return LEANN_EINVAL;
    }
    if (graph->n != chunks->n || graph->n != pq->n || pq->d != ctx->desc.hidden || graph->n > 0xffffffffll) {
        leann_set_error("leann_search: graph (%lld nodes), chunk store (%lld), PQ table (%lld rows, d=%d) and encoder (d=%d) disagree",
                        (long long)graph->n, (long long)chunks->n, (long long)pq->n, pq->d, ctx->desc.hidden);
        return LEANN_ESHAPE;
    }
    if (cache && (!cache->slot_of || !cache->emb || cache->rows < 0 || cache->rows > (1ll << 30))) {
        leann_set_error("leann_search: embedding cache with null pointers or a row count outside 0..2^30");
        return LEANN_EINVAL;
    }
    if (updates && (updates->buffer_n < 0 || updates->buffer_n > (1 << 24) ||
                    (updates->buffer_n > 0 && (!updates->buffer_emb || !updates->buffer_ids)))) {
        leann_set_error("leann_search: add buffer with null pointers or a row count outside 0..2^24");
        return LEANN_EINVAL;
    }
    if (stats_host) *stats_host = leann_search_stats{};
    if (nq == 0) return LEANN_OK;
    LEANN_HIP(hipSetDevice(ctx->device));
    return search_run(ctx, queries_dev, nq, graph, pq, chunks, cache, updates, ef, k, rerank_ratio, batch, out_ids_dev,
                      out_scores_dev, stats_host);
}

}  // extern "C"

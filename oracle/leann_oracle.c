/*
 * LEANN search hot path -- CPU ORACLE (test infrastructure, not product code).
 *
 * Plain, slow, scalar C.  It exists so that tests, the smoke check and the
 * benchmark's cpu_baseline leg have something obviously correct to compare
 * the GPU library with.  Nothing in the product path may call it, and it
 * shares no code, header, table or helper with the GPU sources.
 *
 * What it follows (LEANN, arXiv 2506.08276):
 *   - encoder: the paper only fixes "a BERT-style 110 M-parameter encoder,
 *     768-d output, 256-token chunks" (Sec. 7 set-up, App. D); the layer
 *     equations below are the standard post-LN transformer encoder with
 *     masked mean pooling and L2 normalisation;
 *   - PQ / ADC: the paper cites product quantisation and only gives its
 *     size (Sec. 3 "Storage composition", Sec. 4.1 "Discussion"); the
 *     textbook train / encode / asymmetric-distance (squared L2)
 *     definitions are used;
 *   - search: Algorithm 2 (two-level search, Sec. 4.1) with the batching
 *     rule of Sec. 4.2; Algorithm 1 (Sec. 2) is its alpha = 1, batch = 1
 *     special case; Eq. 1 is the exact top-k used as ground truth.
 *
 * Arithmetic is fp32 (the precision the spec parity bounds are
 * stated against); k-means centroid means accumulate in fp64.  OpenMP is
 * used only across independent chunks.
 *
 * Parity pins live in tests/test_oracle_*.py.  Unpinned by the paper (it
 * prints no worked example): the numerical output of the real trained
 * encoder, and the search trajectory under the readings listed in the
 * design notes (only the alpha = 1 reductions and the invariants are
 * pinned).
 * Parity unpinned: the precision = 1 mode of orc_embed (bf16 rounding at
 * the places a bf16 pipeline stores its tensors).  It is a diagnostic that
 * gives a tighter second bound for the GPU encoder; its only pin is that it
 * stays close to the fp32 mode.  No parity claim rests on it: the parity
 * bounds are asserted against the fp32 mode, and no test uses it to choose
 * what is compared.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_ENOMEM (-2)

typedef struct {
    int32_t layers, hidden, heads, ffn, vocab, max_pos;
    float ln_eps;
} orc_encoder_desc;

/* ------------------------------------------------------------------ */
/* small helpers                                                       */
/* ------------------------------------------------------------------ */

/* round-to-nearest-even fp32 -> bf16 -> fp32 (used only in precision mode 1,
 * which mimics the storage precision of a bf16 pipeline with fp32 sums). */
static float bf16_rne(float x)
{
    uint32_t u;
    memcpy(&u, &x, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return x;
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&x, &u, 4);
    return x;
}

/* splitmix64: the counter-based generator used for every random draw the
 * method itself makes (k-means initialisation / training sample). */
static uint64_t splitmix64(uint64_t *state)
{
    uint64_t z = (*state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

/* Seeded Fisher-Yates permutation of 0..n-1 (i from n-1 down to 1,
 * j = draw mod (i+1)). */
int orc_permutation(int64_t n, uint64_t seed, int64_t *perm)
{
    if (n < 0 || !perm) return ORC_EINVAL;
    for (int64_t i = 0; i < n; ++i) perm[i] = i;
    uint64_t st = seed;
    for (int64_t i = n - 1; i >= 1; --i) {
        uint64_t j = splitmix64(&st) % (uint64_t)(i + 1);
        int64_t t = perm[i];
        perm[i] = perm[j];
        perm[j] = t;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* C1. encoder                                                         */
/* ------------------------------------------------------------------ */
/*
 * Packed weight order (all fp32, row-major; a linear map y = x W^T + b is
 * stored as W[out][in]):
 *   tok_emb[vocab][d], pos_emb[max_pos][d], seg_emb[d], emb_ln_g[d], emb_ln_b[d],
 *   then per layer:
 *   Wqkv[3d][d] (q rows, k rows, v rows), bqkv[3d], Wo[d][d], bo[d],
 *   ln1_g[d], ln1_b[d], W1[F][d], b1[F], W2[d][F], b2[d], ln2_g[d], ln2_b[d].
 */
int64_t orc_weight_count(const orc_encoder_desc *e)
{
    int64_t d = e->hidden, F = e->ffn;
    int64_t per_layer = 3 * d * d + 3 * d + d * d + d + 2 * d + F * d + F + d * F + d + 2 * d;
    return (int64_t)e->vocab * d + (int64_t)e->max_pos * d + d + 2 * d + e->layers * per_layer;
}

typedef struct {
    const float *tok, *pos, *seg, *eg, *eb;
} emb_w;
typedef struct {
    const float *wqkv, *bqkv, *wo, *bo, *g1, *b1n, *w1, *b1, *w2, *b2, *g2, *b2n;
} layer_w;

static const float *take(const float **p, int64_t n)
{
    const float *r = *p;
    *p += n;
    return r;
}

static void split_weights(const orc_encoder_desc *e, const float *w, emb_w *ew, layer_w *lw)
{
    int64_t d = e->hidden, F = e->ffn;
    ew->tok = take(&w, (int64_t)e->vocab * d);
    ew->pos = take(&w, (int64_t)e->max_pos * d);
    ew->seg = take(&w, d);
    ew->eg = take(&w, d);
    ew->eb = take(&w, d);
    for (int l = 0; l < e->layers; ++l) {
        lw[l].wqkv = take(&w, 3 * d * d);
        lw[l].bqkv = take(&w, 3 * d);
        lw[l].wo = take(&w, d * d);
        lw[l].bo = take(&w, d);
        lw[l].g1 = take(&w, d);
        lw[l].b1n = take(&w, d);
        lw[l].w1 = take(&w, F * d);
        lw[l].b1 = take(&w, F);
        lw[l].w2 = take(&w, d * F);
        lw[l].b2 = take(&w, d);
        lw[l].g2 = take(&w, d);
        lw[l].b2n = take(&w, d);
    }
}

/* LayerNorm over one row: biased variance, statistics in fp32. */
static void layer_norm(float *row, int d, const float *g, const float *b, float eps, int prec)
{
    float mean = 0.f;
    for (int i = 0; i < d; ++i) mean += row[i];
    mean /= (float)d;
    float var = 0.f;
    for (int i = 0; i < d; ++i) {
        float c = row[i] - mean;
        var += c * c;
    }
    var /= (float)d;
    float inv = 1.0f / sqrtf(var + eps);
    for (int i = 0; i < d; ++i) {
        float y = (row[i] - mean) * inv * g[i] + b[i];
        row[i] = prec ? bf16_rne(y) : y;
    }
}

/* y[t][o] = sum_i x[t][i] W[o][i] + b[o], one token at a time. */
static void linear(const float *x, int L, int in, const float *W, const float *b, int out, float *y)
{
    for (int t = 0; t < L; ++t)
        for (int o = 0; o < out; ++o) {
            const float *xr = x + (int64_t)t * in, *wr = W + (int64_t)o * in;
            float acc = 0.f;
            for (int i = 0; i < in; ++i) acc += xr[i] * wr[i];
            y[(int64_t)t * out + o] = acc + b[o];
        }
}

static float gelu_erf(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f)); }

/* One chunk.  prec = 0: plain fp32.  prec = 1: every tensor a bf16 pipeline
 * would keep in memory (post-LN activations, QKV, softmax weights entering
 * the value product, attention output, GELU output, the output of the two
 * projections that feed a residual add) is rounded to bf16;
 * sums, softmax and LN statistics stay fp32.  Weights are expected to be
 * rounded by the caller in that mode (orc_embed does it). */
static int encode_chunk(const orc_encoder_desc *e, const emb_w *ew, const layer_w *lw, const int32_t *ids,
                        int L, int prec, float *out)
{
    const int d = e->hidden, H = e->heads, F = e->ffn, dh = d / H;
    float *x = malloc(sizeof(float) * (size_t)L * d);
    float *qkv = malloc(sizeof(float) * (size_t)L * 3 * d);
    float *att = malloc(sizeof(float) * (size_t)L * d);
    float *y = malloc(sizeof(float) * (size_t)L * d);
    float *hid = malloc(sizeof(float) * (size_t)L * F);
    float *p = malloc(sizeof(float) * (size_t)L);
    if (!x || !qkv || !att || !y || !hid || !p) {
        free(x); free(qkv); free(att); free(y); free(hid); free(p);
        return ORC_ENOMEM;
    }
    for (int t = 0; t < L; ++t) {
        const float *te = ew->tok + (int64_t)ids[t] * d, *pe = ew->pos + (int64_t)t * d;
        for (int i = 0; i < d; ++i) x[(int64_t)t * d + i] = te[i] + pe[i] + ew->seg[i];
        layer_norm(x + (int64_t)t * d, d, ew->eg, ew->eb, e->ln_eps, prec);
    }
    const float scale = 1.0f / sqrtf((float)dh);
    for (int l = 0; l < e->layers; ++l) {
        const layer_w *w = &lw[l];
        linear(x, L, d, w->wqkv, w->bqkv, 3 * d, qkv);
        if (prec)
            for (int64_t i = 0; i < (int64_t)L * 3 * d; ++i) qkv[i] = bf16_rne(qkv[i]);
        for (int h = 0; h < H; ++h)
            for (int i = 0; i < L; ++i) {
                const float *qi = qkv + (int64_t)i * 3 * d + h * dh;
                float mx = -INFINITY;
                for (int j = 0; j < L; ++j) { /* keys j >= L do not exist: masked */
                    const float *kj = qkv + (int64_t)j * 3 * d + d + h * dh;
                    float s = 0.f;
                    for (int c = 0; c < dh; ++c) s += qi[c] * kj[c];
                    p[j] = s * scale;
                    if (p[j] > mx) mx = p[j];
                }
                float den = 0.f;
                for (int j = 0; j < L; ++j) {
                    p[j] = expf(p[j] - mx);
                    den += p[j];
                }
                float *ai = att + (int64_t)i * d + h * dh;
                for (int c = 0; c < dh; ++c) {
                    float acc = 0.f;
                    for (int j = 0; j < L; ++j) {
                        float pj = prec ? bf16_rne(p[j]) : p[j];
                        acc += pj * qkv[(int64_t)j * 3 * d + 2 * d + h * dh + c];
                    }
                    float o = acc / den;
                    ai[c] = prec ? bf16_rne(o) : o;
                }
            }
        linear(att, L, d, w->wo, w->bo, d, y);
        for (int t = 0; t < L; ++t) {
            for (int i = 0; i < d; ++i) x[(int64_t)t * d + i] += prec ? bf16_rne(y[(int64_t)t * d + i]) : y[(int64_t)t * d + i];
            layer_norm(x + (int64_t)t * d, d, w->g1, w->b1n, e->ln_eps, prec);
        }
        linear(x, L, d, w->w1, w->b1, F, hid);
        for (int64_t i = 0; i < (int64_t)L * F; ++i) {
            float g = gelu_erf(hid[i]);
            hid[i] = prec ? bf16_rne(g) : g;
        }
        linear(hid, L, F, w->w2, w->b2, d, y);
        for (int t = 0; t < L; ++t) {
            for (int i = 0; i < d; ++i) x[(int64_t)t * d + i] += prec ? bf16_rne(y[(int64_t)t * d + i]) : y[(int64_t)t * d + i];
            layer_norm(x + (int64_t)t * d, d, w->g2, w->b2n, e->ln_eps, prec);
        }
    }
    /* masked mean pool over the L valid tokens, then L2 normalise */
    float nrm = 0.f;
    for (int i = 0; i < d; ++i) {
        float s = 0.f;
        for (int t = 0; t < L; ++t) s += x[(int64_t)t * d + i];
        out[i] = s / (float)L;
        nrm += out[i] * out[i];
    }
    nrm = sqrtf(nrm);
    if (nrm < 1e-12f) nrm = 1e-12f;
    for (int i = 0; i < d; ++i) out[i] /= nrm;
    free(x); free(qkv); free(att); free(y); free(hid); free(p);
    return ORC_OK;
}

/*
 * Embed chunks ids[0..n_ids) (ids == NULL: chunks 0..n_ids-1) of a token
 * store tokens[n_chunks][seq] with valid lengths lengths[n_chunks].
 * out[n_ids][d].  precision: 0 = fp32, 1 = bf16-storage emulation.
 */
int orc_embed(const orc_encoder_desc *e, const float *weights, const int32_t *tokens, const int32_t *lengths,
              int64_t n_chunks, int32_t seq, const int64_t *ids, int64_t n_ids, int32_t precision, float *out)
{
    if (!e || !weights || !tokens || !lengths || !out || n_ids < 0) return ORC_EINVAL;
    if (e->hidden <= 0 || e->heads <= 0 || e->hidden % e->heads || e->layers < 0 || seq > e->max_pos)
        return ORC_EINVAL;
    for (int64_t r = 0; r < n_ids; ++r) {
        int64_t c = ids ? ids[r] : r;
        if (c < 0 || c >= n_chunks) return ORC_EINVAL;
        if (lengths[c] < 1 || lengths[c] > seq) return ORC_EINVAL;
        for (int t = 0; t < lengths[c]; ++t) {
            int32_t tk = tokens[c * seq + t];
            if (tk < 0 || tk >= e->vocab) return ORC_EINVAL;
        }
    }
    float *wr = NULL;
    if (precision) { /* matrices and embedding tables to bf16; biases and LN parameters stay fp32 */
        int64_t cnt = orc_weight_count(e), d = e->hidden, F = e->ffn;
        wr = malloc(sizeof(float) * (size_t)cnt);
        if (!wr) return ORC_ENOMEM;
        memcpy(wr, weights, sizeof(float) * (size_t)cnt);
        float *q = wr;
        int64_t nemb = ((int64_t)e->vocab + e->max_pos + 1) * d;
        for (int64_t i = 0; i < nemb; ++i) q[i] = bf16_rne(q[i]);
        q += nemb + 2 * d;
        for (int l = 0; l < e->layers; ++l) {
            for (int64_t i = 0; i < 3 * d * d; ++i) q[i] = bf16_rne(q[i]);
            q += 3 * d * d + 3 * d;
            for (int64_t i = 0; i < d * d; ++i) q[i] = bf16_rne(q[i]);
            q += d * d + d + 2 * d;
            for (int64_t i = 0; i < F * d; ++i) q[i] = bf16_rne(q[i]);
            q += F * d + F;
            for (int64_t i = 0; i < d * F; ++i) q[i] = bf16_rne(q[i]);
            q += d * F + d + 2 * d;
        }
        weights = wr;
    }
    emb_w ew;
    layer_w *lw = malloc(sizeof(layer_w) * (size_t)(e->layers > 0 ? e->layers : 1));
    if (!lw) { free(wr); return ORC_ENOMEM; }
    split_weights(e, weights, &ew, lw);
    int rc = ORC_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_ids; ++r) {
        int64_t c = ids ? ids[r] : r;
        int st = encode_chunk(e, &ew, lw, tokens + c * seq, lengths[c], precision, out + r * e->hidden);
        if (st != ORC_OK) {
#pragma omp critical
            rc = st;
        }
    }
    free(lw);
    free(wr);
    return rc;
}

/* ------------------------------------------------------------------ */
/* C2. product quantisation and ADC                                    */
/* ------------------------------------------------------------------ */

#define ORC_PQ_MAX_TRAIN 65536

static int nearest_centroid(const float *v, const float *cb, int ksub, int dsub, float *dist_out)
{
    int best = 0;
    float bd = INFINITY;
    for (int c = 0; c < ksub; ++c) {
        float s = 0.f;
        for (int j = 0; j < dsub; ++j) {
            float t = v[j] - cb[c * dsub + j];
            s += t * t;
        }
        if (s < bd) { /* strict: ties keep the lowest index */
            bd = s;
            best = c;
        }
    }
    if (dist_out) *dist_out = bd;
    return best;
}

/*
 * Lloyd k-means per subspace.  x[n][d]; codebook[m_sub][ksub][d/m_sub].
 * Training rows = first min(n, 65536) entries of the seeded permutation;
 * initial centroids = the first ksub of those rows (wrapping when n < ksub).
 * objective[iters] (nullable) receives the summed squared error measured at
 * each assignment step, over all subspaces.
 */
int orc_pq_train(const float *x, int64_t n, int32_t d, int32_t m_sub, int32_t ksub, int32_t iters, uint64_t seed,
                 float *codebook, double *objective)
{
    if (!x || !codebook || n < 1 || d < 1 || m_sub < 1 || d % m_sub || ksub < 1 || ksub > 256 || iters < 0)
        return ORC_EINVAL;
    int dsub = d / m_sub;
    int64_t *perm = malloc(sizeof(int64_t) * (size_t)n);
    if (!perm) return ORC_ENOMEM;
    orc_permutation(n, seed, perm);
    int64_t nt = n < ORC_PQ_MAX_TRAIN ? n : ORC_PQ_MAX_TRAIN;
    int32_t *assign = malloc(sizeof(int32_t) * (size_t)nt);
    double *sum = malloc(sizeof(double) * (size_t)ksub * dsub);
    int64_t *cnt = malloc(sizeof(int64_t) * (size_t)ksub);
    if (!assign || !sum || !cnt) { free(perm); free(assign); free(sum); free(cnt); return ORC_ENOMEM; }
    if (objective)
        for (int it = 0; it < iters; ++it) objective[it] = 0.0;
    for (int m = 0; m < m_sub; ++m) {
        float *cb = codebook + (int64_t)m * ksub * dsub;
        for (int c = 0; c < ksub; ++c)
            memcpy(cb + c * dsub, x + perm[c % nt] * d + m * dsub, sizeof(float) * dsub);
        for (int it = 0; it < iters; ++it) {
            double obj = 0.0;
            for (int64_t r = 0; r < nt; ++r) {
                float dist;
                assign[r] = nearest_centroid(x + perm[r] * d + m * dsub, cb, ksub, dsub, &dist);
                obj += dist;
            }
            if (objective) objective[it] += obj;
            memset(sum, 0, sizeof(double) * (size_t)ksub * dsub);
            memset(cnt, 0, sizeof(int64_t) * (size_t)ksub);
            for (int64_t r = 0; r < nt; ++r) {
                const float *v = x + perm[r] * d + m * dsub;
                for (int j = 0; j < dsub; ++j) sum[assign[r] * dsub + j] += v[j];
                cnt[assign[r]]++;
            }
            for (int c = 0; c < ksub; ++c)
                if (cnt[c] > 0) /* an empty cluster keeps its previous centroid */
                    for (int j = 0; j < dsub; ++j) cb[c * dsub + j] = (float)(sum[c * dsub + j] / (double)cnt[c]);
        }
    }
    free(perm); free(assign); free(sum); free(cnt);
    return ORC_OK;
}

/* codes[n][m_sub]: index of the nearest centroid per subspace. */
int orc_pq_encode(const float *x, int64_t n, int32_t d, int32_t m_sub, int32_t ksub, const float *codebook,
                  uint8_t *codes)
{
    if (!x || !codebook || !codes || d % m_sub || ksub < 1 || ksub > 256) return ORC_EINVAL;
    int dsub = d / m_sub;
#pragma omp parallel for
    for (int64_t r = 0; r < n; ++r)
        for (int m = 0; m < m_sub; ++m)
            codes[r * m_sub + m] = (uint8_t)nearest_centroid(x + r * d + m * dsub,
                                                             codebook + (int64_t)m * ksub * dsub, ksub, dsub, NULL);
    return ORC_OK;
}

/* out[n][d]: concatenation of the centroids the codes name. */
int orc_pq_decode(const uint8_t *codes, int64_t n, int32_t d, int32_t m_sub, int32_t ksub, const float *codebook,
                  float *out)
{
    if (!codes || !codebook || !out || d % m_sub) return ORC_EINVAL;
    int dsub = d / m_sub;
    for (int64_t r = 0; r < n; ++r)
        for (int m = 0; m < m_sub; ++m)
            memcpy(out + r * d + m * dsub, codebook + ((int64_t)m * ksub + codes[r * m_sub + m]) * dsub,
                   sizeof(float) * dsub);
    return ORC_OK;
}

/*
 * Asymmetric distance computation as product quantisation defines it: the squared Euclidean distance
 * between the un-quantised query and the quantised vector splits over the subspaces, so one table per query,
 *   lut[m][c] = -|q_m - codebook[m][c]|^2   (sub-vector summed in index order, then negated),
 * turns Dist(q, x~_v) of Alg. 2 into m_sub lookups.  The sign makes every score in this file "larger is closer";
 * Eq. 1 states the search in Euclidean distance, and for the unit-norm embeddings used here exact L2 and
 * exact inner-product rankings coincide.
 */
int orc_lut(const float *q, int32_t d, int32_t m_sub, int32_t ksub, const float *codebook, float *lut)
{
    if (!q || !codebook || !lut || d % m_sub) return ORC_EINVAL;
    int dsub = d / m_sub;
    for (int m = 0; m < m_sub; ++m)
        for (int c = 0; c < ksub; ++c) {
            float s = 0.f;
            for (int j = 0; j < dsub; ++j) {
                float t = q[m * dsub + j] - codebook[((int64_t)m * ksub + c) * dsub + j];
                s += t * t;
            }
            lut[m * ksub + c] = -s;
        }
    return ORC_OK;
}

/* ADC score of one code row: sum of table entries in order m = 0..m_sub-1 (= -|q - decode(code)|^2). */
static float adc_one(const float *lut, int ksub, const uint8_t *code, int m_sub)
{
    float s = 0.f;
    for (int m = 0; m < m_sub; ++m) s += lut[m * ksub + code[m]];
    return s;
}

/* out[i] = ADC score of node ids[i]; l1[i] (nullable) = sum of |terms|. */
int orc_adc(const float *lut, int32_t m_sub, int32_t ksub, const uint8_t *codes, const uint32_t *ids, int64_t n_ids,
            float *out, float *l1)
{
    if (!lut || !codes || !ids || !out) return ORC_EINVAL;
    for (int64_t i = 0; i < n_ids; ++i) {
        const uint8_t *code = codes + (int64_t)ids[i] * m_sub;
        out[i] = adc_one(lut, ksub, code, m_sub);
        if (l1) {
            float a = 0.f;
            for (int m = 0; m < m_sub; ++m) a += fabsf(lut[m * ksub + code[m]]);
            l1[i] = a;
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------ */
/* C3. search                                                          */
/* ------------------------------------------------------------------ */

/* total order used everywhere: higher score first, then lower id */
static int better(float sa, int64_t ia, float sb, int64_t ib) { return sa > sb || (sa == sb && ia < ib); }

/* Eq. 1 with inner-product similarity: exact top-k by linear scan. */
int orc_exact_topk(const float *q, const float *table, int64_t n, int32_t d, int32_t k, int64_t *out_ids,
                   float *out_scores)
{
    if (!q || !table || !out_ids || !out_scores || k < 1) return ORC_EINVAL;
    int cnt = 0;
    for (int64_t v = 0; v < n; ++v) {
        float s = 0.f;
        for (int i = 0; i < d; ++i) s += q[i] * table[v * d + i];
        int pos = cnt;
        while (pos > 0 && better(s, v, out_scores[pos - 1], out_ids[pos - 1])) --pos;
        if (pos >= k) continue;
        int last = cnt < k ? cnt : k - 1;
        for (int j = last; j > pos; --j) {
            out_scores[j] = out_scores[j - 1];
            out_ids[j] = out_ids[j - 1];
        }
        out_scores[pos] = s;
        out_ids[pos] = v;
        if (cnt < k) ++cnt;
    }
    for (int j = cnt; j < k; ++j) {
        out_ids[j] = -1;
        out_scores[j] = -INFINITY;
    }
    return ORC_OK;
}

typedef int (*orc_embed_fn)(void *user, const int64_t *ids, int64_t n, float *out);

typedef struct {
    int64_t hops, adc_candidates, recomputed, flushes;
} orc_search_stats;

typedef struct {
    float score;
    int64_t id;
    int visited;
} eq_entry;

typedef struct {
    float score;
    int64_t id;
} aq_entry;

/*
 * Two-level search (Algorithm 2) with the cross-hop batching of Sec. 4.2.
 *
 * Per hop: read the best unvisited entry u of the exact queue EQ and mark it
 * visited; ADC-score every neighbour of u not yet ADC-scored for this query
 * and push it into the approximate queue AQ; pop the r best entries of AQ
 * (AQ holds every ADC-scored node that has not been recomputed yet) into the
 * pending list P.  r = ceil(alpha * |new|) in fp32 arithmetic
 * (alpha_mode 0, default) or ceil(alpha * |AQ|) (alpha_mode 1, the other
 * reading of "top alpha% of AQ").  When |P| >= batch, or EQ has no unvisited
 * entry left, P is embedded as one batch, scored by inner product with q
 * and try-inserted into EQ in append order.  The loop ends when EQ has no
 * unvisited entry and P is empty.  The entry point is scored exactly first
 * and is never ADC-scored.
 *
 * log_ids/log_scores (nullable, capacity log_cap): every exactly scored
 * node in scoring order.  visit_order (nullable): the u of every hop.
 */
/*
 * Pending index updates that the output stage of a search takes into account
 * (App. B "Soft Deletion Strategy" and "Batched Add Operation"):
 *  - deleted[v] != 0: node v is soft-deleted.  It is still traversed (its
 *    adjacency list is untouched); the exact queue is filtered by the flag
 *    before the k best active entries are taken.
 *  - buf_emb[buf_n][d], buf_ids[buf_n]: embeddings of added chunks that are
 *    not inserted into the graph yet.  They are scanned exhaustively
 *    (<q, e>, the exact score of Eq. 1) and merged with the graph's result
 *    under the same order (score descending, id ascending).
 * Reading where the text is silent: a buffered id is not subject to the
 * delete flags (they cover graph nodes), and buffered entries never enter
 * the traversal.
 */
typedef struct {
    const uint8_t *deleted; /* [n] or NULL */
    const float *buf_emb;   /* [buf_n][d] or NULL */
    const int64_t *buf_ids; /* [buf_n] */
    int64_t buf_n;
} orc_updates;

static int search_core(const float *q, int32_t d, const uint64_t *row_ptr, const uint32_t *col_idx, int64_t n,
                       uint32_t entry, const float *codebook, const uint8_t *codes, int32_t m_sub, orc_embed_fn embed,
                       void *user, int32_t ef, int32_t k, float alpha, int32_t batch, int32_t alpha_mode,
                       const orc_updates *upd, int64_t *out_ids, float *out_scores, orc_search_stats *stats,
                       int64_t *log_ids, float *log_scores, int64_t log_cap, int64_t *log_n, int64_t *visit_order,
                       int64_t visit_cap, int64_t *visit_n);

int orc_search(const float *q, int32_t d, const uint64_t *row_ptr, const uint32_t *col_idx, int64_t n,
               uint32_t entry, const float *codebook, const uint8_t *codes, int32_t m_sub, orc_embed_fn embed,
               void *user, int32_t ef, int32_t k, float alpha, int32_t batch, int32_t alpha_mode,
               int64_t *out_ids, float *out_scores, orc_search_stats *stats, int64_t *log_ids, float *log_scores,
               int64_t log_cap, int64_t *log_n, int64_t *visit_order, int64_t visit_cap, int64_t *visit_n)
{
    return search_core(q, d, row_ptr, col_idx, n, entry, codebook, codes, m_sub, embed, user, ef, k, alpha, batch,
                       alpha_mode, NULL, out_ids, out_scores, stats, log_ids, log_scores, log_cap, log_n, visit_order,
                       visit_cap, visit_n);
}

static int search_core(const float *q, int32_t d, const uint64_t *row_ptr, const uint32_t *col_idx, int64_t n,
                       uint32_t entry, const float *codebook, const uint8_t *codes, int32_t m_sub, orc_embed_fn embed,
                       void *user, int32_t ef, int32_t k, float alpha, int32_t batch, int32_t alpha_mode,
                       const orc_updates *upd, int64_t *out_ids, float *out_scores, orc_search_stats *stats,
                       int64_t *log_ids, float *log_scores, int64_t log_cap, int64_t *log_n, int64_t *visit_order,
                       int64_t visit_cap, int64_t *visit_n)
{
    if (!q || !row_ptr || !col_idx || !codebook || !codes || !embed || !out_ids || !out_scores) return ORC_EINVAL;
    if (k < 1 || k > ef || !(alpha > 0.f) || alpha > 1.f || batch < 1 || d % m_sub || entry >= (uint64_t)n)
        return ORC_EINVAL;
    const int ksub = 256;
    float *lut = malloc(sizeof(float) * (size_t)m_sub * ksub);
    uint8_t *adc_seen = calloc((size_t)n, 1);
    eq_entry *eq = malloc(sizeof(eq_entry) * (size_t)ef);
    aq_entry *aq = malloc(sizeof(aq_entry) * (size_t)(n > 0 ? n : 1));
    int64_t *pend = malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    float *emb = malloc(sizeof(float) * (size_t)(n > 0 ? n : 1) * d);
    if (!lut || !adc_seen || !eq || !aq || !pend || !emb) {
        free(lut); free(adc_seen); free(eq); free(aq); free(pend); free(emb);
        return ORC_ENOMEM;
    }
    orc_lut(q, d, m_sub, ksub, codebook, lut);
    int64_t n_eq = 0, n_aq = 0, n_pend = 0, nlog = 0, nvisit = 0;
    orc_search_stats st = {0, 0, 0, 0};
    int rc = ORC_OK;

    adc_seen[entry] = 1;
    pend[n_pend++] = entry; /* the entry point's exact score is the first flush */
    for (;;) {
        int64_t u_pos = -1;
        for (int64_t i = 0; i < n_eq; ++i)
            if (!eq[i].visited && (u_pos < 0 || better(eq[i].score, eq[i].id, eq[u_pos].score, eq[u_pos].id)))
                u_pos = i;
        if (u_pos >= 0) {
            int64_t u = eq[u_pos].id;
            eq[u_pos].visited = 1;
            st.hops++;
            if (visit_order && nvisit < visit_cap) visit_order[nvisit] = u;
            nvisit++;
            int64_t n_new = 0;
            for (uint64_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) {
                uint32_t v = col_idx[e];
                if (v >= (uint64_t)n) { rc = ORC_EINVAL; goto done; }
                if (adc_seen[v]) continue;
                adc_seen[v] = 1;
                aq[n_aq].score = adc_one(lut, ksub, codes + (int64_t)v * m_sub, m_sub);
                aq[n_aq].id = v;
                n_aq++;
                n_new++;
            }
            st.adc_candidates += n_new;
            int64_t r = (int64_t)ceilf(alpha * (float)(alpha_mode ? n_aq : n_new));
            for (int64_t t = 0; t < r && n_aq > 0; ++t) {
                int64_t b = 0;
                for (int64_t i = 1; i < n_aq; ++i)
                    if (better(aq[i].score, aq[i].id, aq[b].score, aq[b].id)) b = i;
                pend[n_pend++] = aq[b].id;
                aq[b] = aq[--n_aq];
            }
        }
        int has_unvisited = 0;
        for (int64_t i = 0; i < n_eq; ++i)
            if (!eq[i].visited) has_unvisited = 1;
        if (n_pend >= batch || (!has_unvisited && n_pend > 0)) {
            int erc = embed(user, pend, n_pend, emb);
            if (erc != ORC_OK) { rc = erc; goto done; }
            st.flushes++;
            st.recomputed += n_pend;
            for (int64_t c = 0; c < n_pend; ++c) {
                float s = 0.f;
                for (int i = 0; i < d; ++i) s += q[i] * emb[c * d + i];
                if (log_ids && nlog < log_cap) {
                    log_ids[nlog] = pend[c];
                    log_scores[nlog] = s;
                }
                nlog++;
                if (n_eq < ef) {
                    eq[n_eq].score = s; eq[n_eq].id = pend[c]; eq[n_eq].visited = 0;
                    n_eq++;
                } else {
                    int64_t wpos = 0; /* the tail: worst entry under the total order */
                    for (int64_t i = 1; i < n_eq; ++i)
                        if (better(eq[wpos].score, eq[wpos].id, eq[i].score, eq[i].id)) wpos = i;
                    if (better(s, pend[c], eq[wpos].score, eq[wpos].id)) {
                        eq[wpos].score = s; eq[wpos].id = pend[c]; eq[wpos].visited = 0;
                    }
                }
            }
            n_pend = 0;
            has_unvisited = 0;
            for (int64_t i = 0; i < n_eq; ++i)
                if (!eq[i].visited) has_unvisited = 1;
        }
        if (!has_unvisited && n_pend == 0) break;
    }
    /* Output: the k best of EQ.  With pending updates: the k best of (EQ without
     * soft-deleted nodes) united with the exhaustively scored add buffer. */
    {
        const int64_t nb = (upd && upd->buf_emb) ? upd->buf_n : 0;
        float *bs = nb ? malloc(sizeof(float) * (size_t)nb) : NULL;
        uint8_t *btaken = nb ? calloc((size_t)nb, 1) : NULL;
        if (nb && (!bs || !btaken)) { free(bs); free(btaken); rc = ORC_ENOMEM; goto done; }
        for (int64_t b = 0; b < nb; ++b) {
            float sc = 0.f;
            for (int i = 0; i < d; ++i) sc += q[i] * upd->buf_emb[b * d + i];
            bs[b] = sc;
        }
        if (upd && upd->deleted)
            for (int64_t i = 0; i < n_eq; ++i)
                if (upd->deleted[eq[i].id]) eq[i].visited = -1; /* filtered out */
        for (int j = 0; j < k; ++j) {
            int64_t b = -1, bb = -1;
            for (int64_t i = 0; i < n_eq; ++i)
                if (eq[i].visited >= 0 && (b < 0 || better(eq[i].score, eq[i].id, eq[b].score, eq[b].id))) b = i;
            for (int64_t i = 0; i < nb; ++i)
                if (!btaken[i] && (bb < 0 || better(bs[i], upd->buf_ids[i], bs[bb], upd->buf_ids[bb]))) bb = i;
            const int from_buf = bb >= 0 && (b < 0 || better(bs[bb], upd->buf_ids[bb], eq[b].score, eq[b].id));
            if (from_buf) {
                out_ids[j] = upd->buf_ids[bb];
                out_scores[j] = bs[bb];
                btaken[bb] = 1;
            } else if (b >= 0) {
                out_ids[j] = eq[b].id;
                out_scores[j] = eq[b].score;
                eq[b].visited = -1; /* taken */
            } else {
                out_ids[j] = -1;
                out_scores[j] = -INFINITY;
            }
        }
        free(bs); free(btaken);
    }
done:
    if (stats) *stats = st;
    if (log_n) *log_n = nlog;
    if (visit_n) *visit_n = nvisit;
    free(lut); free(adc_seen); free(eq); free(aq); free(pend); free(emb);
    return rc;
}

/* embedder: rows of a table of exact embeddings (table[n][d]) */
typedef struct {
    const float *table;
    int32_t d;
} table_user;

static int embed_from_table(void *user, const int64_t *ids, int64_t n, float *out)
{
    table_user *t = user;
    for (int64_t i = 0; i < n; ++i) memcpy(out + i * t->d, t->table + ids[i] * t->d, sizeof(float) * t->d);
    return ORC_OK;
}

/* embedder: run the encoder oracle on the token store */
typedef struct {
    const orc_encoder_desc *e;
    const float *w;
    const int32_t *tokens, *lengths;
    int64_t n_chunks;
    int32_t seq, precision;
} encoder_user;

static int embed_from_encoder(void *user, const int64_t *ids, int64_t n, float *out)
{
    encoder_user *u = user;
    return orc_embed(u->e, u->w, u->tokens, u->lengths, u->n_chunks, u->seq, ids, n, u->precision, out);
}

/* orc_search with embeddings looked up in a table the oracle computed earlier
 * (equal to recomputation because the encoder is batch-composition invariant). */
int orc_search_table(const float *q, int32_t d, const uint64_t *row_ptr, const uint32_t *col_idx, int64_t n,
                     uint32_t entry, const float *codebook, const uint8_t *codes, int32_t m_sub,
                     const float *table, int32_t ef, int32_t k, float alpha, int32_t batch, int32_t alpha_mode,
                     int64_t *out_ids, float *out_scores, orc_search_stats *stats, int64_t *log_ids,
                     float *log_scores, int64_t log_cap, int64_t *log_n, int64_t *visit_order, int64_t visit_cap,
                     int64_t *visit_n)
{
    table_user u = {table, d};
    return orc_search(q, d, row_ptr, col_idx, n, entry, codebook, codes, m_sub, embed_from_table, &u, ef, k, alpha,
                      batch, alpha_mode, out_ids, out_scores, stats, log_ids, log_scores, log_cap, log_n,
                      visit_order, visit_cap, visit_n);
}

/* orc_search_table with pending updates (soft-delete flags, add buffer). */
int orc_search_table_updates(const float *q, int32_t d, const uint64_t *row_ptr, const uint32_t *col_idx, int64_t n,
                             uint32_t entry, const float *codebook, const uint8_t *codes, int32_t m_sub,
                             const float *table, int32_t ef, int32_t k, float alpha, int32_t batch, int32_t alpha_mode,
                             const uint8_t *deleted, const float *buf_emb, const int64_t *buf_ids, int64_t buf_n,
                             int64_t *out_ids, float *out_scores, orc_search_stats *stats, int64_t *log_ids,
                             float *log_scores, int64_t log_cap, int64_t *log_n, int64_t *visit_order,
                             int64_t visit_cap, int64_t *visit_n)
{
    table_user u = {table, d};
    orc_updates upd = {deleted, buf_emb, buf_ids, buf_n};
    if (buf_n < 0 || (buf_n > 0 && (!buf_emb || !buf_ids))) return ORC_EINVAL;
    return search_core(q, d, row_ptr, col_idx, n, entry, codebook, codes, m_sub, embed_from_table, &u, ef, k, alpha,
                       batch, alpha_mode, &upd, out_ids, out_scores, stats, log_ids, log_scores, log_cap, log_n,
                       visit_order, visit_cap, visit_n);
}

/* orc_search with true recomputation: every flush runs the encoder oracle. */
int orc_search_encoder(const float *q, const uint64_t *row_ptr, const uint32_t *col_idx, int64_t n, uint32_t entry,
                       const float *codebook, const uint8_t *codes, int32_t m_sub, const orc_encoder_desc *e,
                       const float *weights, const int32_t *tokens, const int32_t *lengths, int32_t seq,
                       int32_t precision, int32_t ef, int32_t k, float alpha, int32_t batch, int32_t alpha_mode,
                       int64_t *out_ids, float *out_scores, orc_search_stats *stats)
{
    encoder_user u = {e, weights, tokens, lengths, n, seq, precision};
    return orc_search(q, e->hidden, row_ptr, col_idx, n, entry, codebook, codes, m_sub, embed_from_encoder, &u, ef,
                      k, alpha, batch, alpha_mode, out_ids, out_scores, stats, NULL, NULL, 0, NULL, NULL, 0, NULL);
}

/* ------------------------------------------------------------------ */
/* C4. graph construction (Algorithm 3 and the node-insertion listing   */
/*     of the update appendix)                                          */
/* ------------------------------------------------------------------ */

/*
 * The index graph is built by inserting the nodes one after the other
 * (Algorithm 3, "for v in V(G)").  For node v:
 *   W   <- Search(v, efC): Algorithm 1 on the graph built so far, exact
 *          similarities <e_v, e_x> from the stored embeddings (they exist while
 *          the index is built), queue length efC;
 *   R   <- Shrink(W, M0): walk W by ascending distance to v and keep x unless a
 *          kept y is closer to x than v is (the RNG rule of the appendix:
 *          Dist(x, y) < Dist(x, v)); stop at M0 kept.  M0 = M for the nodes
 *          flagged as high-degree, m for the others (Algorithm 3);
 *   add the edges v -> r and r -> v for r in R;
 *   a neighbour r whose list now exceeds M is shrunk to M with the same rule,
 *   anchored at r ("allow all nodes to form bidirectional links ... up to the
 *   higher threshold M").
 * Similarity = inner product of the (unit-norm) embeddings, so "closer" =
 * larger similarity; total order (similarity descending, id ascending).
 *
 * Readings where the text is silent:
 *  - insertion order = id order; the search of an insertion starts at node 0
 *    (the first node inserted);
 *  - a list that does not exceed its cap is kept as it is (no RNG pass);
 *  - batch > 1 is a batch-synchronous generalisation: the nodes of a batch
 *    search the graph as it was before the batch, then their edges are committed
 *    in id order and every neighbour that received edges is shrunk once, at the
 *    end of the batch.  Batch k holds min(batch, max(1, inserted / ramp)) nodes.
 *    batch = 1 is the listing itself.
 */

typedef struct {
    int32_t *adj; /* [n][cap] */
    int32_t *deg; /* [n] */
    int32_t cap;
} build_graph;

static float simf(const float *emb, int32_t d, int64_t a, int64_t b)
{
    float s = 0.f;
    for (int i = 0; i < d; ++i) s += emb[a * d + i] * emb[b * d + i];
    return s;
}

/* Shrink: ids[0..cnt) with similarities sim[] to the anchor; keeps at most cap, writes them (best first) to out. */
static int shrink_rng(const float *emb, int32_t d, const int32_t *ids, const float *sim, int cnt, int cap,
                      int32_t *out, uint8_t *taken /* scratch [cnt] */)
{
    int kept = 0;
    memset(taken, 0, (size_t)cnt);
    for (int step = 0; step < cnt && kept < cap; ++step) {
        int b = -1;
        for (int i = 0; i < cnt; ++i)
            if (!taken[i] && (b < 0 || better(sim[i], ids[i], sim[b], ids[b]))) b = i;
        taken[b] = 1;
        int ok = 1;
        for (int j = 0; j < kept && ok; ++j)
            if (simf(emb, d, ids[b], out[j]) > sim[b]) ok = 0; /* a kept node is closer to x than the anchor is */
        if (ok) out[kept++] = ids[b];
    }
    return kept;
}

/* Algorithm 1 on the build graph with exact similarities to node v; fills w_ids / w_sim (unsorted), returns count. */
static int build_search(const float *emb, int32_t d, const build_graph *g, int64_t n_inserted, int64_t v, int efC,
                        int32_t *w_ids, float *w_sim, uint8_t *w_vis, uint8_t *seen /* [n], zero on entry and exit */,
                        int32_t *touched)
{
    if (n_inserted == 0) return 0;
    int n_w = 0, n_touched = 0;
    w_ids[0] = 0; w_sim[0] = simf(emb, d, v, 0); w_vis[0] = 0; n_w = 1;
    seen[0] = 1; touched[n_touched++] = 0;
    for (;;) {
        int u = -1;
        for (int i = 0; i < n_w; ++i)
            if (!w_vis[i] && (u < 0 || better(w_sim[i], w_ids[i], w_sim[u], w_ids[u]))) u = i;
        if (u < 0) break;
        w_vis[u] = 1;
        const int32_t un = w_ids[u];
        for (int e = 0; e < g->deg[un]; ++e) {
            const int32_t x = g->adj[(int64_t)un * g->cap + e];
            if (seen[x]) continue;
            seen[x] = 1; touched[n_touched++] = x;
            const float s = simf(emb, d, v, x);
            if (n_w < efC) {
                w_ids[n_w] = x; w_sim[n_w] = s; w_vis[n_w] = 0; ++n_w;
            } else {
                int worst = 0;
                for (int i = 1; i < n_w; ++i)
                    if (better(w_sim[worst], w_ids[worst], w_sim[i], w_ids[i])) worst = i;
                if (better(s, x, w_sim[worst], w_ids[worst])) { w_ids[worst] = x; w_sim[worst] = s; w_vis[worst] = 0; }
            }
        }
    }
    for (int i = 0; i < n_touched; ++i) seen[touched[i]] = 0;
    return n_w;
}

/*
 * emb[n][d]; is_hub[n] (NULL: every node may keep M edges); out: CSR with
 * row_ptr[n+1] and col_idx (capacity n * M).  Returns the number of edges in
 * *n_edges.  searched_total (optional): sum of |W| over all insertions.
 */
int orc_build_graph(const float *emb, int64_t n, int32_t d, const uint8_t *is_hub, int32_t efC, int32_t M, int32_t m,
                    int32_t batch, int32_t ramp, uint64_t *row_ptr, uint32_t *col_idx, int64_t *n_edges,
                    int64_t *searched_total)
{
    if (!emb || !row_ptr || !col_idx || n < 1 || d < 1 || efC < 1 || M < 1 || m < 1 || m > M || batch < 1 || ramp < 1)
        return ORC_EINVAL;
    const int cap = M + batch; /* a list can grow by one edge per node of a batch before it is shrunk */
    build_graph g = {calloc((size_t)n * cap, sizeof(int32_t)), calloc((size_t)n, sizeof(int32_t)), cap};
    int32_t *fwd = malloc(sizeof(int32_t) * (size_t)batch * M);
    int32_t *fwd_n = malloc(sizeof(int32_t) * (size_t)batch);
    int32_t *w_ids = malloc(sizeof(int32_t) * (size_t)efC);
    float *w_sim = malloc(sizeof(float) * (size_t)efC);
    uint8_t *w_vis = malloc((size_t)efC);
    uint8_t *seen = calloc((size_t)n, 1);
    int32_t *touched = malloc(sizeof(int32_t) * (size_t)n);
    uint8_t *got = calloc((size_t)n, 1);
    const int tmp_n = (cap > efC ? cap : efC) + 1;
    int32_t *tmp_ids = malloc(sizeof(int32_t) * (size_t)tmp_n);
    float *tmp_sim = malloc(sizeof(float) * (size_t)tmp_n);
    uint8_t *taken = malloc((size_t)tmp_n);
    int rc = ORC_OK;
    int64_t searched = 0;
    if (!g.adj || !g.deg || !fwd || !fwd_n || !w_ids || !w_sim || !w_vis || !seen || !touched || !got || !tmp_ids ||
        !tmp_sim || !taken) {
        rc = ORC_ENOMEM;
        goto out;
    }
    for (int64_t s = 0; s < n;) {
        int64_t b = s / ramp;
        if (b < 1) b = 1;
        if (b > batch) b = batch;
        if (s + b > n) b = n - s;
        /* searches and neighbour selection on the graph as it is before the batch */
        for (int64_t i = 0; i < b; ++i) {
            const int64_t v = s + i;
            const int n_w = build_search(emb, d, &g, s, v, efC, w_ids, w_sim, w_vis, seen, touched);
            searched += n_w;
            const int cap_v = (!is_hub || is_hub[v]) ? M : m;
            fwd_n[i] = shrink_rng(emb, d, w_ids, w_sim, n_w, cap_v, fwd + i * M, taken);
        }
        /* commit in id order: forward lists, then reverse edges */
        for (int64_t i = 0; i < b; ++i) {
            const int64_t v = s + i;
            for (int j = 0; j < fwd_n[i]; ++j) g.adj[v * cap + j] = fwd[i * M + j];
            g.deg[v] = fwd_n[i];
        }
        for (int64_t i = 0; i < b; ++i) {
            const int64_t v = s + i;
            for (int j = 0; j < fwd_n[i]; ++j) {
                const int32_t r = fwd[i * M + j];
                g.adj[(int64_t)r * cap + g.deg[r]++] = (int32_t)v;
                got[r] = 1;
            }
        }
        /* neighbours that received edges: back under the cap M */
        for (int64_t i = 0; i < b; ++i)
            for (int j = 0; j < fwd_n[i]; ++j) {
                const int32_t r = fwd[i * M + j];
                if (!got[r]) continue;
                got[r] = 0;
                if (g.deg[r] <= M) continue;
                const int cnt = g.deg[r];
                for (int e = 0; e < cnt; ++e) {
                    tmp_ids[e] = g.adj[(int64_t)r * cap + e];
                    tmp_sim[e] = simf(emb, d, r, tmp_ids[e]);
                }
                g.deg[r] = shrink_rng(emb, d, tmp_ids, tmp_sim, cnt, M, g.adj + (int64_t)r * cap, taken);
            }
        s += b;
    }
    {
        int64_t e = 0;
        for (int64_t v = 0; v < n; ++v) {
            row_ptr[v] = (uint64_t)e;
            for (int j = 0; j < g.deg[v]; ++j) col_idx[e++] = (uint32_t)g.adj[v * cap + j];
        }
        row_ptr[n] = (uint64_t)e;
        if (n_edges) *n_edges = e;
    }
    if (searched_total) *searched_total = searched;
out:
    free(g.adj); free(g.deg); free(fwd); free(fwd_n); free(w_ids); free(w_sim); free(w_vis); free(seen); free(touched);
    free(got); free(tmp_ids); free(tmp_sim); free(taken);
    return rc;
}

/* Algorithm 3, "nodes with the top beta% highest degrees": the ceil(beta * n) nodes of largest out-degree in a CSR
 * graph, ties to the lower id.  is_hub[n] receives 0 / 1. */
int orc_top_degree(const uint64_t *row_ptr, int64_t n, double beta, uint8_t *is_hub)
{
    if (!row_ptr || !is_hub || n < 1 || !(beta >= 0.0) || beta > 1.0) return ORC_EINVAL;
    int64_t want = (int64_t)ceil(beta * (double)n);
    if (want > n) want = n;
    memset(is_hub, 0, (size_t)n);
    for (int64_t c = 0; c < want; ++c) { /* selection by repeated maximum: quadratic, plain */
        int64_t b = -1;
        for (int64_t v = 0; v < n; ++v) {
            if (is_hub[v]) continue;
            const int64_t dv = (int64_t)(row_ptr[v + 1] - row_ptr[v]);
            if (b < 0 || dv > (int64_t)(row_ptr[b + 1] - row_ptr[b])) b = v;
        }
        is_hub[b] = 1;
    }
    return ORC_OK;
}

/* Shrink alone (for its pins): candidates ids[cnt] around anchor node a of emb; out gets at most cap ids, best first. */
int orc_shrink(const float *emb, int64_t n, int32_t d, int64_t anchor, const int32_t *ids, int32_t cnt, int32_t cap,
               int32_t *out, int32_t *n_out)
{
    if (!emb || !ids || !out || !n_out || cnt < 0 || cap < 1 || anchor < 0 || anchor >= n) return ORC_EINVAL;
    float *sim = malloc(sizeof(float) * (size_t)(cnt + 1));
    uint8_t *taken = malloc((size_t)cnt + 1);
    if (!sim || !taken) { free(sim); free(taken); return ORC_ENOMEM; }
    for (int i = 0; i < cnt; ++i) sim[i] = simf(emb, d, anchor, ids[i]);
    *n_out = shrink_rng(emb, d, ids, sim, cnt, cap, out, taken);
    free(sim); free(taken);
    return ORC_OK;
}

// Internal declarations shared by the translation units of libleann (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/leann.h"

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

void leann_set_error(const char *fmt, ...);

#define LEANN_HIP(call)                                                                         \
    do {                                                                                        \
        hipError_t e_ = (call);                                                                 \
        if (e_ != hipSuccess) {                                                                 \
            leann_set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return e_ == hipErrorOutOfMemory ? LEANN_ENOMEM : LEANN_EDEVICE;                    \
        }                                                                                       \
    } while (0)

#define LEANN_TRY(call)              \
    do {                             \
        int rc_ = (call);            \
        if (rc_ != LEANN_OK) return rc_; \
    } while (0)

// Per-layer device pointers into the context's own copy of the weights.
struct LayerWeights {
    const bf16_t *wqkv, *wo, *w1, *w2;                          // [out][in] bf16
    const float *bqkv, *bo, *g1, *be1, *b1, *b2, *g2, *be2;     // fp32
};

// Growable device buffer owned by the context.
struct DevBuf {
    void *p = nullptr;
    size_t bytes = 0;
    int reserve(size_t need);
    void release();
};

struct leann_ctx {
    leann_encoder_desc desc;
    int device = 0;
    int num_cus = 256;
    int ln_blocks_per_cu = 4;
    hipStream_t stream = nullptr;
    // weights
    DevBuf w_bf16, w_f32;
    const bf16_t *tok_emb = nullptr, *pos_emb = nullptr, *seg_emb = nullptr;
    const float *emb_g = nullptr, *emb_b = nullptr;
    std::vector<LayerWeights> layers;
    // limits
    int64_t max_tokens = 1048576;  // padded tokens per encoder pass (workspaces: about 17 KB per token at BERT-base width)
    int32_t aq_capacity = 0;  // 0 = derive from ef and graph
    int32_t gemm_large_tile = 256;   // 256: 256x256 block tiles for large passes; 128: never (leann_set_gemm_tiles)
    int32_t gemm_small_rows = 2048;  // passes of at most this many padded rows use 64x64 tiles
    // encoder workspace
    DevBuf x, qkv, att, delta, hid, cu, len, meta, enc_ids;
    // search workspace
    DevBuf s_state, s_emb, s_lut, s_seen, s_misc, s_owner, s_buf, s_memo_slot, s_memo_emb;
    int64_t memo_rows = 0;  // rows of the per-call embedding memo (leann_set_call_memo), 0 = off
    // optional per-kernel timing (leann_profile_begin / leann_profile_end)
    bool prof_on = false;
    DevBuf prof_tokens;  // device int64: valid tokens sent through the encoder while profiling
    struct ProfSpan {
        int kind;
        hipEvent_t a, b;
    };
    std::vector<ProfSpan> prof_spans;
    std::vector<hipEvent_t> prof_pool;
};

// Brackets one kernel launch with HIP events on the context's stream when profiling is on.
struct ProfScope {
    leann_ctx *ctx;
    hipEvent_t b = nullptr;
    ProfScope(leann_ctx *c, int kind);
    ~ProfScope();
};

struct leann_pq {
    int64_t n = 0;
    int32_t d = 0, m_sub = 0;
    float *codebook = nullptr;    // device fp32 [m_sub][256][d/m_sub]
    uint8_t *codes = nullptr;     // device u8 [n][m_sub]
    bool owns_codes = true;
    int device = 0;
};

// Per-device set-up of each source file's kernels (LDS limits); called by leann_create with the device current.
int enc_init_device();
int enc_ln_blocks_per_cu(int *out);  // resident blocks of the LayerNorm kernel per CU on the current device
int pq_init_device();
int search_init_device();

// ---- encoder.hip
// Embeds the chunks named by ids_dev[0..n) (NULL: first_id .. first_id+n) into out[n][d] (fp32), in passes of at
// most ctx->max_tokens padded tokens.  err_dev: device int, set non-zero on invalid tokens / lengths / ids.
int enc_forward(leann_ctx *ctx, const leann_chunks *chunks, const int64_t *ids_dev, int64_t first_id, int64_t n,
                float *out_dev, int *err_dev, int64_t *tok_count_dev);

// ---- pq.hip
int pq_build_lut(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_pq *pq, float *lut_dev);

// ---- search.hip
int search_run(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_graph *graph, const leann_pq *pq,
               const leann_chunks *chunks, const leann_emb_cache *cache, const leann_updates *upd, int32_t ef, int32_t k, float alpha,
               int32_t batch, int64_t *out_ids_dev, float *out_scores_dev, leann_search_stats *stats);

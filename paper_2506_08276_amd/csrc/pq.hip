// Product quantisation: training, encoding, per-query lookup tables and the stand-alone ADC scorer
// (LEANN Sec. 3 offline stage: the PQ table kept in place of the embeddings; Alg. 2: the approximate distance that
// ranks new neighbours).  256 centroids per subspace.
#include <math.h>

#include <mutex>
#include <vector>

#include "common.h"

namespace {

constexpr int KSUB = 256;
constexpr int MAX_TRAIN = 65536;
constexpr int MAX_DSUB = 32;

// rows[i] of x (fp32 [n][d]) -> xt[i][d]
__global__ void gather_rows_kernel(const float *__restrict__ x, const int64_t *__restrict__ rows, int64_t nt, int d,
                                   float *__restrict__ xt)
{
    const int64_t i = blockIdx.x;
    if (i >= nt) return;
    const float *src = x + rows[i] * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) xt[i * d + c] = src[c];
}

// nearest centroid (squared L2, ties to the lowest index) of every row in subspace m = blockIdx.y.
// Writes int32 assign[m][r] (training) and/or u8 codes[r][m_sub] (encoding).
__global__ __launch_bounds__(256) void assign_kernel(const float *__restrict__ x, int64_t n, int d, int m_sub,
                                                     const float *__restrict__ codebook, int32_t *__restrict__ assign,
                                                     uint8_t *__restrict__ codes)
{
    extern __shared__ float cb[];  // [256][dsub]
    const int m = blockIdx.y, dsub = d / m_sub;
    for (int i = threadIdx.x; i < KSUB * dsub; i += 256) cb[i] = codebook[(size_t)m * KSUB * dsub + i];
    __syncthreads();
    const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (r >= n) return;
    float v[MAX_DSUB];
#pragma unroll
    for (int j = 0; j < MAX_DSUB; ++j) v[j] = j < dsub ? x[r * d + m * dsub + j] : 0.f;
    int best = 0;
    float bd = INFINITY;
    for (int c = 0; c < KSUB; ++c) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < MAX_DSUB; ++j)
            if (j < dsub) {
                float t = v[j] - cb[c * dsub + j];
                s += t * t;
            }
        if (s < bd) {
            bd = s;
            best = c;
        }
    }
    if (assign) assign[(size_t)m * n + r] = best;
    if (codes) codes[r * m_sub + m] = (uint8_t)best;
}

// centroid (c = blockIdx.x, m = blockIdx.y) <- mean of its training rows; fixed-order block reduction.
__global__ __launch_bounds__(256) void update_kernel(const float *__restrict__ xt, int64_t nt, int d, int m_sub,
                                                     const int32_t *__restrict__ assign, float *__restrict__ codebook)
{
    __shared__ float red[256];
    __shared__ int cnt[256];
    const int c = blockIdx.x, m = blockIdx.y, dsub = d / m_sub, tid = threadIdx.x;
    float acc[MAX_DSUB];
#pragma unroll
    for (int j = 0; j < MAX_DSUB; ++j) acc[j] = 0.f;
    int n_own = 0;
    const int32_t *as = assign + (size_t)m * nt;
    for (int64_t r = tid; r < nt; r += 256)
        if (as[r] == c) {
            ++n_own;
#pragma unroll
            for (int j = 0; j < MAX_DSUB; ++j)
                if (j < dsub) acc[j] += xt[r * d + m * dsub + j];
        }
    cnt[tid] = n_own;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if (tid < o) cnt[tid] += cnt[tid + o];
        __syncthreads();
    }
    const int total = cnt[0];
    if (total == 0) return;  // an empty cluster keeps its centroid
    for (int j = 0; j < dsub; ++j) {
        float mine = 0.f;
#pragma unroll
        for (int jj = 0; jj < MAX_DSUB; ++jj)
            if (jj == j) mine = acc[jj];
        __syncthreads();
        red[tid] = mine;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (tid < o) red[tid] += red[tid + o];
            __syncthreads();
        }
        if (tid == 0) codebook[((size_t)m * KSUB + c) * dsub + j] = red[0] / (float)total;
    }
}

// lut[q][m][c] = -|q_m - codebook[m][c]|^2 (PQ's asymmetric distance, negated so that larger is closer),
// sub-vector summed in index order.  grid (nq, m_sub), 256 threads.
__global__ __launch_bounds__(256) void lut_kernel(const float *__restrict__ queries, int d, int m_sub,
                                                  const float *__restrict__ codebook, float *__restrict__ lut)
{
    __shared__ float qs[MAX_DSUB];
    const int q = blockIdx.x, m = blockIdx.y, dsub = d / m_sub, c = threadIdx.x;
    if (c < dsub) qs[c] = queries[(size_t)q * d + m * dsub + c];
    __syncthreads();
    const float *cb = codebook + ((size_t)m * KSUB + c) * dsub;
    float s = 0.f;
    for (int j = 0; j < dsub; ++j) {
        const float t = qs[j] - cb[j];
        s += t * t;
    }
    lut[((size_t)q * m_sub + m) * KSUB + c] = -s;
}

// out[q][j] = sum_m lut[q][m][codes[cand[q][j]][m]], m ascending.  grid (nq, parts), 256 threads; the query's table
// sits in LDS and serves the block's whole share of the candidates (`per_block`, a multiple of 2048): the 32 KB table
// load is paid once per block, not once per 2048 candidates.  A thread owns 8 candidates per round: all their ids,
// then all their code rows are requested before the first lookup, so that the random row gathers overlap instead of
// queueing up; the ids of the next round are fetched while the current round's lookups run.
constexpr int ADC_PER_ROUND = 2048, ADC_PER_THREAD = ADC_PER_ROUND / 256;

__global__ __launch_bounds__(256) void adc_kernel(const float *__restrict__ lut, const uint8_t *__restrict__ codes,
                                                  int64_t n, int m_sub, const uint32_t *__restrict__ cand, int nc,
                                                  int per_block, float *__restrict__ out, int *__restrict__ err)
{
    extern __shared__ float tab[];  // [m_sub][256]
    const int q = blockIdx.x;
    const int beg = blockIdx.y * per_block, end = min(nc, beg + per_block);
    if (beg >= end) return;
    const uint32_t *cq = cand + (size_t)q * nc;
    float *oq = out + (size_t)q * nc;
    uint32_t v[ADC_PER_THREAD];
#pragma unroll
    for (int i = 0; i < ADC_PER_THREAD; ++i) {
        const int j = beg + threadIdx.x + i * 256;
        v[i] = j < end ? cq[j] : 0xffffffffu;
    }
    const float4 *src = reinterpret_cast<const float4 *>(lut + (size_t)q * m_sub * KSUB);
    for (int i = threadIdx.x; i < m_sub * KSUB / 4; i += 256) reinterpret_cast<float4 *>(tab)[i] = src[i];
    bool bad = false;
    if (m_sub == 32) {  // 32-byte rows: both halves of every row in flight before any lookup
        for (int j0 = beg + threadIdx.x; j0 < end + threadIdx.x; j0 += ADC_PER_ROUND) {
            u32x4 c0[ADC_PER_THREAD], c1[ADC_PER_THREAD];
            bool ok[ADC_PER_THREAD];
#pragma unroll
            for (int i = 0; i < ADC_PER_THREAD; ++i) {
                ok[i] = v[i] < n;
                const uint8_t *code = codes + (size_t)(ok[i] ? v[i] : 0) * 32;
                c0[i] = *reinterpret_cast<const u32x4 *>(code);  // plain loads: streaming ("nontemporal") ones are 15-35 % slower here
                c1[i] = *reinterpret_cast<const u32x4 *>(code + 16);
            }
#pragma unroll
            for (int i = 0; i < ADC_PER_THREAD; ++i) {  // ids of the next round
                const int j = j0 + ADC_PER_ROUND + i * 256;
                v[i] = j < end ? cq[j] : 0xffffffffu;
            }
            if (j0 < beg + ADC_PER_ROUND) __syncthreads();  // first round: the table is complete (uniform condition)
#pragma unroll
            for (int i = 0; i < ADC_PER_THREAD; ++i) {
                const int j = j0 + i * 256;
                if (j >= end) continue;
                float s = 0.f;  // subspace order; the compiler issues the lookups in runs ahead of the additions
#pragma unroll
                for (int m = 0; m < 16; ++m) s += tab[m * KSUB + ((c0[i][m >> 2] >> (8 * (m & 3))) & 255u)];
#pragma unroll
                for (int m = 0; m < 16; ++m) s += tab[(16 + m) * KSUB + ((c1[i][m >> 2] >> (8 * (m & 3))) & 255u)];
                if (!ok[i]) {
                    bad = true;
                    s = -INFINITY;
                }
                oq[j] = s;
            }
        }
        if (bad) atomicOr(err, 1);
        return;
    }
    __syncthreads();
    for (int j0 = beg + threadIdx.x; j0 < end + threadIdx.x; j0 += ADC_PER_ROUND) {
#pragma unroll
        for (int i = 0; i < ADC_PER_THREAD; ++i) {
            const int j = j0 + i * 256;
            if (j >= end) continue;
            const uint32_t id = cq[j];
            float s = -INFINITY;
            if (id < n) {
                const uint8_t *code = codes + (size_t)id * m_sub;
                s = 0.f;
                if ((m_sub & 15) == 0) {
                    for (int m0 = 0; m0 < m_sub; m0 += 16) {
                        const u32x4 w = *reinterpret_cast<const u32x4 *>(code + m0);
#pragma unroll
                        for (int m = 0; m < 16; ++m) s += tab[(m0 + m) * KSUB + ((w[m >> 2] >> (8 * (m & 3))) & 255u)];
                    }
                } else {
                    for (int m = 0; m < m_sub; ++m) s += tab[m * KSUB + code[m]];
                }
            } else {
                bad = true;
            }
            oq[j] = s;
        }
    }
    if (bad) atomicOr(err, 1);
}

// Launch shape of adc_kernel: enough blocks to fill the chip several times over, each with as large a share of its
// query's candidates as that allows.
void adc_launch_shape(int64_t nq, int nc, int *parts, int *per_block)
{
    const int rounds = (nc + ADC_PER_ROUND - 1) / ADC_PER_ROUND;
    const int64_t want_blocks = 256 * 64;  // blocks in the grid at least (when there is that much work): many short tails even out
    int64_t p = (want_blocks + nq - 1) / nq;
    if (p < 1) p = 1;
    if (p > rounds) p = rounds;
    const int rounds_per_block = (int)((rounds + p - 1) / p);
    *per_block = rounds_per_block * ADC_PER_ROUND;
    *parts = (rounds + rounds_per_block - 1) / rounds_per_block;
}

uint64_t splitmix64(uint64_t &st)
{
    uint64_t z = (st += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return z ^ (z >> 31);
}

int check_pq_shape(int64_t n, int32_t d, int32_t m_sub)
{
    if (n < 1 || d < 1 || m_sub < 1 || d % m_sub) {
        leann_set_error("PQ shape: n=%lld d=%d m_sub=%d (need d %% m_sub == 0)", (long long)n, d, m_sub);
        return LEANN_EINVAL;
    }
    if (d / m_sub > MAX_DSUB) {
        leann_set_error("PQ sub-vector length %d exceeds %d", d / m_sub, MAX_DSUB);
        return LEANN_ESHAPE;
    }
    return LEANN_OK;
}

int alloc_pq(leann_ctx *ctx, int64_t n, int32_t d, int32_t m_sub, bool own_codes, leann_pq **out)
{
    leann_pq *pq = new leann_pq();
    pq->n = n;
    pq->d = d;
    pq->m_sub = m_sub;
    pq->device = ctx->device;
    pq->owns_codes = own_codes;
    if (hipMalloc(&pq->codebook, (size_t)m_sub * KSUB * (d / m_sub) * sizeof(float)) != hipSuccess ||
        (own_codes && hipMalloc(&pq->codes, (size_t)n * m_sub) != hipSuccess)) {
        leann_set_error("device allocation for the PQ table failed");
        leann_pq_free(pq);
        return LEANN_ENOMEM;
    }
    *out = pq;
    return LEANN_OK;
}

// ---- workspace of leann_adc_noalloc: a fixed device array instead of a grown allocation.
// Layout: lookup tables fp32 [NOALLOC_MAX_QUERIES][m_sub][256] with m_sub * 256 * 4 <= NOALLOC_LUT_BYTES per query,
// then one 256-byte slot whose first int is the kernel's bad-id flag.  Every GPU the library runs on holds its own
// copy of the array until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; what kernels and copies get is the per-device address looked up below.
constexpr int NOALLOC_MAX_QUERIES = 128;
constexpr int NOALLOC_LUT_BYTES = 32 * KSUB * (int)sizeof(float);  // per query: up to 32 subspaces
constexpr size_t NOALLOC_FLAG_OFFSET = (size_t)NOALLOC_MAX_QUERIES * NOALLOC_LUT_BYTES;
static __device__ __align__(256) unsigned char scratch[NOALLOC_FLAG_OFFSET + 256];

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};  // device address of `scratch` on each device, 0 = not looked up yet

__global__ void clear_flag_kernel(int *flag) { *flag = 0; }

}  // namespace

int pq_init_device()
{
    LEANN_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(adc_kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
    // once per device, with that device current (leann_create made it so): where this device keeps `scratch`
    int dev = -1;
    LEANN_HIP(hipGetDevice(&dev));
    if (dev >= 0 && dev < NOALLOC_MAX_DEVICES) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void *ptr = nullptr;
            LEANN_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
            g_scratch_ptr[dev] = ptr;
        }
    }
    return LEANN_OK;
}

int pq_build_lut(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_pq *pq, float *lut_dev)
{
    if (nq <= 0) return LEANN_OK;
    ProfScope prof(ctx, LEANN_PROF_LUT);
    hipLaunchKernelGGL(lut_kernel, dim3((unsigned)nq, pq->m_sub), dim3(256), 0, ctx->stream, queries_dev, pq->d,
                       pq->m_sub, pq->codebook, lut_dev);
    LEANN_HIP(hipGetLastError());
    return LEANN_OK;
}

extern "C" {

int leann_build_pq(leann_ctx *ctx, const float *emb_dev, int64_t n, int32_t d, int32_t m_sub, int32_t iters,
                   uint64_t seed, leann_pq **out)
{
    if (!ctx || !emb_dev || !out || iters < 0) {
        leann_set_error("leann_build_pq: null argument or negative iteration count");
        return LEANN_EINVAL;
    }
    LEANN_TRY(check_pq_shape(n, d, m_sub));
    LEANN_HIP(hipSetDevice(ctx->device));
    const int dsub = d / m_sub;
    // seeded Fisher-Yates permutation; its prefix is the training sample, its first 256 rows the initial centroids
    std::vector<int64_t> perm((size_t)n);
    for (int64_t i = 0; i < n; ++i) perm[i] = i;
    uint64_t st = seed;
    for (int64_t i = n - 1; i >= 1; --i) {
        uint64_t j = splitmix64(st) % (uint64_t)(i + 1);
        std::swap(perm[i], perm[j]);
    }
    const int64_t nt = n < MAX_TRAIN ? n : MAX_TRAIN;
    leann_pq *pq = nullptr;
    LEANN_TRY(alloc_pq(ctx, n, d, m_sub, true, &pq));
    int64_t *rows_dev = nullptr;
    float *xt = nullptr;
    int32_t *assign = nullptr;
    int rc = LEANN_OK;
    auto fail = [&](int code) {
        (void)hipFree(rows_dev);
        (void)hipFree(xt);
        (void)hipFree(assign);
        leann_pq_free(pq);
        return code;
    };
    if (hipMalloc(&rows_dev, (size_t)nt * sizeof(int64_t)) != hipSuccess ||
        hipMalloc(&xt, (size_t)nt * d * sizeof(float)) != hipSuccess ||
        hipMalloc(&assign, (size_t)nt * m_sub * sizeof(int32_t)) != hipSuccess) {
        leann_set_error("device allocation for PQ training failed");
        return fail(LEANN_ENOMEM);
    }
    if (hipMemcpyAsync(rows_dev, perm.data(), (size_t)nt * sizeof(int64_t), hipMemcpyHostToDevice, ctx->stream) !=
        hipSuccess)
        return fail(LEANN_EDEVICE);
    hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)nt), dim3(256), 0, ctx->stream, emb_dev, rows_dev, nt, d, xt);
    // initial centroids: training rows 0..255 (wrapping when there are fewer rows)
    std::vector<float> head((size_t)std::min<int64_t>(nt, KSUB) * d);
    if (hipMemcpyAsync(head.data(), xt, head.size() * sizeof(float), hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
        hipStreamSynchronize(ctx->stream) != hipSuccess)
        return fail(LEANN_EDEVICE);
    std::vector<float> cb0((size_t)m_sub * KSUB * dsub);
    for (int m = 0; m < m_sub; ++m)
        for (int c = 0; c < KSUB; ++c)
            for (int j = 0; j < dsub; ++j)
                cb0[((size_t)m * KSUB + c) * dsub + j] = head[(size_t)(c % nt) * d + m * dsub + j];
    if (hipMemcpyAsync(pq->codebook, cb0.data(), cb0.size() * sizeof(float), hipMemcpyHostToDevice, ctx->stream) !=
        hipSuccess)
        return fail(LEANN_EDEVICE);
    const size_t smem = (size_t)KSUB * dsub * sizeof(float);
    for (int it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(assign_kernel, dim3((unsigned)((nt + 255) / 256), m_sub), dim3(256), smem, ctx->stream, xt, nt,
                           d, m_sub, pq->codebook, assign, (uint8_t *)nullptr);
        hipLaunchKernelGGL(update_kernel, dim3(KSUB, m_sub), dim3(256), 0, ctx->stream, xt, nt, d, m_sub, assign,
                           pq->codebook);
    }
    hipLaunchKernelGGL(assign_kernel, dim3((unsigned)((n + 255) / 256), m_sub), dim3(256), smem, ctx->stream, emb_dev, n,
                       d, m_sub, pq->codebook, (int32_t *)nullptr, pq->codes);
    if (hipGetLastError() != hipSuccess || hipStreamSynchronize(ctx->stream) != hipSuccess) {
        leann_set_error("PQ training kernels failed");
        return fail(LEANN_EDEVICE);
    }
    (void)hipFree(rows_dev);
    (void)hipFree(xt);
    (void)hipFree(assign);
    *out = pq;
    return rc;
}

int leann_pq_export(leann_ctx *ctx, const leann_pq *pq, float *codebook_host, uint8_t *codes_host)
{
    if (!ctx || !pq) {
        leann_set_error("leann_pq_export: null handle");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    LEANN_HIP(hipStreamSynchronize(ctx->stream));
    if (codebook_host)
        LEANN_HIP(hipMemcpy(codebook_host, pq->codebook, (size_t)pq->m_sub * KSUB * (pq->d / pq->m_sub) * sizeof(float),
                            hipMemcpyDeviceToHost));
    if (codes_host) LEANN_HIP(hipMemcpy(codes_host, pq->codes, (size_t)pq->n * pq->m_sub, hipMemcpyDeviceToHost));
    return LEANN_OK;
}

int leann_pq_import(leann_ctx *ctx, const float *codebook_host, const uint8_t *codes_host, int64_t n, int32_t d,
                    int32_t m_sub, leann_pq **out)
{
    if (!ctx || !codebook_host || !codes_host || !out) {
        leann_set_error("leann_pq_import: null argument");
        return LEANN_EINVAL;
    }
    LEANN_TRY(check_pq_shape(n, d, m_sub));
    LEANN_HIP(hipSetDevice(ctx->device));
    leann_pq *pq = nullptr;
    LEANN_TRY(alloc_pq(ctx, n, d, m_sub, true, &pq));
    if (hipMemcpy(pq->codebook, codebook_host, (size_t)m_sub * KSUB * (d / m_sub) * sizeof(float),
                  hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(pq->codes, codes_host, (size_t)n * m_sub, hipMemcpyHostToDevice) != hipSuccess) {
        leann_set_error("copying the PQ table to the device failed");
        leann_pq_free(pq);
        return LEANN_EDEVICE;
    }
    *out = pq;
    return LEANN_OK;
}

int leann_pq_wrap(leann_ctx *ctx, const float *codebook_host, const uint8_t *codes_dev, int64_t n, int32_t d,
                  int32_t m_sub, leann_pq **out)
{
    if (!ctx || !codebook_host || !codes_dev || !out) {
        leann_set_error("leann_pq_wrap: null argument");
        return LEANN_EINVAL;
    }
    LEANN_TRY(check_pq_shape(n, d, m_sub));
    LEANN_HIP(hipSetDevice(ctx->device));
    leann_pq *pq = nullptr;
    LEANN_TRY(alloc_pq(ctx, n, d, m_sub, false, &pq));
    pq->codes = const_cast<uint8_t *>(codes_dev);
    if (hipMemcpy(pq->codebook, codebook_host, (size_t)m_sub * KSUB * (d / m_sub) * sizeof(float),
                  hipMemcpyHostToDevice) != hipSuccess) {
        leann_set_error("copying the codebook to the device failed");
        leann_pq_free(pq);
        return LEANN_EDEVICE;
    }
    *out = pq;
    return LEANN_OK;
}

int leann_pq_info(const leann_pq *pq, int64_t *n, int32_t *d, int32_t *m_sub)
{
    if (!pq) {
        leann_set_error("leann_pq_info: null handle");
        return LEANN_EINVAL;
    }
    if (n) *n = pq->n;
    if (d) *d = pq->d;
    if (m_sub) *m_sub = pq->m_sub;
    return LEANN_OK;
}

void leann_pq_free(leann_pq *pq)
{
    if (!pq) return;
    (void)hipFree(pq->codebook);
    if (pq->owns_codes) (void)hipFree(pq->codes);
    delete pq;
}

int leann_adc(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_pq *pq, const uint32_t *cand_ids_dev,
              int32_t nc, float *out_dev)
{
    if (!ctx || !queries_dev || !pq || !cand_ids_dev || !out_dev || nq < 0 || nc < 0) {
        leann_set_error("leann_adc: null argument or negative count");
        return LEANN_EINVAL;
    }
    if (nq == 0 || nc == 0) return LEANN_OK;
    LEANN_HIP(hipSetDevice(ctx->device));
    const size_t lut_bytes = (size_t)nq * pq->m_sub * KSUB * sizeof(float);
    LEANN_TRY(ctx->s_lut.reserve(lut_bytes));
    LEANN_TRY(ctx->meta.reserve(256));
    int *err = (int *)ctx->meta.p;
    LEANN_HIP(hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
    LEANN_TRY(pq_build_lut(ctx, queries_dev, nq, pq, (float *)ctx->s_lut.p));
    const int smem = pq->m_sub * KSUB * (int)sizeof(float);
    if (smem > 96 * 1024) {
        leann_set_error("lookup table of %d bytes does not fit the ADC kernel's LDS budget", smem);
        return LEANN_ESHAPE;
    }
    {
        ProfScope prof(ctx, LEANN_PROF_ADC);
        int parts = 1, per_block = ADC_PER_ROUND;
        adc_launch_shape(nq, nc, &parts, &per_block);
        hipLaunchKernelGGL(adc_kernel, dim3((unsigned)nq, parts), dim3(256), smem, ctx->stream,
                           (const float *)ctx->s_lut.p, pq->codes, pq->n, pq->m_sub, cand_ids_dev, nc, per_block, out_dev,
                           err);
    }
    LEANN_HIP(hipGetLastError());
    int herr = 0;
    LEANN_HIP(hipMemcpyAsync(&herr, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    LEANN_HIP(hipStreamSynchronize(ctx->stream));
    if (herr) {
        leann_set_error("leann_adc: candidate id outside [0, n)");
        return LEANN_EINVAL;
    }
    return LEANN_OK;
}

int leann_adc_noalloc(leann_ctx *ctx, const float *queries_dev, int64_t nq, const leann_pq *pq,
                      const uint32_t *cand_ids_dev, int32_t nc, float *out_dev)
{
    if (!ctx || !queries_dev || !pq || !cand_ids_dev || !out_dev || nq < 0 || nc < 0) {
        leann_set_error("leann_adc_noalloc: null argument or negative count");
        return LEANN_EINVAL;
    }
    const int smem = pq->m_sub * KSUB * (int)sizeof(float);
    if (nq > NOALLOC_MAX_QUERIES || smem > NOALLOC_LUT_BYTES) {
        leann_set_error("leann_adc_noalloc: %lld queries x %d subspaces exceed the fixed workspace (at most %d queries, "
                        "%d subspaces); use leann_adc", (long long)nq, pq->m_sub, NOALLOC_MAX_QUERIES,
                        NOALLOC_LUT_BYTES / (KSUB * (int)sizeof(float)));
        return LEANN_ECAPACITY;
    }
    if (ctx->device < 0 || ctx->device >= NOALLOC_MAX_DEVICES || !g_scratch_ptr[ctx->device]) {
        leann_set_error("leann_adc_noalloc: no fixed workspace was set up for device %d", ctx->device);
        return LEANN_EDEVICE;
    }
    if (nq == 0 || nc == 0) return LEANN_OK;
    LEANN_HIP(hipSetDevice(ctx->device));
    unsigned char *base = static_cast<unsigned char *>(g_scratch_ptr[ctx->device]);
    float *lut = reinterpret_cast<float *>(base);
    int *flag = reinterpret_cast<int *>(base + NOALLOC_FLAG_OFFSET);
    // the array keeps the last call's contents: the flag starts at zero (a kernel, not a memset, so that the call
    // can be recorded into a graph); the tables are overwritten for exactly the queries that are read
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, ctx->stream, flag);
    hipLaunchKernelGGL(lut_kernel, dim3((unsigned)nq, pq->m_sub), dim3(256), 0, ctx->stream, queries_dev, pq->d,
                       pq->m_sub, pq->codebook, lut);
    int parts = 1, per_block = ADC_PER_ROUND;
    adc_launch_shape(nq, nc, &parts, &per_block);
    hipLaunchKernelGGL(adc_kernel, dim3((unsigned)nq, parts), dim3(256), smem, ctx->stream, (const float *)lut, pq->codes,
                       pq->n, pq->m_sub, cand_ids_dev, nc, per_block, out_dev, flag);
    LEANN_HIP(hipGetLastError());
    return LEANN_OK;
}

}  // extern "C"

// Graph construction by insertion (Algorithm 3 and the node-insertion listing of the update appendix) on the device.
//
// Nodes enter in id order, in batches: the nodes of a batch search the graph as it was before the batch (Algorithm 1
// with exact similarities from the stored embeddings), pick their neighbours with the RNG rule, then the forward and
// reverse edges of the batch are committed and every node that received edges is brought back under the degree cap M.
// With batch = 1 this is the sequential listing; larger batches are what fills the device (one wavefront per
// inserted node).  Batch k holds min(batch, max(1, inserted / ramp)) nodes, so the first nodes still go in one by one.
#include "common.h"

#include <algorithm>

namespace {

constexpr int EFC_MAX = 256;    // construction queue length
constexpr int M_MAX = 64;       // degree cap
constexpr int BATCH_MAX = 1024;  // nodes per batch
constexpr int LIST_MAX = M_MAX + BATCH_MAX;

struct BuildState {
    const float *emb;   // [n][d]
    int d;
    int32_t *adj;       // [n][stride]
    int32_t *deg;       // [n] current list length
    int32_t *deg0;      // [n] list length when the batch started
    int stride;         // M + batch
    uint16_t *stamp;    // [batch][n] visited marks of the searches: seen iff == epoch
    int64_t n;
    int32_t *fwd;       // [batch][M] neighbours chosen by the nodes of the batch
    int32_t *fwd_n;     // [batch]
    int32_t *touched;   // nodes that received reverse edges in this batch
    int32_t *n_touched;
    const uint8_t *is_hub;
    int M, m, efC;
};

__device__ inline bool better_i(float sa, int32_t ia, float sb, int32_t ib) { return sa > sb || (sa == sb && ia < ib); }

__device__ inline void wave_best_i(float &s, int32_t &id, int &pos)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float s2 = __shfl_xor(s, o, 64);
        const int32_t id2 = __shfl_xor(id, o, 64);
        const int p2 = __shfl_xor(pos, o, 64);
        if (p2 >= 0 && (pos < 0 || better_i(s2, id2, s, id))) {
            s = s2;
            id = id2;
            pos = p2;
        }
    }
}

// <emb[a], emb[b]> by one wavefront; every lane gets the result.  Lane l sums elements l, l + 64, ...
__device__ inline float wave_dot(const float *__restrict__ ea, const float *__restrict__ eb, int d, int lane)
{
    float acc = 0.f;
    for (int i = lane; i < d; i += 64) acc += ea[i] * eb[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    return acc;
}

// RNG selection among cand[0..cnt) (similarities sim[] to the anchor) into out[], at most cap: walk by (similarity
// desc, id asc); keep x unless a kept y is closer to x than the anchor is.  taken[] is scratch.  One wavefront; all
// arrays in LDS.  Returns the number kept (uniform).
__device__ inline int wave_shrink(const BuildState &s, const int32_t *cand, const float *sim, unsigned char *taken, int cnt,
                                  int cap, int32_t *out, int lane)
{
    for (int i = lane; i < cnt; i += 64) taken[i] = 0;
    __builtin_amdgcn_wave_barrier();
    int kept = 0;
    for (int step = 0; step < cnt && kept < cap; ++step) {
        float bs = -INFINITY;
        int32_t bid = 0x7fffffff;
        int bpos = -1;
        for (int i = lane; i < cnt; i += 64)
            if (!taken[i] && (bpos < 0 || better_i(sim[i], cand[i], bs, bid))) {
                bs = sim[i];
                bid = cand[i];
                bpos = i;
            }
        wave_best_i(bs, bid, bpos);
        if (lane == 0) taken[bpos] = 1;
        const float *ex = s.emb + (size_t)bid * s.d;
        bool ok = true;
        for (int j = 0; j < kept && ok; ++j)
            if (wave_dot(ex, s.emb + (size_t)out[j] * s.d, s.d, lane) > bs) ok = false;
        if (ok) {
            if (lane == 0) out[kept] = bid;
            ++kept;
        }
        __builtin_amdgcn_wave_barrier();
    }
    return kept;
}

// One wavefront per node of the batch: Search(v, efC) on the graph of the first `inserted` nodes, then Shrink(W, M0).
__global__ __launch_bounds__(64) void build_search_select_kernel(BuildState s, int64_t inserted, int epoch)
{
    __shared__ float w_sim[EFC_MAX];
    __shared__ int32_t w_id[EFC_MAX];
    __shared__ unsigned char w_vis[EFC_MAX];
    __shared__ unsigned char taken[EFC_MAX];
    __shared__ int32_t kept_ids[M_MAX];
    const int slot = blockIdx.x, lane = threadIdx.x;
    const int64_t v = inserted + slot;
    if (inserted == 0) {  // the first node has nothing to link to
        if (lane == 0) s.fwd_n[slot] = 0;
        return;
    }
    const float *ev = s.emb + (size_t)v * s.d;
    uint16_t *stamp = s.stamp + (size_t)slot * s.n;
    int n_w = 1;
    {
        const float s0 = wave_dot(ev, s.emb, s.d, lane);
        if (lane == 0) {
            w_sim[0] = s0;
            w_id[0] = 0;
            w_vis[0] = 0;
        }
    }
    __builtin_amdgcn_wave_barrier();
    for (;;) {
        float bs = -INFINITY;
        int32_t bid = 0x7fffffff;
        int bpos = -1;
        for (int i = lane; i < n_w; i += 64)
            if (!w_vis[i] && (bpos < 0 || better_i(w_sim[i], w_id[i], bs, bid))) {
                bs = w_sim[i];
                bid = w_id[i];
                bpos = i;
            }
        wave_best_i(bs, bid, bpos);
        if (bpos < 0) break;
        if (lane == 0) w_vis[bpos] = 1;
        const int du = s.deg[bid];  // <= M: lists are under the cap between batches
        const int32_t *nb = s.adj + (size_t)bid * s.stride;
        int32_t x = -1;
        if (lane < du) {
            x = nb[lane];
            if (x == 0 || stamp[x] == (uint16_t)epoch) x = -1;  // node 0 is the entry point: seen from the start
            else stamp[x] = (uint16_t)epoch;
        }
        unsigned long long todo = __ballot(x >= 0);
        while (todo) {
            const int src = __ffsll((long long)todo) - 1;
            todo &= todo - 1;
            const int32_t xi = __shfl(x, src, 64);
            const float sx = wave_dot(ev, s.emb + (size_t)xi * s.d, s.d, lane);
            if (n_w < s.efC) {
                if (lane == 0) {
                    w_sim[n_w] = sx;
                    w_id[n_w] = xi;
                    w_vis[n_w] = 0;
                }
                ++n_w;
            } else {  // replace the worst entry when the newcomer is better
                float ws = INFINITY;
                int32_t wid = -1;
                int wpos = -1;
                for (int i = lane; i < n_w; i += 64)
                    if (wpos < 0 || better_i(ws, wid, w_sim[i], w_id[i])) {
                        ws = w_sim[i];
                        wid = w_id[i];
                        wpos = i;
                    }
#pragma unroll
                for (int o = 32; o > 0; o >>= 1) {
                    const float s2 = __shfl_xor(ws, o, 64);
                    const int32_t id2 = __shfl_xor(wid, o, 64);
                    const int p2 = __shfl_xor(wpos, o, 64);
                    if (p2 >= 0 && (wpos < 0 || better_i(ws, wid, s2, id2))) {
                        ws = s2;
                        wid = id2;
                        wpos = p2;
                    }
                }
                if (better_i(sx, xi, ws, wid) && lane == 0) {
                    w_sim[wpos] = sx;
                    w_id[wpos] = xi;
                    w_vis[wpos] = 0;
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
    const int cap = (!s.is_hub || s.is_hub[v]) ? s.M : s.m;
    const int kept = wave_shrink(s, w_id, w_sim, taken, n_w, cap, kept_ids, lane);
    if (lane < kept) s.fwd[(size_t)slot * s.M + lane] = kept_ids[lane];
    if (lane == 0) s.fwd_n[slot] = kept;
}

// Forward lists of the batch's nodes, reverse edges appended to their targets (order fixed later), targets noted.
__global__ __launch_bounds__(64) void build_commit_kernel(BuildState s, int64_t inserted)
{
    const int slot = blockIdx.x, lane = threadIdx.x;
    const int64_t v = inserted + slot;
    const int cnt = s.fwd_n[slot];
    if (lane < cnt) {
        const int32_t r = s.fwd[(size_t)slot * s.M + lane];
        s.adj[(size_t)v * s.stride + lane] = r;
        const int pos = atomicAdd(&s.deg[r], 1);  // < deg0[r] + batch <= stride
        s.adj[(size_t)r * s.stride + pos] = (int32_t)v;
        if (pos == s.deg0[r]) s.touched[atomicAdd(s.n_touched, 1)] = r;
    }
    if (lane == 0) {
        s.deg[v] = cnt;
        s.deg0[v] = cnt;
    }
}

// One wavefront per node that received reverse edges: put the new edges in id order (the order of insertion), and if
// the list exceeds M shrink it with the RNG rule anchored at the node.
__global__ __launch_bounds__(64) void build_reverse_kernel(BuildState s)
{
    __shared__ int32_t list[LIST_MAX];
    __shared__ int32_t sorted[BATCH_MAX];
    __shared__ float sim[LIST_MAX];
    __shared__ unsigned char taken[LIST_MAX];
    __shared__ int32_t kept_ids[M_MAX];
    const int lane = threadIdx.x;
    if ((int)blockIdx.x >= *s.n_touched) return;
    const int32_t r = s.touched[blockIdx.x];
    const int cnt = s.deg[r], old = s.deg0[r];
    int32_t *row = s.adj + (size_t)r * s.stride;
    for (int i = lane; i < cnt; i += 64) list[i] = row[i];
    __builtin_amdgcn_wave_barrier();
    // rank sort of the appended ids (all different)
    const int na = cnt - old;
    for (int i = lane; i < na; i += 64) {
        const int32_t x = list[old + i];
        int rank = 0;
        for (int j = 0; j < na; ++j) rank += list[old + j] < x;
        sorted[rank] = x;
    }
    __builtin_amdgcn_wave_barrier();
    for (int i = lane; i < na; i += 64) list[old + i] = sorted[i];
    __builtin_amdgcn_wave_barrier();
    if (cnt <= s.M) {
        for (int i = lane; i < na; i += 64) row[old + i] = list[old + i];
        if (lane == 0) s.deg0[r] = cnt;
        return;
    }
    const float *er = s.emb + (size_t)r * s.d;
    for (int i = 0; i < cnt; ++i) {
        const float v = wave_dot(er, s.emb + (size_t)list[i] * s.d, s.d, lane);
        if (lane == 0) sim[i] = v;
    }
    __builtin_amdgcn_wave_barrier();
    const int kept = wave_shrink(s, list, sim, taken, cnt, s.M, kept_ids, lane);
    if (lane < kept) row[lane] = kept_ids[lane];
    if (lane == 0) {
        s.deg[r] = kept;
        s.deg0[r] = kept;
    }
}

// CSR out of the fixed-stride lists: one block; row_ptr by a chunked scan, then the copy.
__global__ __launch_bounds__(1024) void build_csr_kernel(BuildState s, uint64_t *__restrict__ row_ptr, uint32_t *__restrict__ col_idx)
{
    __shared__ unsigned long long part[1024];
    const int tid = threadIdx.x;
    const int64_t per = (s.n + 1023) / 1024;
    const int64_t beg = tid * per, end = beg + per < s.n ? beg + per : s.n;
    unsigned long long sum = 0;
    for (int64_t v = beg; v < end; ++v) sum += (unsigned long long)s.deg[v];
    part[tid] = sum;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const unsigned long long t = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += t;
        __syncthreads();
    }
    unsigned long long run = tid ? part[tid - 1] : 0;
    for (int64_t v = beg; v < end; ++v) {
        row_ptr[v] = run;
        const int dv = s.deg[v];
        for (int j = 0; j < dv; ++j) col_idx[run + j] = (uint32_t)s.adj[(size_t)v * s.stride + j];
        run += dv;
    }
    if (tid == 1023) row_ptr[s.n] = part[1023];
}

// Flags of the ceil(beta * n) nodes of largest out-degree, ties to the lower id.  One block: histogram of the degrees,
// the threshold degree, then the lowest ids at the threshold by a chunked count.
__global__ __launch_bounds__(1024) void top_degree_kernel(const uint64_t *__restrict__ row_ptr, int64_t n, int64_t want,
                                                          uint8_t *__restrict__ is_hub, int *__restrict__ err)
{
    constexpr int DMAX = 4096;
    __shared__ unsigned int hist[DMAX + 1];
    __shared__ unsigned long long part[1024];
    __shared__ int thr_s;
    __shared__ long long need_s;
    const int tid = threadIdx.x;
    for (int i = tid; i <= DMAX; i += 1024) hist[i] = 0;
    __syncthreads();
    const int64_t per = (n + 1023) / 1024;
    const int64_t beg = tid * per, end = beg + per < n ? beg + per : n;
    for (int64_t v = beg; v < end; ++v) {
        const unsigned long long dv = row_ptr[v + 1] - row_ptr[v];
        if (dv > DMAX) {
            atomicOr(err, 1);
            continue;
        }
        atomicAdd(&hist[dv], 1u);
    }
    __syncthreads();
    if (tid == 0) {
        long long left = want;
        int t = DMAX;
        while (t > 0 && left > (long long)hist[t]) left -= hist[t--];
        thr_s = t;         // degrees above t are all in; `left` of those at t (lowest ids)
        need_s = left;
    }
    __syncthreads();
    const int thr = thr_s;
    const long long need = need_s;
    unsigned long long at = 0;
    for (int64_t v = beg; v < end; ++v) at += (row_ptr[v + 1] - row_ptr[v]) == (unsigned long long)thr;
    part[tid] = at;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
        const unsigned long long t = tid >= o ? part[tid - o] : 0;
        __syncthreads();
        part[tid] += t;
        __syncthreads();
    }
    long long before = tid ? (long long)part[tid - 1] : 0;
    for (int64_t v = beg; v < end; ++v) {
        const unsigned long long dv = row_ptr[v + 1] - row_ptr[v];
        uint8_t flag = 0;
        if (dv <= DMAX) {
            if ((int)dv > thr) flag = 1;
            else if ((int)dv == thr) flag = before++ < need;
        }
        is_hub[v] = flag;
    }
}

}  // namespace

int leann_build_graph(leann_ctx *ctx, const float *emb_dev, int64_t n, int32_t d, const uint8_t *is_hub_dev, int32_t efC,
                      int32_t M, int32_t m, int32_t batch, int32_t ramp, uint64_t *row_ptr_dev, uint32_t *col_idx_dev,
                      int64_t *n_edges_host)
{
    if (!ctx || !emb_dev || !row_ptr_dev || !col_idx_dev || n < 1 || d < 1) {
        leann_set_error("leann_build_graph: null argument or empty input");
        return LEANN_EINVAL;
    }
    if (efC < 1 || efC > EFC_MAX || M < 1 || M > M_MAX || m < 1 || m > M || batch < 1 || batch > BATCH_MAX || ramp < 1 ||
        n > 0x7fffffffll) {
        leann_set_error("leann_build_graph: need 1 <= efC <= %d, 1 <= m <= M <= %d, 1 <= batch <= %d, ramp >= 1, n < 2^31",
                        EFC_MAX, M_MAX, BATCH_MAX);
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    hipStream_t st = ctx->stream;
    const int stride = M + batch;
    DevBuf adj, deg, stamp, misc;
    int rc = LEANN_OK;
    auto done = [&](int code) {
        (void)hipStreamSynchronize(st);
        adj.release();
        deg.release();
        stamp.release();
        misc.release();
        return code;
    };
    if ((rc = adj.reserve((size_t)n * stride * sizeof(int32_t))) != LEANN_OK) return done(rc);
    if ((rc = deg.reserve((size_t)n * 2 * sizeof(int32_t))) != LEANN_OK) return done(rc);
    if ((rc = stamp.reserve((size_t)batch * n * sizeof(uint16_t))) != LEANN_OK) return done(rc);
    const size_t fwd_bytes = (size_t)batch * M * sizeof(int32_t);
    if ((rc = misc.reserve(fwd_bytes + (size_t)batch * sizeof(int32_t) + (size_t)batch * M * sizeof(int32_t) + 256)) != LEANN_OK)
        return done(rc);
    BuildState s;
    s.emb = emb_dev;
    s.d = d;
    s.adj = (int32_t *)adj.p;
    s.deg = (int32_t *)deg.p;
    s.deg0 = s.deg + n;
    s.stride = stride;
    s.stamp = (uint16_t *)stamp.p;
    s.n = n;
    s.fwd = (int32_t *)misc.p;
    s.fwd_n = s.fwd + (size_t)batch * M;
    s.touched = s.fwd_n + batch;
    s.n_touched = s.touched + (size_t)batch * M;
    s.is_hub = is_hub_dev;
    s.M = M;
    s.m = m;
    s.efC = efC;
    hipError_t e = hipMemsetAsync(deg.p, 0, (size_t)n * 2 * sizeof(int32_t), st);
    if (e == hipSuccess) e = hipMemsetAsync(stamp.p, 0, (size_t)batch * n * sizeof(uint16_t), st);
    int epoch = 0;
    for (int64_t ins = 0; ins < n && e == hipSuccess;) {
        int64_t b = std::max<int64_t>(1, ins / ramp);
        b = std::min<int64_t>(std::min<int64_t>(b, batch), n - ins);
        if (++epoch == 65536) {  // the 16-bit marks wrap: start over with clean ones
            e = hipMemsetAsync(stamp.p, 0, (size_t)batch * n * sizeof(uint16_t), st);
            epoch = 1;
            if (e != hipSuccess) break;
        }
        e = hipMemsetAsync(s.n_touched, 0, sizeof(int32_t), st);
        if (e != hipSuccess) break;
        hipLaunchKernelGGL(build_search_select_kernel, dim3((unsigned)b), dim3(64), 0, st, s, ins, epoch);
        hipLaunchKernelGGL(build_commit_kernel, dim3((unsigned)b), dim3(64), 0, st, s, ins);
        hipLaunchKernelGGL(build_reverse_kernel, dim3((unsigned)(b * M)), dim3(64), 0, st, s);
        ins += b;
    }
    if (e == hipSuccess) {
        hipLaunchKernelGGL(build_csr_kernel, dim3(1), dim3(1024), 0, st, s, row_ptr_dev, col_idx_dev);
        e = hipGetLastError();
    }
    unsigned long long edges = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&edges, row_ptr_dev + n, sizeof(edges), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) {
        leann_set_error("leann_build_graph: %s", hipGetErrorString(e));
        return done(LEANN_EDEVICE);
    }
    if (n_edges_host) *n_edges_host = (int64_t)edges;
    return done(LEANN_OK);
}

int leann_top_degree(leann_ctx *ctx, const uint64_t *row_ptr_dev, int64_t n, double beta, uint8_t *is_hub_dev)
{
    if (!ctx || !row_ptr_dev || !is_hub_dev || n < 1 || !(beta >= 0.0) || beta > 1.0) {
        leann_set_error("leann_top_degree: null argument, empty graph or beta outside [0, 1]");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    LEANN_TRY(ctx->meta.reserve(256));
    int *err = (int *)ctx->meta.p;
    LEANN_HIP(hipMemsetAsync(err, 0, sizeof(int), ctx->stream));
    int64_t want = (int64_t)ceil(beta * (double)n);
    if (want > n) want = n;
    hipLaunchKernelGGL(top_degree_kernel, dim3(1), dim3(1024), 0, ctx->stream, row_ptr_dev, n, want, is_hub_dev, err);
    LEANN_HIP(hipGetLastError());
    int h_err = 0;
    LEANN_HIP(hipMemcpyAsync(&h_err, err, sizeof(int), hipMemcpyDeviceToHost, ctx->stream));
    LEANN_HIP(hipStreamSynchronize(ctx->stream));
    if (h_err) {
        leann_set_error("leann_top_degree: a node has more than 4096 neighbours");
        return LEANN_ECAPACITY;
    }
    return LEANN_OK;
}

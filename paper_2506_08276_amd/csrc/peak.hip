// Measured denominator for the encoder's roofline: what the matrix pipes of this GPU sustain on nothing but
// independent bf16 MFMA 32x32x16 instructions, for three kinds of operand bits.  The published 2.5 PFLOP/s assumes
// the 2.4 GHz peak clock; under matrix load the clock follows the power the operands' bit toggling draws, so the
// sustained rate depends on the data.  Benchmark hook only: nothing on the search path calls it.
#include "common.h"

namespace {

// operand words for lane-owned fragments: kind 0 zeros, 1 values near one (constant sign and exponent, few mantissa
// bits), 2 random sign, exponent in [2^-4, 2) and mantissa (the statistics of normalised activations and weights)
__global__ void peak_fill_kernel(uint16_t *out, int n, int kind)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint32_t x = (uint32_t)i * 2654435761u + 12345u;
    x ^= x >> 15;
    x *= 2246822519u;
    x ^= x >> 13;
    uint16_t v = 0;
    if (kind == 1) v = (uint16_t)(0x3f80 + (x & 3));
    if (kind == 2) v = (uint16_t)(((x >> 20 & 1) << 15) | ((123 + (x >> 8) % 5) << 7) | (x & 127));
    out[i] = v;
}

// Every wave holds 4 + 2 operand fragments and 8 accumulators of 32 x 32 (the GEMM's wave tile) and issues
// `iters` rounds of the 8 independent MFMAs.  The sum of the accumulators is written so that the work is live.
__global__ __launch_bounds__(256) void peak_mfma_kernel(const bf16x8 *__restrict__ in, f32x16 *__restrict__ out, int iters)
{
    bf16x8 a[4], b[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = in[threadIdx.x + 256 * i];
#pragma unroll
    for (int i = 0; i < 2; ++i) b[i] = in[threadIdx.x + 256 * (4 + i)];
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 2 + j], 0, 0, 0);
    }
    f32x16 s = acc[0];
#pragma unroll
    for (int i = 1; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] += acc[i][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// Ceiling of the ADC scorer's access pattern: nothing but gathers of uniformly random 32-byte rows (the two 16-byte
// halves of a row by one lane, eight rows in flight per lane), the loaded words folded into one value per thread so
// that the loads are live.  No lookup tables, no arithmetic: what the memory system delivers for this pattern.
__global__ __launch_bounds__(256) void peak_gather_kernel(const unsigned char *__restrict__ table,
                                                          const uint32_t *__restrict__ ids, int per_thread,
                                                          uint32_t *__restrict__ out)
{
    const size_t base = ((size_t)blockIdx.x * 256 + threadIdx.x) * per_thread;
    uint32_t acc = 0;
    for (int i0 = 0; i0 < per_thread; i0 += 8) {
        u32x4 a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const unsigned char *row = table + (size_t)ids[base + i0 + i] * 32;
            a[i] = *reinterpret_cast<const u32x4 *>(row);
            b[i] = *reinterpret_cast<const u32x4 *>(row + 16);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) acc ^= a[i][0] ^ a[i][3] ^ b[i][1] ^ b[i][2];
    }
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

__global__ void peak_ids_kernel(uint32_t *ids, size_t n, uint32_t rows)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        uint64_t x = (i + 1) * 0x9e3779b97f4a7c15ull;
        x ^= x >> 30;
        x *= 0xbf58476d1ce4e5b9ull;
        x ^= x >> 27;
        x *= 0x94d049bb133111ebull;
        x ^= x >> 31;
        ids[i] = (uint32_t)(x % rows);
    }
}

// Operand-feed ceiling of the GEMM: what a CU's vector L1 delivers when eight waves do nothing but the GEMM's operand
// loads.  A block of 512 threads walks the columns of a 256-row window of a panel of 1536-byte rows (K = 768 bf16) with
// 16-byte loads, four lanes per 64-byte row piece as in the GEMM, eight loads in flight per lane; the words are folded
// into one value per thread so that the loads are live.  A small panel stays in the XCDs' L2 (the windows of the blocks
// overlap), a large one comes from memory.
__global__ __launch_bounds__(512) void peak_pull_kernel(const unsigned char *__restrict__ panel, int rows, int iters,
                                                        uint32_t *__restrict__ out)
{
    constexpr int ROWB = 1536, PIECE = 64, LPR = PIECE / 16, RPI = 512 / LPR, AHEAD = 8;
    const int tid = threadIdx.x, r = tid / LPR, c = tid % LPR;
    const int row_base = (int)((blockIdx.x * 64u) % (unsigned)(rows - 256 - RPI));
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        u32x4 v[AHEAD];
#pragma unroll
        for (int j = 0; j < AHEAD; ++j) {
            const int step = it * AHEAD + j;
            const int col = (step % (ROWB / PIECE)) * PIECE;
            const int rr = row_base + ((step / (ROWB / PIECE)) * RPI + r) % 256;
            v[j] = *reinterpret_cast<const u32x4 *>(panel + (size_t)rr * ROWB + col + c * 16);
        }
#pragma unroll
        for (int j = 0; j < AHEAD; ++j) acc ^= v[j][0] ^ v[j][1] ^ v[j][2] ^ v[j][3];
    }
    out[(size_t)blockIdx.x * 512 + tid] = acc;
}

}  // namespace

extern "C" int leann_bench_l1pull(leann_ctx *ctx, int64_t panel_rows, int32_t launches, double *bytes_per_s_host,
                                  double *ms_host)
{
    if (!ctx || !bytes_per_s_host || panel_rows < 1024 || panel_rows > (1 << 22) || launches < 1 || launches > 1000) {
        leann_set_error("leann_bench_l1pull: null argument, panel rows outside 1024..2^22, or launch count outside 1..1000");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    const int grid = ctx->num_cus, iters = 2000;
    DevBuf panel, out;
    int rc = panel.reserve((size_t)panel_rows * 1536);
    if (rc == LEANN_OK) rc = out.reserve((size_t)grid * 512 * sizeof(uint32_t));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (rc == LEANN_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) {
        leann_set_error("leann_bench_l1pull: event creation failed");
        rc = LEANN_EDEVICE;
    }
    float ms = 0.f;
    if (rc == LEANN_OK) {
        hipStream_t st = ctx->stream;
        hipError_t e = hipMemsetAsync(panel.p, 1, (size_t)panel_rows * 1536, st);
        hipLaunchKernelGGL(peak_pull_kernel, dim3(grid), dim3(512), 0, st, (const unsigned char *)panel.p, (int)panel_rows,
                           iters, (uint32_t *)out.p);
        (void)hipEventRecord(e0, st);
        for (int l = 0; l < launches; ++l)
            hipLaunchKernelGGL(peak_pull_kernel, dim3(grid), dim3(512), 0, st, (const unsigned char *)panel.p,
                               (int)panel_rows, iters, (uint32_t *)out.p);
        (void)hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipGetLastError();
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) {
            leann_set_error("leann_bench_l1pull: %s", hipGetErrorString(e));
            rc = LEANN_EDEVICE;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    panel.release();
    out.release();
    if (rc != LEANN_OK) return rc;
    *bytes_per_s_host = (double)grid * 512 * 16.0 * iters * 8 * launches / (ms * 1e-3);
    if (ms_host) *ms_host = ms / launches;
    return LEANN_OK;
}

extern "C" int leann_bench_gather(leann_ctx *ctx, const uint8_t *table_dev, int64_t table_rows, int32_t launches,
                                  double *rows_per_s_host, double *ms_host)
{
    if (!ctx || !table_dev || !rows_per_s_host || table_rows < 1 || table_rows > 0xffffffffll || launches < 1 ||
        launches > 1000) {
        leann_set_error("leann_bench_gather: null argument, row count outside 1..2^32-1, or launch count outside 1..1000");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    const int per_thread = 64, grid = 4096;                     // 67 108 864 gathers per launch
    const size_t n_ids = (size_t)grid * 256 * per_thread;
    DevBuf ids, out;
    int rc = ids.reserve(n_ids * sizeof(uint32_t));
    if (rc == LEANN_OK) rc = out.reserve((size_t)grid * 256 * sizeof(uint32_t));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (rc == LEANN_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) {
        leann_set_error("leann_bench_gather: event creation failed");
        rc = LEANN_EDEVICE;
    }
    float ms = 0.f;
    if (rc == LEANN_OK) {
        hipStream_t st = ctx->stream;
        hipLaunchKernelGGL(peak_ids_kernel, dim3(4096), dim3(256), 0, st, (uint32_t *)ids.p, n_ids, (uint32_t)table_rows);
        hipLaunchKernelGGL(peak_gather_kernel, dim3(grid), dim3(256), 0, st, table_dev, (const uint32_t *)ids.p, per_thread,
                           (uint32_t *)out.p);
        (void)hipEventRecord(e0, st);
        for (int l = 0; l < launches; ++l)
            hipLaunchKernelGGL(peak_gather_kernel, dim3(grid), dim3(256), 0, st, table_dev, (const uint32_t *)ids.p,
                               per_thread, (uint32_t *)out.p);
        (void)hipEventRecord(e1, st);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) {
            leann_set_error("leann_bench_gather: %s", hipGetErrorString(e));
            rc = LEANN_EDEVICE;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    ids.release();
    out.release();
    if (rc != LEANN_OK) return rc;
    *rows_per_s_host = (double)n_ids * launches / (ms * 1e-3);
    if (ms_host) *ms_host = ms / launches;
    return LEANN_OK;
}

extern "C" int leann_bench_mfma(leann_ctx *ctx, int32_t operand_kind, int32_t blocks_per_cu, int32_t iters,
                                int32_t launches, double *tflops_host, double *ms_host)
{
    if (!ctx || !tflops_host || operand_kind < 0 || operand_kind > 2 || blocks_per_cu < 1 || blocks_per_cu > 2 ||
        iters < 1 || iters > (1 << 20) || launches < 1 || launches > 1000) {
        leann_set_error("leann_bench_mfma: null argument, operand kind outside 0..2, blocks per CU outside 1..2, or counts out of range");
        return LEANN_EINVAL;
    }
    LEANN_HIP(hipSetDevice(ctx->device));
    const int grid = ctx->num_cus * blocks_per_cu;
    const int n_in = 6 * 256 * 8;  // six fragments of eight bf16 per thread
    DevBuf in, out;
    int rc = in.reserve((size_t)n_in * sizeof(uint16_t));
    if (rc == LEANN_OK) rc = out.reserve((size_t)grid * 256 * sizeof(f32x16));
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (rc == LEANN_OK && (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)) {
        leann_set_error("leann_bench_mfma: event creation failed");
        rc = LEANN_EDEVICE;
    }
    float ms = 0.f;
    if (rc == LEANN_OK) {
        hipStream_t st = ctx->stream;
        hipLaunchKernelGGL(peak_fill_kernel, dim3((n_in + 255) / 256), dim3(256), 0, st, (uint16_t *)in.p, n_in, operand_kind);
        for (int l = 0; l < 3; ++l)  // warm-up: clocks settle under load
            hipLaunchKernelGGL(peak_mfma_kernel, dim3(grid), dim3(256), 0, st, (const bf16x8 *)in.p, (f32x16 *)out.p, iters);
        (void)hipEventRecord(e0, st);
        for (int l = 0; l < launches; ++l)
            hipLaunchKernelGGL(peak_mfma_kernel, dim3(grid), dim3(256), 0, st, (const bf16x8 *)in.p, (f32x16 *)out.p, iters);
        (void)hipEventRecord(e1, st);
        hipError_t e = hipGetLastError();
        if (e == hipSuccess) e = hipStreamSynchronize(st);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) {
            leann_set_error("leann_bench_mfma: %s", hipGetErrorString(e));
            rc = LEANN_EDEVICE;
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    in.release();
    out.release();
    if (rc != LEANN_OK) return rc;
    // 4 waves per block, 8 MFMAs of 2 * 32 * 32 * 16 flops per round
    const double flops = (double)grid * 4.0 * iters * 8.0 * 32768.0 * launches;
    *tflops_host = flops / (ms * 1e-3) / 1e12;
    if (ms_host) *ms_host = ms / launches;
    return LEANN_OK;
}

// Training-side steps around the convolution path: pattern pool generation (Section 4.2), adaptive
// finalisation counters (Section 4.3) and the gradient of the modified group-lasso penalty (Section 4.4,
// Eq. 3 and Eq. 4). All are one pass over [F][C][9] float32 tensors: bound by HBM traffic.
//
// Results that are integers (masks, counts, picks) come from float32 arithmetic in a fixed order without
// fused multiply-add (this file is compiled with -ffp-contract=off) and from integer atomics only.
#include "pc_internal.h"

#include <algorithm>
#include <vector>

#define TS_BLOCK 256

// 9 floats of TS_BLOCK consecutive kernels from global memory to LDS with contiguous loads.
__device__ __forceinline__ void ts_stage(float *dst, const float *__restrict__ src, int n)
{
    // all loads first (index clamped, so they are unconditional), then the LDS writes: one memory round trip
    float r[9];
#pragma unroll
    for (int j = 0; j < 9; ++j) {
        const int i = j * TS_BLOCK + threadIdx.x;
        r[j] = src[i < n * 9 ? i : n * 9 - 1];
    }
#pragma unroll
    for (int j = 0; j < 9; ++j) {
        const int i = j * TS_BLOCK + threadIdx.x;
        if (i < n * 9) dst[i] = r[j];
    }
}

// ------------------------------------------------------------------ pool generation, steps 1-4
// Neighbour sets of the 9 positions as bit masks: with diagonals (step 2) and without (step 3).
__device__ __forceinline__ unsigned ts_neighbours(int t, bool diagonal)
{
    const int r = t / 3, s = t - 3 * r;
    unsigned m = 0;
#pragma unroll
    for (int u = 0; u < 9; ++u) {
        const int dr = u / 3 - r, ds = u % 3 - s;
        const int ar = dr < 0 ? -dr : dr, as = ds < 0 ? -ds : ds;
        const bool adj = u != t && ar <= 1 && as <= 1 && (diagonal || ar + as == 1);
        m |= adj ? (1u << u) : 0u;
    }
    return m;
}

// One chunk of TS_BLOCK kernels starting at k0: candidate pattern of every kernel, counted in the LDS histogram lh.
__device__ __forceinline__ void ts_dppg_chunk(const float *__restrict__ W, const float *__restrict__ G, int64_t nk, int64_t k0,
                                              uint32_t *lh, uint16_t *__restrict__ masks, float *sw, float *sg)
{
    const int n = nk - k0 < TS_BLOCK ? (int)(nk - k0) : TS_BLOCK;
    ts_stage(sw, W + k0 * 9, n);
    if (G) ts_stage(sg, G + k0 * 9, n);
    __syncthreads();
    if (threadIdx.x < n) {
        float s[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const float w = sw[threadIdx.x * 9 + t];
            if (G) {
                const float gw = sg[threadIdx.x * 9 + t] * w;
                s[t] = gw * gw;
            } else {
                s[t] = w * w;
            }
        }
        // step 1: first maximum over the 9 positions (every update below is a select: no divergent branches)
        int t1 = 0;
        float b1 = s[0];
#pragma unroll
        for (int t = 1; t < 9; ++t) {
            const bool up = s[t] > b1;
            b1 = up ? s[t] : b1;
            t1 = up ? t : t1;
        }
        // step 2: first maximum over the neighbours of t1, diagonals included
        const unsigned n8 = ts_neighbours(t1, true);
        int t2 = -1;
        float b2 = 0.0f;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const bool up = (((n8 >> t) & 1u) != 0u) & ((t2 < 0) | (s[t] > b2));
            b2 = up ? s[t] : b2;
            t2 = up ? t : t2;
        }
        // step 3: candidate positions, diagonals excluded
        const unsigned base = (1u << t1) | (1u << t2);
        const unsigned cand = (ts_neighbours(t1, false) | ts_neighbours(t2, false)) & ~base;
        // step 4: best pair of candidates. The importances are squares (never below +0), so adding +0 for a
        // position outside the pattern changes no bit and the 9 additions equal ((s_a+s_b)+s_c)+s_d, taps ascending.
        // sb[t] is the term of position t when it is neither a nor b: s[t] for the two first positions, else +0.
        float sb[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) sb[t] = ((base >> t) & 1u) ? s[t] : 0.0f;
        unsigned best_m = 0u;
        float best = 0.0f;
#pragma unroll
        for (int a = 0; a < 9; ++a)
#pragma unroll
            for (int b = a + 1; b < 9; ++b) {
                float acc = 0.0f;
#pragma unroll
                for (int t = 0; t < 9; ++t) acc = acc + ((t == a || t == b) ? s[t] : sb[t]);
                const unsigned pair = (1u << a) | (1u << b);
                const bool take = ((cand & pair) == pair) & ((best_m == 0u) | (acc > best));
                best = take ? acc : best;
                best_m = take ? (base | pair) : best_m;
            }
        atomicAdd(&lh[best_m], 1u);
        if (masks) masks[k0 + threadIdx.x] = (uint16_t)best_m;
    }
    __syncthreads();                                // the staging buffers are free again; lh is complete after the last chunk
}

__global__ void __launch_bounds__(TS_BLOCK)
pc_dppg_kernel(const float *__restrict__ W, const float *__restrict__ G, int64_t nk, uint32_t *__restrict__ hist,
               uint16_t *__restrict__ masks)
{
    // A workgroup walks chunks of TS_BLOCK kernels with the grid as stride and counts in LDS; it adds its counts
    // to the pool once, at the end (few workgroups: little contention on the pool's 44 live counters).
    __shared__ float sw[TS_BLOCK * 9], sg[TS_BLOCK * 9];
    __shared__ uint32_t lh[512];
    lh[threadIdx.x] = 0u;
    lh[threadIdx.x + 256] = 0u;
    for (int64_t k0 = (int64_t)blockIdx.x * TS_BLOCK; k0 < nk; k0 += (int64_t)gridDim.x * TS_BLOCK)
        ts_dppg_chunk(W, G, nk, k0, lh, masks, sw, sg);
    for (int i = threadIdx.x; i < 512; i += TS_BLOCK)
        if (lh[i]) atomicAdd(&hist[i], lh[i]);      // integer counts: the order of the additions does not matter
}

// The layers of a network in one launch: chunk ch belongs to the layer l with blk0[l] <= ch < blk0[l + 1].
struct TsBatchArg {
    int32_t n;
    int32_t blk0[PC_BATCH_MAX + 1];
    int64_t nk[PC_BATCH_MAX];
    const float *W[PC_BATCH_MAX], *G[PC_BATCH_MAX];
    const uint8_t *pid[PC_BATCH_MAX], *keep[PC_BATCH_MAX];
    void *out[PC_BATCH_MAX];          // masks (pool generation), counts, picked ids or dW, by kernel
    const uint32_t *counts[PC_BATCH_MAX];
};

__global__ void __launch_bounds__(TS_BLOCK) pc_dppg_batch_kernel(TsBatchArg b, uint32_t *__restrict__ hist)
{
    __shared__ float sw[TS_BLOCK * 9], sg[TS_BLOCK * 9];
    __shared__ uint32_t lh[512];
    lh[threadIdx.x] = 0u;
    lh[threadIdx.x + 256] = 0u;
    const int total = b.blk0[b.n];
    for (int ch = (int)blockIdx.x; ch < total; ch += (int)gridDim.x) {
        const int l = pc_batch_find(b.blk0, b.n, ch);
        ts_dppg_chunk(b.W[l], b.G[l], b.nk[l], (int64_t)(ch - b.blk0[l]) * TS_BLOCK, lh, static_cast<uint16_t *>(b.out[l]), sw, sg);
    }
    for (int i = threadIdx.x; i < 512; i += TS_BLOCK)
        if (lh[i]) atomicAdd(&hist[i], lh[i]);
}

extern "C" pc_status pc_dppg_accumulate(pc_ctx *ctx, const float *W, const float *G, int32_t F, int32_t C,
                                        uint32_t *hist, uint16_t *masks)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!W || !hist) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_dppg_accumulate: null pointer");
    if (F < 1 || C < 1 || F > 65535 || C > 65535)
        return pc_fail(ctx, PC_ERR_BAD_SHAPE, "pc_dppg_accumulate: F=%d C=%d out of range", F, C);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    const int64_t nk = (int64_t)F * C;
    int64_t nb = (nk + TS_BLOCK - 1) / TS_BLOCK;
    if (nb > 2 * (int64_t)ctx->num_cu) nb = 2 * (int64_t)ctx->num_cu;
    hipLaunchKernelGGL(pc_dppg_kernel, dim3((unsigned)nb), dim3(TS_BLOCK), 0, ctx->stream, W, G, nk, hist, masks);
    return pc_hip_check(ctx, hipGetLastError(), "pool generation launch");
}

extern "C" pc_status pc_dppg_pool(pc_ctx *ctx, const uint32_t *hist, int32_t n_patterns, uint16_t *lib_host,
                                  uint32_t *score_host, int32_t *n_found)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!hist || !lib_host || !n_found) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_dppg_pool: null pointer");
    if (n_patterns < 1 || n_patterns > PC_MAX_P)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_dppg_pool: n_patterns=%d outside 1..%d", n_patterns, PC_MAX_P);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    std::vector<uint32_t> h(512);
    PC_HIP(ctx, hipMemcpyAsync(h.data(), hist, 512 * sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    PC_HIP(ctx, hipStreamSynchronize(ctx->stream));
    std::vector<int> order;
    for (int m = 0; m < 512; ++m)
        if (h[m]) order.push_back(m);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return h[a] > h[b]; });   // stable: lower mask first
    const int n = (int)order.size() < n_patterns ? (int)order.size() : n_patterns;
    for (int i = 0; i < n; ++i) {
        lib_host[i] = (uint16_t)order[i];
        if (score_host) score_host[i] = h[order[i]];
    }
    *n_found = n;
    return PC_OK;
}

// ------------------------------------------------------------------ adaptive finalisation
__global__ void __launch_bounds__(256)
pc_finalize_count_kernel(const uint8_t *__restrict__ pid, int64_t nk, int P, uint32_t *__restrict__ counts)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nk) return;
    const int p = pid[k];
    if (p < P) counts[k * P + p] += 1u;             // one thread per kernel: no other thread touches this row
}

__global__ void __launch_bounds__(256)
pc_finalize_pick_kernel(const uint32_t *__restrict__ counts, int64_t nk, int P, uint8_t *__restrict__ pid)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nk) return;
    int best = 0;
    uint32_t bc = counts[k * P];
    for (int p = 1; p < P; ++p) {
        const uint32_t c = counts[k * P + p];
        if (c > bc) { bc = c; best = p; }
    }
    pid[k] = (uint8_t)best;
}

__global__ void __launch_bounds__(256) pc_finalize_count_batch_kernel(TsBatchArg b, int P)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    const int64_t k = (int64_t)((int)blockIdx.x - b.blk0[l]) * 256 + threadIdx.x;
    if (k >= b.nk[l]) return;
    const int p = b.pid[l][k];
    if (p < P) static_cast<uint32_t *>(b.out[l])[k * P + p] += 1u;
}

__global__ void __launch_bounds__(256) pc_finalize_pick_batch_kernel(TsBatchArg b, int P)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    const int64_t k = (int64_t)((int)blockIdx.x - b.blk0[l]) * 256 + threadIdx.x;
    if (k >= b.nk[l]) return;
    const uint32_t *counts = b.counts[l];
    int best = 0;
    uint32_t bc = counts[k * P];
    for (int p = 1; p < P; ++p) {
        const uint32_t c = counts[k * P + p];
        if (c > bc) { bc = c; best = p; }
    }
    static_cast<uint8_t *>(b.out[l])[k] = (uint8_t)best;
}

static pc_status ts_check_counts(pc_ctx *ctx, const char *who, const void *a, const void *b, int32_t F, int32_t C, int32_t P)
{
    if (!a || !b) return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: null pointer", who);
    if (F < 1 || C < 1 || F > 65535 || C > 65535) return pc_fail(ctx, PC_ERR_BAD_SHAPE, "%s: F=%d C=%d out of range", who, F, C);
    if (P < 1 || P > PC_MAX_P) return pc_fail(ctx, PC_ERR_BAD_LIBRARY, "%s: P=%d outside 1..%d", who, P, PC_MAX_P);
    return PC_OK;
}

extern "C" pc_status pc_finalize_count(pc_ctx *ctx, const uint8_t *pid, int32_t F, int32_t C, int32_t P, uint32_t *counts)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = ts_check_counts(ctx, "pc_finalize_count", pid, counts, F, C, P);
    if (s != PC_OK) return s;
    PC_HIP(ctx, hipSetDevice(ctx->device));
    const int64_t nk = (int64_t)F * C;
    hipLaunchKernelGGL(pc_finalize_count_kernel, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, ctx->stream, pid, nk, P, counts);
    return pc_hip_check(ctx, hipGetLastError(), "finalisation count launch");
}

extern "C" pc_status pc_finalize_pick(pc_ctx *ctx, const uint32_t *counts, int32_t F, int32_t C, int32_t P, uint8_t *pid)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = ts_check_counts(ctx, "pc_finalize_pick", counts, pid, F, C, P);
    if (s != PC_OK) return s;
    PC_HIP(ctx, hipSetDevice(ctx->device));
    const int64_t nk = (int64_t)F * C;
    hipLaunchKernelGGL(pc_finalize_pick_kernel, dim3((unsigned)((nk + 255) / 256)), dim3(256), 0, ctx->stream, counts, nk, P, pid);
    return pc_hip_check(ctx, hipGetLastError(), "finalisation pick launch");
}

// ------------------------------------------------------------------ modified group lasso
// One thread per kernel; W and dW pass through LDS so that global accesses are contiguous.
__device__ __forceinline__ void ts_group_lasso_block(const float *__restrict__ W, const uint8_t *__restrict__ pid,
                                                     const uint8_t *__restrict__ keep, int64_t nk, const LibArg &la, float lambda_p,
                                                     float lambda_i, float *__restrict__ dW, double *__restrict__ block_pen,
                                                     int blk)
{
    __shared__ float sw[TS_BLOCK * 9], sd[TS_BLOCK * 9];
    __shared__ uint16_t lmask[PC_MAX_P + 2];
    __shared__ double red[TS_BLOCK];
    const int64_t k0 = (int64_t)blk * TS_BLOCK;
    const int n = nk - k0 < TS_BLOCK ? (int)(nk - k0) : TS_BLOCK;
    if (threadIdx.x < la.P) lmask[threadIdx.x] = la.mask[threadIdx.x];
    ts_stage(sw, W + k0 * 9, n);
    ts_stage(sd, dW + k0 * 9, n);
    int p = 0, kp = 1;
    if (threadIdx.x < n) { p = pid[k0 + threadIdx.x]; kp = keep[k0 + threadIdx.x]; }
    __syncthreads();
    double pen = 0.0;
    if (threadIdx.x < n) {
        const unsigned m = p < la.P ? lmask[p] : 0x1FFu;   // an id outside the pool penalises nothing by pattern
        float w[9];
        float zn2 = 0.0f, un2 = 0.0f;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            w[t] = sw[threadIdx.x * 9 + t];
            const float sq = w[t] * w[t];
            zn2 = zn2 + (((m >> t) & 1u) ? 0.0f : sq);
            un2 = un2 + sq;
        }
        if (kp) un2 = 0.0f;
        const float zn = sqrtf(zn2), un = sqrtf(un2);
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            float g = 0.0f;
            if (!((m >> t) & 1u) && zn > 0.0f) g = lambda_p * (w[t] / zn);
            if (!kp && un > 0.0f) g = g + lambda_i * (w[t] / un);
            sd[threadIdx.x * 9 + t] += g;
        }
        pen = (double)lambda_p * (double)zn + (double)lambda_i * (double)un;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 9; ++j) {
        const int i = j * TS_BLOCK + threadIdx.x;
        if (i < n * 9) dW[k0 * 9 + i] = sd[i];
    }
    if (block_pen) {                                // fixed-order tree over the workgroup
        red[threadIdx.x] = pen;
        __syncthreads();
        for (int d = TS_BLOCK / 2; d > 0; d >>= 1) {
            if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
            __syncthreads();
        }
        if (threadIdx.x == 0) block_pen[blockIdx.x] = red[0];    // one slot per workgroup of the launch
    }
}

__global__ void __launch_bounds__(TS_BLOCK)
pc_group_lasso_kernel(const float *__restrict__ W, const uint8_t *__restrict__ pid, const uint8_t *__restrict__ keep, int64_t nk,
                      LibArg la, float lambda_p, float lambda_i, float *__restrict__ dW, double *__restrict__ block_pen)
{
    ts_group_lasso_block(W, pid, keep, nk, la, lambda_p, lambda_i, dW, block_pen, (int)blockIdx.x);
}

__global__ void __launch_bounds__(TS_BLOCK)
pc_group_lasso_batch_kernel(TsBatchArg b, LibArg la, float lambda_p, float lambda_i, double *__restrict__ block_pen)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    ts_group_lasso_block(b.W[l], b.pid[l], b.keep[l], b.nk[l], la, lambda_p, lambda_i, static_cast<float *>(b.out[l]), block_pen,
                         (int)blockIdx.x - b.blk0[l]);
}

// penalty = the workgroup sums added in a fixed order by one workgroup
__global__ void __launch_bounds__(256) pc_group_lasso_sum_kernel(const double *__restrict__ block_pen, int nb, double *__restrict__ out)
{
    __shared__ double red[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < nb; i += 256) s += block_pen[i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
        if (threadIdx.x < d) red[threadIdx.x] += red[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0];
}

extern "C" pc_status pc_group_lasso_grad(pc_ctx *ctx, const float *W, const uint8_t *pid, const uint8_t *keep, int32_t F,
                                         int32_t C, const uint16_t *lib, int32_t P, float lambda_p, float lambda_i,
                                         float *dW, double *penalty)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!W || !pid || !keep || !lib || !dW) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_group_lasso_grad: null pointer");
    if (F < 1 || C < 1 || F > 65535 || C > 65535)
        return pc_fail(ctx, PC_ERR_BAD_SHAPE, "pc_group_lasso_grad: F=%d C=%d out of range", F, C);
    pc_status s = pc_check_library(lib, P);
    if (s != PC_OK) return pc_fail(ctx, s, "pc_group_lasso_grad: bad library (P=%d)", P);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    LibArg la;
    pc_fill_lib(&la, lib, P);
    const int64_t nk = (int64_t)F * C;
    const unsigned nb = (unsigned)((nk + TS_BLOCK - 1) / TS_BLOCK);
    double *block_pen = nullptr;
    if (penalty) {
        void *scr = nullptr;
        s = pc_scratch(ctx, sizeof(double) * nb, &scr);
        if (s != PC_OK) return s;
        block_pen = (double *)scr;
    }
    hipLaunchKernelGGL(pc_group_lasso_kernel, dim3(nb), dim3(TS_BLOCK), 0, ctx->stream, W, pid, keep, nk, la, lambda_p, lambda_i,
                       dW, block_pen);
    if (penalty)
        hipLaunchKernelGGL(pc_group_lasso_sum_kernel, dim3(1), dim3(256), 0, ctx->stream, block_pen, (int)nb, penalty);
    return pc_hip_check(ctx, hipGetLastError(), "group lasso launch");
}

// ------------------------------------------------------------------ the same steps for the layers of a network at once
// Fills the table for layers [l0, l0 + m); false with a message when a layer is malformed.
static pc_status ts_fill_batch(pc_ctx *ctx, const char *who, TsBatchArg *b, int l0, int m, const int32_t *F, const int32_t *C)
{
    memset(b, 0, sizeof(*b));
    b->n = m;
    for (int i = 0; i < m; ++i) {
        const int l = l0 + i;
        if (F[l] < 1 || C[l] < 1 || F[l] > 65535 || C[l] > 65535)
            return pc_fail(ctx, PC_ERR_BAD_SHAPE, "%s: layer %d: F=%d C=%d out of range", who, l, F[l], C[l]);
        b->nk[i] = (int64_t)F[l] * C[l];
        b->blk0[i + 1] = b->blk0[i] + (int32_t)((b->nk[i] + TS_BLOCK - 1) / TS_BLOCK);
    }
    return PC_OK;
}

extern "C" pc_status pc_dppg_accumulate_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W, const float *const *G,
                                              const int32_t *F, const int32_t *C, uint32_t *hist, uint16_t *const *masks)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_dppg_accumulate_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!W || !F || !C || !hist) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_dppg_accumulate_batch: null pointer");
    for (int l = 0; l < n_layers; ++l)
        if (!W[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_dppg_accumulate_batch: null pointer in layer %d", l);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    for (int l0 = 0; l0 < n_layers; l0 += PC_BATCH_MAX) {
        const int m = n_layers - l0 < PC_BATCH_MAX ? n_layers - l0 : PC_BATCH_MAX;
        TsBatchArg b;
        pc_status s = ts_fill_batch(ctx, "pc_dppg_accumulate_batch", &b, l0, m, F, C);
        if (s != PC_OK) return s;
        for (int i = 0; i < m; ++i) {
            b.W[i] = W[l0 + i];
            b.G[i] = G ? G[l0 + i] : nullptr;
            b.out[i] = masks ? masks[l0 + i] : nullptr;
        }
        int nb = b.blk0[m];
        if (nb > 2 * ctx->num_cu) nb = 2 * ctx->num_cu;
        hipLaunchKernelGGL(pc_dppg_batch_kernel, dim3((unsigned)nb), dim3(TS_BLOCK), 0, ctx->stream, b, hist);
    }
    return pc_hip_check(ctx, hipGetLastError(), "pool generation (several layers) launch");
}

extern "C" pc_status pc_finalize_count_batch(pc_ctx *ctx, int32_t n_layers, const uint8_t *const *pid, const int32_t *F,
                                             const int32_t *C, int32_t P, uint32_t *const *counts)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_finalize_count_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!pid || !F || !C || !counts) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_finalize_count_batch: null pointer");
    if (P < 1 || P > PC_MAX_P) return pc_fail(ctx, PC_ERR_BAD_LIBRARY, "pc_finalize_count_batch: P=%d outside 1..%d", P, PC_MAX_P);
    for (int l = 0; l < n_layers; ++l)
        if (!pid[l] || !counts[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_finalize_count_batch: null pointer in layer %d", l);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    for (int l0 = 0; l0 < n_layers; l0 += PC_BATCH_MAX) {
        const int m = n_layers - l0 < PC_BATCH_MAX ? n_layers - l0 : PC_BATCH_MAX;
        TsBatchArg b;
        pc_status s = ts_fill_batch(ctx, "pc_finalize_count_batch", &b, l0, m, F, C);
        if (s != PC_OK) return s;
        for (int i = 0; i < m; ++i) { b.pid[i] = pid[l0 + i]; b.out[i] = counts[l0 + i]; }
        hipLaunchKernelGGL(pc_finalize_count_batch_kernel, dim3((unsigned)b.blk0[m]), dim3(256), 0, ctx->stream, b, P);
    }
    return pc_hip_check(ctx, hipGetLastError(), "finalisation count (several layers) launch");
}

extern "C" pc_status pc_finalize_pick_batch(pc_ctx *ctx, int32_t n_layers, const uint32_t *const *counts, const int32_t *F,
                                            const int32_t *C, int32_t P, uint8_t *const *pid)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_finalize_pick_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!pid || !F || !C || !counts) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_finalize_pick_batch: null pointer");
    if (P < 1 || P > PC_MAX_P) return pc_fail(ctx, PC_ERR_BAD_LIBRARY, "pc_finalize_pick_batch: P=%d outside 1..%d", P, PC_MAX_P);
    for (int l = 0; l < n_layers; ++l)
        if (!pid[l] || !counts[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_finalize_pick_batch: null pointer in layer %d", l);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    for (int l0 = 0; l0 < n_layers; l0 += PC_BATCH_MAX) {
        const int m = n_layers - l0 < PC_BATCH_MAX ? n_layers - l0 : PC_BATCH_MAX;
        TsBatchArg b;
        pc_status s = ts_fill_batch(ctx, "pc_finalize_pick_batch", &b, l0, m, F, C);
        if (s != PC_OK) return s;
        for (int i = 0; i < m; ++i) { b.counts[i] = counts[l0 + i]; b.out[i] = pid[l0 + i]; }
        hipLaunchKernelGGL(pc_finalize_pick_batch_kernel, dim3((unsigned)b.blk0[m]), dim3(256), 0, ctx->stream, b, P);
    }
    return pc_hip_check(ctx, hipGetLastError(), "finalisation pick (several layers) launch");
}

extern "C" pc_status pc_group_lasso_grad_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W, const uint8_t *const *pid,
                                               const uint8_t *const *keep, const int32_t *F, const int32_t *C, const uint16_t *lib,
                                               int32_t P, float lambda_p, float lambda_i, float *const *dW, double *penalty)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_group_lasso_grad_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!W || !pid || !keep || !F || !C || !lib || !dW) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_group_lasso_grad_batch: null pointer");
    if (n_layers > PC_BATCH_MAX && penalty)
        return pc_fail(ctx, PC_ERR_UNSUPPORTED, "pc_group_lasso_grad_batch: the penalty of more than %d layers takes several calls", PC_BATCH_MAX);
    for (int l = 0; l < n_layers; ++l)
        if (!W[l] || !pid[l] || !keep[l] || !dW[l])
            return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_group_lasso_grad_batch: null pointer in layer %d", l);
    pc_status s = pc_check_library(lib, P);
    if (s != PC_OK) return pc_fail(ctx, s, "pc_group_lasso_grad_batch: bad library (P=%d)", P);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    LibArg la;
    pc_fill_lib(&la, lib, P);
    for (int l0 = 0; l0 < n_layers; l0 += PC_BATCH_MAX) {
        const int m = n_layers - l0 < PC_BATCH_MAX ? n_layers - l0 : PC_BATCH_MAX;
        TsBatchArg b;
        s = ts_fill_batch(ctx, "pc_group_lasso_grad_batch", &b, l0, m, F, C);
        if (s != PC_OK) return s;
        for (int i = 0; i < m; ++i) {
            b.W[i] = W[l0 + i]; b.pid[i] = pid[l0 + i]; b.keep[i] = keep[l0 + i]; b.out[i] = dW[l0 + i];
        }
        const int nb = b.blk0[m];
        double *block_pen = nullptr;
        if (penalty) {
            void *scr = nullptr;
            s = pc_scratch(ctx, sizeof(double) * (size_t)nb, &scr);
            if (s != PC_OK) return s;
            block_pen = (double *)scr;
        }
        hipLaunchKernelGGL(pc_group_lasso_batch_kernel, dim3((unsigned)nb), dim3(TS_BLOCK), 0, ctx->stream, b, la, lambda_p, lambda_i,
                           block_pen);
        if (penalty)
            hipLaunchKernelGGL(pc_group_lasso_sum_kernel, dim3(1), dim3(256), 0, ctx->stream, block_pen, nb, penalty);
    }
    return pc_hip_check(ctx, hipGetLastError(), "group lasso (several layers) launch");
}

// Pattern/kernel selection (Section 4.1, Eq. 1 and Eq. 2) and packing (Section 5.1) kernels.
//
// Selection is bit-reproducible: float32, fixed operation order, no fused multiply-add
// (this file must be compiled with -ffp-contract=off).
#include "pc_internal.h"

// ------------------------------------------------------------------ selection
// One thread per kernel (f,c): 9 tap importances, the best pattern of the pool, the ranking score.
__global__ void __launch_bounds__(256)
pc_select_score_kernel(const float *__restrict__ W, const float *__restrict__ G, int64_t nk, LibArg la,
                       int score_mode, uint8_t *__restrict__ pid, float *__restrict__ R)
{
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= nk) return;
    float s[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        float w = W[k * 9 + t];
        if (G) {
            float gw = G[k * 9 + t] * w;
            s[t] = gw * gw;
        } else {
            s[t] = w * w;
        }
    }
    int best = 0;
    float best_score = 0.0f;
    for (int p = 0; p < la.P; ++p) {
        unsigned m = la.mask[p];
        float acc = 0.0f;
        bool first = true;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (m & (1u << t)) {
                acc = first ? s[t] : acc + s[t];
                first = false;
            }
        }
        if (p == 0 || acc > best_score) {
            best_score = acc;
            best = p;
        }
    }
    pid[k] = (uint8_t)best;
    if (score_mode == PC_SCORE_KERNEL) {
        float acc = s[0];
#pragma unroll
        for (int t = 1; t < 9; ++t) acc = acc + s[t];
        R[k] = acc;
    } else {
        R[k] = best_score;
    }
}

// Exact rank inside a segment of length L: element i is kept iff fewer than n_keep elements
// precede it in the order (score descending, index ascending).
#define PC_RANK_CHUNK 2048
__global__ void __launch_bounds__(256)
pc_select_rank_kernel(const float *__restrict__ R, int64_t L, int64_t n_keep, uint8_t *__restrict__ keep)
{
    __shared__ float tile[PC_RANK_CHUNK];
    const float *seg = R + (int64_t)blockIdx.y * L;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    bool live = i < L;
    float mine = live ? seg[i] : 0.0f;
    int64_t before = 0;
    for (int64_t j0 = 0; j0 < L; j0 += PC_RANK_CHUNK) {
        int64_t m = L - j0 < PC_RANK_CHUNK ? L - j0 : PC_RANK_CHUNK;
        __syncthreads();
        for (int64_t j = threadIdx.x; j < m; j += blockDim.x) tile[j] = seg[j0 + j];
        __syncthreads();
        if (live) {
            int cnt = 0;
            for (int64_t j = 0; j < m; ++j) {
                float o = tile[j];
                cnt += (o > mine) || (o == mine && (j0 + j) < i);
            }
            before += cnt;
        }
    }
    if (live) keep[(int64_t)blockIdx.y * L + i] = before < n_keep ? 1 : 0;
}

// Exact top-n_keep of every row of R (n rows of length L, L <= PC_TOPN_MAX) in the order (score descending,
// index ascending), one workgroup per row: a 4-pass radix select over order-preserving 32-bit keys finds the
// score of the n_keep-th kernel and how many kernels with exactly that score are kept; those are the ones
// with the lowest indices. Counts are integers: the result does not depend on the order of the atomics.
#define PC_TOPN_MAX 8192
__device__ __forceinline__ uint32_t pc_order_key(float f)
{
    const uint32_t b = __float_as_uint(f);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);   // a > b as floats  <=>  key(a) > key(b) as unsigned
}

__global__ void __launch_bounds__(256)
pc_select_topn_row_kernel(const float *__restrict__ R, int L, int n_keep, uint8_t *__restrict__ keep)
{
    extern __shared__ uint32_t keys[];          // L keys
    __shared__ int hist[256], above[256];
    __shared__ uint32_t s_prefix;
    __shared__ int s_remaining, s_wave_cnt[4], s_base;
    const float *seg = R + (int64_t)blockIdx.x * L;
    uint8_t *out = keep + (int64_t)blockIdx.x * L;
    if (n_keep <= 0 || n_keep >= L) {
        for (int i = threadIdx.x; i < L; i += 256) out[i] = n_keep > 0 ? 1 : 0;
        return;
    }
    for (int i = threadIdx.x; i < L; i += 256) keys[i] = pc_order_key(seg[i]);
    if (threadIdx.x == 0) { s_prefix = 0u; s_remaining = n_keep; }
    __syncthreads();
    for (int shift = 24; shift >= 0; shift -= 8) {
        hist[threadIdx.x] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        const uint32_t himask = shift == 24 ? 0u : 0xFFFFFFFFu << (shift + 8);
        for (int i = threadIdx.x; i < L; i += 256) {
            const uint32_t k = keys[i];
            if ((k & himask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
        }
        __syncthreads();
        // above[d] = number of candidates whose digit is larger than d (suffix sum, exclusive)
        above[threadIdx.x] = hist[threadIdx.x];
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {
            const int add = threadIdx.x + d < 256 ? above[threadIdx.x + d] : 0;
            __syncthreads();
            above[threadIdx.x] += add;
            __syncthreads();
        }
        const int incl = above[threadIdx.x], excl = incl - hist[threadIdx.x];
        const int rem = s_remaining;
        __syncthreads();
        if (excl < rem && rem <= incl) {        // exactly one digit holds the rem-th largest candidate
            s_prefix = prefix | ((uint32_t)threadIdx.x << shift);
            s_remaining = rem - excl;
        }
        __syncthreads();
    }
    const uint32_t T = s_prefix;
    const int take_equal = s_remaining;         // kernels with key == T that are kept: the first ones by index
    if (threadIdx.x == 0) s_base = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i0 = 0; i0 < L; i0 += 256) {
        const int i = i0 + threadIdx.x;
        const uint32_t k = i < L ? keys[i] : 0u;
        const bool eq = i < L && k == T;
        const unsigned long long b = __ballot(eq);
        if (lane == 0) s_wave_cnt[wave] = __popcll(b);
        __syncthreads();
        int before = s_base + __popcll(b & ((1ull << lane) - 1ull));
        for (int w2 = 0; w2 < wave; ++w2) before += s_wave_cnt[w2];
        if (i < L) out[i] = (k > T || (eq && before < take_equal)) ? 1 : 0;
        __syncthreads();
        if (threadIdx.x == 0) s_base += s_wave_cnt[0] + s_wave_cnt[1] + s_wave_cnt[2] + s_wave_cnt[3];
        __syncthreads();
    }
}

pc_status pc_launch_select(pc_ctx *ctx, const float *W, const float *G, int F, int C, const LibArg &la,
                           pc_keep_mode km, int64_t n_keep, pc_score_mode sm, uint8_t *pid, uint8_t *keep)
{
    int64_t nk = (int64_t)F * C;
    void *scr = nullptr;
    pc_status s = pc_scratch(ctx, sizeof(float) * (size_t)nk, &scr);
    if (s != PC_OK) return s;
    float *R = (float *)scr;
    unsigned blocks = (unsigned)((nk + 255) / 256);
    hipLaunchKernelGGL(pc_select_score_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, G, nk, la, (int)sm, pid, R);
    int64_t L = (km == PC_KEEP_PER_FILTER) ? C : nk;
    unsigned nseg = (km == PC_KEEP_PER_FILTER) ? (unsigned)F : 1u;
    if (L <= PC_TOPN_MAX) {
        hipLaunchKernelGGL(pc_select_topn_row_kernel, dim3(nseg), dim3(256), sizeof(uint32_t) * (size_t)L, ctx->stream, R, (int)L,
                           (int)(n_keep < L ? n_keep : L), keep);
    } else {
        dim3 grid((unsigned)((L + 255) / 256), nseg);
        hipLaunchKernelGGL(pc_select_rank_kernel, grid, dim3(256), 0, ctx->stream, R, L, n_keep, keep);
    }
    return pc_hip_check(ctx, hipGetLastError(), "select launch");
}

// ------------------------------------------------------------------ packing
// Table rows are filters (row stride C, element stride 1 in the [F][C] maps) for the
// filter-major table, channels (row stride 1, element stride C) for the channel-major one.

// Kept kernels of every row, per pattern id.
__global__ void __launch_bounds__(256)
pc_pack_count_kernel(const uint8_t *__restrict__ pid, const uint8_t *__restrict__ keep, int rows, int len,
                     int64_t row_stride, int64_t elem_stride, int P, int32_t *__restrict__ grp,
                     int32_t *__restrict__ rowptr)
{
    __shared__ int hist[PC_MAX_P + 1];
    int row = blockIdx.x;
    for (int p = threadIdx.x; p <= PC_MAX_P; p += blockDim.x) hist[p] = 0;
    __syncthreads();
    for (int e = threadIdx.x; e < len; e += blockDim.x) {
        int64_t k = row * row_stride + e * elem_stride;
        if (keep[k] && pid[k] < P) atomicAdd(&hist[pid[k]], 1);   // integer counts: order does not matter
    }
    __syncthreads();
    for (int p = threadIdx.x; p < P; p += blockDim.x) grp[(int64_t)row * (PC_MAX_P + 1) + p] = hist[p];
    if (threadIdx.x == 0) {
        int tot = 0;
        for (int p = 0; p < P; ++p) tot += hist[p];
        rowptr[row] = tot;
    }
}

// In-place exclusive scan of rowptr[0..rows) with the total written to rowptr[rows]. One block.
__global__ void __launch_bounds__(1024) pc_pack_scan_kernel(int32_t *rowptr, int rows)
{
    __shared__ int part[1024];
    int per = (rows + 1023) / 1024;
    int lo = threadIdx.x * per, hi = lo + per < rows ? lo + per : rows;
    int sum = 0;
    for (int i = lo; i < hi; ++i) sum += rowptr[i];
    part[threadIdx.x] = sum;
    __syncthreads();
    // inclusive prefix over the 1024 partial sums (integers: any order gives the same result)
    for (int d = 1; d < 1024; d <<= 1) {
        int add = threadIdx.x >= d ? part[threadIdx.x - d] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    if (threadIdx.x == 1023) rowptr[rows] = part[1023];
    int run = part[threadIdx.x] - sum;
    for (int i = lo; i < hi; ++i) {
        int v = rowptr[i];
        rowptr[i] = run;
        run += v;
    }
}

__device__ __forceinline__ float4 pc_gather_taps(const float *__restrict__ W, int64_t k, const uint8_t *tp, bool bf16)
{
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float w = W[k * 9 + tp[j]];
        v[j] = bf16 ? pc_bf16_to_f32(pc_f32_to_bf16(w)) : w;
    }
    return make_float4(v[0], v[1], v[2], v[3]);
}

// Places the kept kernels of one row at rowptr[row] + (pattern group start) + (rank inside the group).
// Each wave takes patterns wave, wave+4, ... and walks the row 64 elements at a time; the rank of
// an element is the number of earlier group members, so the order inside a group is ascending.
__global__ void __launch_bounds__(256)
pc_pack_place_kernel(const float *__restrict__ W, const uint8_t *__restrict__ pid, const uint8_t *__restrict__ keep,
                     int rows, int len, int64_t row_stride, int64_t elem_stride, LibArg la, int bf16,
                     int filter_major, PackView v)
{
    __shared__ int start[PC_MAX_P + 1];
    int row = blockIdx.x;
    int32_t *grp = (filter_major ? v.fm_grp : v.cm_grp) + (int64_t)row * (PC_MAX_P + 1);
    const int32_t *rowptr = filter_major ? v.fm_rowptr : v.cm_rowptr;
    if (threadIdx.x == 0) {
        int run = rowptr[row];
        for (int p = 0; p < la.P; ++p) {
            int cnt = grp[p];
            start[p] = run;
            grp[p] = run;
            run += cnt;
        }
        grp[la.P] = run;
    }
    __syncthreads();
    int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int p = wave; p < la.P; p += 4) {
        int run = start[p];
        for (int e0 = 0; e0 < len; e0 += 64) {
            int e = e0 + lane;
            int64_t k = row * row_stride + e * elem_stride;
            bool hit = e < len && keep[k] && pid[k] == p;
            unsigned long long b = __ballot(hit);
            if (hit) {
                int slot = run + __popcll(b & ((1ull << lane) - 1ull));
                float4 val = pc_gather_taps(W, k, la.taps[p], bf16 != 0);
                if (filter_major) {
                    v.fm_c[slot] = (uint16_t)e;
                    v.fm_pid[slot] = (uint8_t)p;
                    v.slot_f[slot] = (uint16_t)row;
                    v.fm_val[slot] = val;
                    v.slot_of[k] = slot;
                    v.kinfo[k] = ((uint32_t)slot << 9) | la.mask[p];
                } else {
                    v.cm_f[slot] = (uint16_t)e;
                    v.cm_slot[slot] = v.slot_of[k];
                    v.cm_val[slot] = val;
                }
            }
            run += __popcll(b);
        }
    }
    if (filter_major) {
        for (int e = threadIdx.x; e < len; e += blockDim.x) {
            int64_t k = row * row_stride + e * elem_stride;
            if (!keep[k]) { v.slot_of[k] = -1; v.kinfo[k] = 0xFFFFFFFFu; }
        }
    }
}

// Re-gathers values with unchanged tables (one thread per kernel (f,c)).
__global__ void __launch_bounds__(256)
pc_pack_regather_fm_kernel(const float *__restrict__ W, LibArg la, int bf16, PackView v)
{
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= (int64_t)v.F * v.C) return;
    int slot = v.slot_of[k];
    if (slot < 0) return;
    v.fm_val[slot] = pc_gather_taps(W, k, la.taps[v.fm_pid[slot]], bf16 != 0);
}

__global__ void __launch_bounds__(256) pc_pack_regather_cm_kernel(PackView v)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= v.cm_rowptr[v.C]) return;
    v.cm_val[i] = v.fm_val[v.cm_slot[i]];
}

pc_status pc_launch_pack(pc_ctx *ctx, pc_packed *pk, const float *W, const uint8_t *pid, const uint8_t *keep)
{
    PackView v = pk->v;
    LibArg la;
    pc_fill_lib(&la, pk->lib, v.P);
    int bf16 = pk->dtype == PC_BF16;
    hipStream_t st = ctx->stream;
    // filter-major
    hipLaunchKernelGGL(pc_pack_count_kernel, dim3(v.F), dim3(256), 0, st, pid, keep, v.F, v.C, (int64_t)v.C,
                       (int64_t)1, v.P, v.fm_grp, v.fm_rowptr);
    hipLaunchKernelGGL(pc_pack_scan_kernel, dim3(1), dim3(1024), 0, st, v.fm_rowptr, v.F);
    hipLaunchKernelGGL(pc_pack_place_kernel, dim3(v.F), dim3(256), 0, st, W, pid, keep, v.F, v.C, (int64_t)v.C,
                       (int64_t)1, la, bf16, 1, v);
    // channel-major: the table of the gather kernels' backward-data pass (the matrix-core kernels read operand tiles)
    if (pk->variant != PC_VARIANT_MFMA) {
        hipLaunchKernelGGL(pc_pack_count_kernel, dim3(v.C), dim3(256), 0, st, pid, keep, v.C, v.F, (int64_t)1,
                           (int64_t)v.C, v.P, v.cm_grp, v.cm_rowptr);
        hipLaunchKernelGGL(pc_pack_scan_kernel, dim3(1), dim3(1024), 0, st, v.cm_rowptr, v.C);
        hipLaunchKernelGGL(pc_pack_place_kernel, dim3(v.C), dim3(256), 0, st, W, pid, keep, v.C, v.F, (int64_t)1,
                           (int64_t)v.C, la, bf16, 0, v);
    }
    pc_status s = pc_hip_check(ctx, hipGetLastError(), "pack launch");
    if (s == PC_OK && pk->variant == PC_VARIANT_MFMA) s = pc_launch_pack_tiles(ctx, pk, W);
    return s;
}

pc_status pc_launch_update_values(pc_ctx *ctx, pc_packed *pk, const float *W)
{
    PackView v = pk->v;
    LibArg la;
    pc_fill_lib(&la, pk->lib, v.P);
    int bf16 = pk->dtype == PC_BF16;
    int64_t nk = (int64_t)v.F * v.C;
    unsigned blocks = (unsigned)((nk + 255) / 256);
    hipLaunchKernelGGL(pc_pack_regather_fm_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, la, bf16, v);
    if (pk->variant != PC_VARIANT_MFMA)
        hipLaunchKernelGGL(pc_pack_regather_cm_kernel, dim3(blocks), dim3(256), 0, ctx->stream, v);
    pc_status s = pc_hip_check(ctx, hipGetLastError(), "update_values launch");
    if (s == PC_OK && pk->variant == PC_VARIANT_MFMA) s = pc_launch_pack_tiles(ctx, pk, W);
    return s;
}

// dense[f][c][t] = value of the kept tap, 0 elsewhere. Source: a compact array or the pack's own values.
__global__ void __launch_bounds__(256)
pc_scatter_kernel(const float *__restrict__ compact, float *__restrict__ dense, LibArg la, PackView v)
{
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= (int64_t)v.F * v.C) return;
    float out[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) out[t] = 0.0f;
    int slot = v.slot_of[k];
    if (slot >= 0) {
        float4 val = compact ? reinterpret_cast<const float4 *>(compact)[slot] : v.fm_val[slot];
        unsigned m = la.mask[v.fm_pid[slot]];
        float vv[4] = {val.x, val.y, val.z, val.w};
        int j = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            if (m & (1u << t)) {
                out[t] = j == 0 ? vv[0] : j == 1 ? vv[1] : j == 2 ? vv[2] : vv[3];
                ++j;
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 9; ++t) dense[k * 9 + t] = out[t];
}

pc_status pc_launch_scatter(pc_ctx *ctx, const pc_packed *pk, const float *compact, float *dense, int from_pack)
{
    PackView v = pk->v;
    LibArg la;
    pc_fill_lib(&la, pk->lib, v.P);
    int64_t nk = (int64_t)v.F * v.C;
    unsigned blocks = (unsigned)((nk + 255) / 256);
    hipLaunchKernelGGL(pc_scatter_kernel, dim3(blocks), dim3(256), 0, ctx->stream, from_pack ? nullptr : compact, dense,
                       la, v);
    return pc_hip_check(ctx, hipGetLastError(), "scatter launch");
}

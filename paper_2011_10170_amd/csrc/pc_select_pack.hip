// Pattern/kernel selection (Section 4.1, Eq. 1 and Eq. 2) and packing (Section 5.1) kernels.
//
// Selection is bit-reproducible: float32, fixed operation order, no fused multiply-add
// (this file must be compiled with -ffp-contract=off).
#include "pc_internal.h"

// ------------------------------------------------------------------ selection
// Tap importances of one kernel -> best pattern of the pool and the ranking score. Every sum is taken in
// ascending tap order, one rounded float32 addition at a time. The importances are squares, so none is below +0
// and adding +0 for a tap outside the pattern changes no bit: the 9 unconditional additions below give exactly
// ((s_a + s_b) + s_c) + s_d of the pattern's taps a < b < c < d. masks may point to kernel arguments or LDS.
__device__ __forceinline__ void pc_score_taps(const float (&s)[9], const uint16_t *masks, int P, int score_mode,
                                              int *pid_out, float *rank_out)
{
    int best = 0;
    float best_score = 0.0f;
#pragma unroll 2
    for (int p = 0; p < P; ++p) {
        const unsigned m = masks[p];
        float acc = 0.0f;
#pragma unroll
        for (int t = 0; t < 9; ++t) acc = acc + (((m >> t) & 1u) ? s[t] : 0.0f);
        if (p == 0 || acc > best_score) {
            best_score = acc;
            best = p;
        }
    }
    *pid_out = best;
    if (score_mode == PC_SCORE_KERNEL) {
        float acc = s[0];
#pragma unroll
        for (int t = 1; t < 9; ++t) acc = acc + s[t];
        *rank_out = acc;
    } else {
        *rank_out = best_score;
    }
}

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
    int best;
    float r;
    pc_score_taps(s, la.mask, la.P, score_mode, &best, &r);
    pid[k] = (uint8_t)best;
    R[k] = r;
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

// Selection of one filter row in one workgroup (rows of up to PC_TOPN_MAX kernels): scores as in the kernel
// above, then the top n_keep of the row by the same radix select, without the round trip of the scores through
// memory. W and G reach the lanes through LDS so that the global loads are contiguous.
__device__ __forceinline__ void pc_select_row_body(const float *__restrict__ W, const float *__restrict__ G, int C, const LibArg &la,
                                                   int score_mode, int n_keep, uint8_t *__restrict__ pid,
                                                   uint8_t *__restrict__ keep, int row)
{
    extern __shared__ uint32_t dyn[];           // C keys, then blockDim.x * 9 floats of W, then as many of G
    __shared__ int hist[256];
    __shared__ uint32_t s_prefix;
    __shared__ int s_remaining, s_wave_cnt[16], s_base;
    __shared__ uint16_t s_mask[PC_MAX_P + 2];
    const int T = blockDim.x, tid = threadIdx.x;
    if (tid < la.P) s_mask[tid] = la.mask[tid];   // visible after the first barrier of the loop below
    uint32_t *keys = dyn;
    float *sw = reinterpret_cast<float *>(dyn + C);
    float *sg = sw + (size_t)T * 9;
    const int64_t row0 = (int64_t)row * C;
    for (int c0 = 0; c0 < C; c0 += T) {
        const int n = C - c0 < T ? C - c0 : T;
        const float *wsrc = W + (row0 + c0) * 9;
        const float *gsrc = G ? G + (row0 + c0) * 9 : nullptr;
        if (c0) __syncthreads();
        // all loads of the thread first (index clamped, so they are unconditional), then the LDS writes: one memory
        // round trip per chunk instead of one per element
        float rw[9], rg[9];
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const int i = j * T + tid, ic = i < n * 9 ? i : n * 9 - 1;
            rw[j] = wsrc[ic];
            rg[j] = gsrc ? gsrc[ic] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 9; ++j) {
            const int i = j * T + tid;
            if (i < n * 9) {
                sw[i] = rw[j];
                if (gsrc) sg[i] = rg[j];
            }
        }
        __syncthreads();
        if (tid < n) {
            float s[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const float w = sw[tid * 9 + t];
                if (gsrc) {
                    const float gw = sg[tid * 9 + t] * w;
                    s[t] = gw * gw;
                } else {
                    s[t] = w * w;
                }
            }
            int best;
            float r;
            pc_score_taps(s, s_mask, la.P, score_mode, &best, &r);
            pid[row0 + c0 + tid] = (uint8_t)best;
            keys[c0 + tid] = pc_order_key(r);
        }
    }
    uint8_t *out = keep + row0;
    if (n_keep <= 0 || n_keep >= C) {
        for (int i = tid; i < C; i += T) out[i] = n_keep > 0 ? 1 : 0;
        return;
    }
    if (tid == 0) { s_prefix = 0u; s_remaining = n_keep; }
    const int lane = tid & 63, wave = tid >> 6;
    for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) hist[tid] = 0;
        __syncthreads();                        // also orders the keys / s_prefix writes before their readers
        const uint32_t prefix = s_prefix;
        const uint32_t himask = shift == 24 ? 0u : 0xFFFFFFFFu << (shift + 8);
        for (int i = tid; i < C; i += T) {
            const uint32_t k = keys[i];
            if ((k & himask) == prefix) atomicAdd(&hist[(k >> shift) & 255u], 1);
        }
        __syncthreads();
        if (wave == 0) {
            // lane l owns digits 4l..4l+3; hi = candidates with a digit above the lane's four
            const int h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
            const int mine = h0 + h1 + h2 + h3;
            int incl = mine;
            for (int off = 1; off < 64; off <<= 1) {
                const int t = __shfl_down(incl, off);
                if (lane + off < 64) incl += t;
            }
            const int rem = s_remaining;
            const int hi = incl - mine;
            // exactly one digit d has (candidates above d) < rem <= (candidates above d) + hist[d]
            const int e3 = hi, e2 = e3 + h3, e1 = e2 + h2, e0 = e1 + h1;
            int d = -1, ex = 0;
            if (e3 < rem && rem <= e3 + h3) { d = 3; ex = e3; }
            else if (e2 < rem && rem <= e2 + h2) { d = 2; ex = e2; }
            else if (e1 < rem && rem <= e1 + h1) { d = 1; ex = e1; }
            else if (e0 < rem && rem <= e0 + h0) { d = 0; ex = e0; }
            if (d >= 0) {
                s_prefix = prefix | ((uint32_t)(4 * lane + d) << shift);
                s_remaining = rem - ex;
            }
        }
        __syncthreads();
    }
    const uint32_t Tk = s_prefix;
    const int take_equal = s_remaining;         // kernels with key == Tk that are kept: the first ones by index
    const int nwaves = T >> 6;
    if (tid == 0) s_base = 0;
    __syncthreads();
    for (int i0 = 0; i0 < C; i0 += T) {
        const int i = i0 + tid;
        const uint32_t k = i < C ? keys[i] : 0u;
        const bool eq = i < C && k == Tk;
        const unsigned long long b = __ballot(eq);
        if (lane == 0) s_wave_cnt[wave] = __popcll(b);
        __syncthreads();
        int before = s_base + __popcll(b & ((1ull << lane) - 1ull));
        for (int w2 = 0; w2 < wave; ++w2) before += s_wave_cnt[w2];
        if (i < C) out[i] = (k > Tk || (eq && before < take_equal)) ? 1 : 0;
        __syncthreads();
        if (tid == 0) {
            int add = 0;
            for (int w2 = 0; w2 < nwaves; ++w2) add += s_wave_cnt[w2];
            s_base += add;
        }
        __syncthreads();
    }
}

__global__ void __launch_bounds__(512)
pc_select_row_kernel(const float *__restrict__ W, const float *__restrict__ G, int C, LibArg la, int score_mode,
                     int n_keep, uint8_t *__restrict__ pid, uint8_t *__restrict__ keep)
{
    pc_select_row_body(W, G, C, la, score_mode, n_keep, pid, keep, (int)blockIdx.x);
}

// The same for the filter rows of several layers in one launch: workgroup b serves row b - row0[l] of the layer l
// whose range holds b. Dynamic LDS is sized for the widest layer.
struct SelBatchArg {
    int32_t n, score_mode;
    int32_t row0[PC_BATCH_MAX + 1];
    int32_t C[PC_BATCH_MAX], n_keep[PC_BATCH_MAX];
    const float *W[PC_BATCH_MAX], *G[PC_BATCH_MAX];
    uint8_t *pid[PC_BATCH_MAX], *keep[PC_BATCH_MAX];
};

__global__ void __launch_bounds__(512) pc_select_rows_batch_kernel(SelBatchArg b, LibArg la)
{
    const int l = pc_batch_find(b.row0, b.n, (int)blockIdx.x);
    pc_select_row_body(b.W[l], b.G[l], b.C[l], la, b.score_mode, b.n_keep[l], b.pid[l], b.keep[l], (int)blockIdx.x - b.row0[l]);
}

// ---- exact top-n_keep of long segments (more than PC_TOPN_MAX scores): the same radix select across workgroups.
// Segment g has L scores; state per segment: hist[4][256] (zeroed first), then per-workgroup counts of the scores
// equal to the threshold. Pass q counts the digit (bits 31-8q .. 24-8q of the order-preserving key) of the
// scores whose higher digits equal the prefix chosen by the passes before; every workgroup derives that prefix
// again from the finished histograms (a 256-bin scan per pass) instead of reading it from a single writer.
#define PC_TOPN_CHUNK 2048      // scores per workgroup in the counting and writing kernels

// Wave 0 replays passes 0..upto-1: prefix and remaining count after them. All threads call it; ends with a barrier.
__device__ __forceinline__ void pc_topn_replay(const uint32_t *__restrict__ hist, int upto, int n_keep, uint32_t *s_prefix,
                                               int *s_rem)
{
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        uint32_t prefix = 0u;
        int rem = n_keep;
        for (int q = 0; q < upto; ++q) {
            const uint32_t *h = hist + q * 256 + 4 * lane;      // lane owns digits 4*lane .. 4*lane+3
            const int h0 = (int)h[0], h1 = (int)h[1], h2 = (int)h[2], h3 = (int)h[3];
            const int mine = h0 + h1 + h2 + h3;
            int incl = mine;
            for (int off = 1; off < 64; off <<= 1) {
                const int t = __shfl_down(incl, off);
                if (lane + off < 64) incl += t;
            }
            const int e3 = incl - mine, e2 = e3 + h3, e1 = e2 + h2, e0 = e1 + h1;   // candidates with a larger digit
            int d = -1, ex = 0;
            if (e3 < rem && rem <= e3 + h3) { d = 3; ex = e3; }
            else if (e2 < rem && rem <= e2 + h2) { d = 2; ex = e2; }
            else if (e1 < rem && rem <= e1 + h1) { d = 1; ex = e1; }
            else if (e0 < rem && rem <= e0 + h0) { d = 0; ex = e0; }
            const unsigned long long found = __ballot(d >= 0);  // exactly one lane while 1 <= rem <= candidates
            const int src = found ? __ffsll((long long)found) - 1 : 0;
            const int digit = __shfl(4 * lane + (d < 0 ? 0 : d), src);
            const int exs = __shfl(ex, src);
            prefix |= (uint32_t)digit << (24 - 8 * q);
            rem -= exs;
        }
        if (lane == 0) { *s_prefix = prefix; *s_rem = rem; }
    }
    __syncthreads();
}

__global__ void __launch_bounds__(256) pc_topn_zero_kernel(uint32_t *__restrict__ state, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) state[i] = 0u;
}

__global__ void __launch_bounds__(256)
pc_topn_hist_kernel(const float *__restrict__ R, int64_t L, int n_keep, uint32_t *__restrict__ hist_all, int pass)
{
    __shared__ int lh[256];
    __shared__ uint32_t s_prefix;
    __shared__ int s_rem;
    const float *seg = R + (int64_t)blockIdx.y * L;
    uint32_t *hist = hist_all + (int64_t)blockIdx.y * 1024;
    lh[threadIdx.x] = 0;
    pc_topn_replay(hist, pass, n_keep, &s_prefix, &s_rem);
    const uint32_t prefix = s_prefix;
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : 0xFFFFFFFFu << (shift + 8);
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < L; i += (int64_t)gridDim.x * 256) {
        const uint32_t k = pc_order_key(seg[i]);
        if ((k & himask) == prefix) atomicAdd(&lh[(k >> shift) & 255u], 1);
    }
    __syncthreads();
    if (lh[threadIdx.x]) atomicAdd(&hist[pass * 256 + threadIdx.x], (uint32_t)lh[threadIdx.x]);   // integers: order-free
}

// Scores equal to the threshold in every chunk of PC_TOPN_CHUNK scores.
__global__ void __launch_bounds__(256)
pc_topn_count_equal_kernel(const float *__restrict__ R, int64_t L, int n_keep, const uint32_t *__restrict__ hist_all,
                           uint32_t *__restrict__ blk_eq, int nchunks)
{
    __shared__ uint32_t s_prefix;
    __shared__ int s_rem, s_cnt[4];
    const float *seg = R + (int64_t)blockIdx.y * L;
    pc_topn_replay(hist_all + (int64_t)blockIdx.y * 1024, 4, n_keep, &s_prefix, &s_rem);
    const uint32_t T = s_prefix;
    const int64_t i0 = (int64_t)blockIdx.x * PC_TOPN_CHUNK;
    int cnt = 0;
    for (int j = threadIdx.x; j < PC_TOPN_CHUNK; j += 256)
        if (i0 + j < L && pc_order_key(seg[i0 + j]) == T) ++cnt;
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off);
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) blk_eq[(int64_t)blockIdx.y * nchunks + blockIdx.x] = (uint32_t)(s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3]);
}

// In-place exclusive scan of the chunk counts of every segment (one workgroup per segment).
__global__ void __launch_bounds__(256) pc_topn_scan_kernel(uint32_t *__restrict__ blk_eq, int nchunks)
{
    __shared__ uint32_t part[256];
    uint32_t *v = blk_eq + (int64_t)blockIdx.x * nchunks;
    const int per = (nchunks + 255) / 256;
    const int lo = threadIdx.x * per, hi = lo + per < nchunks ? lo + per : nchunks;
    uint32_t sum = 0;
    for (int i = lo; i < hi; ++i) sum += v[i];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {
        const uint32_t add = threadIdx.x >= d ? part[threadIdx.x - d] : 0u;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t run = part[threadIdx.x] - sum;
    for (int i = lo; i < hi; ++i) {
        const uint32_t c = v[i];
        v[i] = run;
        run += c;
    }
}

// keep = 1 for scores above the threshold and for the first take_equal scores equal to it (by index).
__global__ void __launch_bounds__(256)
pc_topn_write_kernel(const float *__restrict__ R, int64_t L, int n_keep, const uint32_t *__restrict__ hist_all,
                     const uint32_t *__restrict__ blk_excl, int nchunks, uint8_t *__restrict__ keep)
{
    __shared__ uint32_t s_prefix;
    __shared__ int s_rem, s_wave_cnt[4];
    const float *seg = R + (int64_t)blockIdx.y * L;
    uint8_t *out = keep + (int64_t)blockIdx.y * L;
    pc_topn_replay(hist_all + (int64_t)blockIdx.y * 1024, 4, n_keep, &s_prefix, &s_rem);
    const uint32_t T = s_prefix;
    const int take_equal = s_rem;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int base = (int)blk_excl[(int64_t)blockIdx.y * nchunks + blockIdx.x];
    const int64_t i0 = (int64_t)blockIdx.x * PC_TOPN_CHUNK;
    for (int j0 = 0; j0 < PC_TOPN_CHUNK; j0 += 256) {
        const int64_t i = i0 + j0 + threadIdx.x;
        const uint32_t k = i < L ? pc_order_key(seg[i]) : 0u;
        const bool eq = i < L && k == T;
        const unsigned long long b = __ballot(eq);
        if (lane == 0) s_wave_cnt[wave] = __popcll(b);
        __syncthreads();
        int before = base + __popcll(b & ((1ull << lane) - 1ull));
        for (int w2 = 0; w2 < wave; ++w2) before += s_wave_cnt[w2];
        if (i < L) out[i] = (k > T || (eq && before < take_equal)) ? 1 : 0;
        base += s_wave_cnt[0] + s_wave_cnt[1] + s_wave_cnt[2] + s_wave_cnt[3];
        __syncthreads();
    }
}

__global__ void __launch_bounds__(256) pc_fill_u8_kernel(uint8_t *__restrict__ p, int64_t n, uint8_t v)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}

pc_status pc_launch_select(pc_ctx *ctx, const float *W, const float *G, int F, int C, const LibArg &la,
                           pc_keep_mode km, int64_t n_keep, pc_score_mode sm, uint8_t *pid, uint8_t *keep)
{
    int64_t nk = (int64_t)F * C;
    if (km == PC_KEEP_PER_FILTER && C <= PC_TOPN_MAX) {
        const int T = C <= 256 ? 256 : 512;
        const size_t lds = sizeof(uint32_t) * (size_t)C + 2 * sizeof(float) * 9 * (size_t)T;   // at most 68 KiB
        static pc_per_device_once attr;
        if (pc_once_pending(attr, ctx->device)) {
            PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_select_row_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)(sizeof(uint32_t) * PC_TOPN_MAX + 2 * sizeof(float) * 9 * 512)));
            pc_once_done(attr, ctx->device);
        }
        const int nk_row = (int)(n_keep < C ? n_keep : C);
        hipLaunchKernelGGL(pc_select_row_kernel, dim3((unsigned)F), dim3((unsigned)T), lds, ctx->stream, W, G, C, la, (int)sm,
                           nk_row, pid, keep);
        return pc_hip_check(ctx, hipGetLastError(), "select launch");
    }
    const int64_t L = (km == PC_KEEP_PER_FILTER) ? C : nk;
    const unsigned nseg = (km == PC_KEEP_PER_FILTER) ? (unsigned)F : 1u;
    if (L >= ((int64_t)1 << 31)) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "select: %lld scores in one segment (limit 2^31 - 1)", (long long)L);
    const int nchunks = (int)((L + PC_TOPN_CHUNK - 1) / PC_TOPN_CHUNK);
    const size_t r_bytes = (sizeof(float) * (size_t)nk + 255) / 256 * 256;
    const size_t state_words = L > PC_TOPN_MAX ? (size_t)nseg * (1024 + (size_t)nchunks) : 0;
    void *scr = nullptr;
    pc_status s = pc_scratch(ctx, r_bytes + sizeof(uint32_t) * state_words, &scr);
    if (s != PC_OK) return s;
    float *R = (float *)scr;
    unsigned blocks = (unsigned)((nk + 255) / 256);
    hipLaunchKernelGGL(pc_select_score_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, G, nk, la, (int)sm, pid, R);
    if (L <= PC_TOPN_MAX) {
        hipLaunchKernelGGL(pc_select_topn_row_kernel, dim3(nseg), dim3(256), sizeof(uint32_t) * (size_t)L, ctx->stream, R, (int)L,
                           (int)(n_keep < L ? n_keep : L), keep);
    } else if (n_keep <= 0 || n_keep >= L) {
        hipLaunchKernelGGL(pc_fill_u8_kernel, dim3(blocks), dim3(256), 0, ctx->stream, keep, nk, (uint8_t)(n_keep > 0 ? 1 : 0));
    } else {
        uint32_t *hist = reinterpret_cast<uint32_t *>(static_cast<unsigned char *>(scr) + r_bytes);
        uint32_t *blk_eq = hist + (size_t)nseg * 1024;
        hipLaunchKernelGGL(pc_topn_zero_kernel, dim3((unsigned)((nseg * 1024 + 255) / 256)), dim3(256), 0, ctx->stream, hist,
                           (int64_t)nseg * 1024);
        int hb = (int)((L + 255) / 256);
        const int hb_max = nseg >= 64 ? 8 : 4 * ctx->num_cu;     // workgroups per segment in the counting passes
        if (hb > hb_max) hb = hb_max;
        for (int pass = 0; pass < 4; ++pass)
            hipLaunchKernelGGL(pc_topn_hist_kernel, dim3((unsigned)hb, nseg), dim3(256), 0, ctx->stream, R, L, (int)n_keep, hist, pass);
        hipLaunchKernelGGL(pc_topn_count_equal_kernel, dim3((unsigned)nchunks, nseg), dim3(256), 0, ctx->stream, R, L, (int)n_keep,
                           hist, blk_eq, nchunks);
        hipLaunchKernelGGL(pc_topn_scan_kernel, dim3(nseg), dim3(256), 0, ctx->stream, blk_eq, nchunks);
        hipLaunchKernelGGL(pc_topn_write_kernel, dim3((unsigned)nchunks, nseg), dim3(256), 0, ctx->stream, R, L, (int)n_keep, hist,
                           blk_eq, nchunks, keep);
    }
    return pc_hip_check(ctx, hipGetLastError(), "select launch");
}

// Layers whose rows fit the one-workgroup kernel go into launches of up to PC_BATCH_MAX layers; the others are
// served one by one by pc_launch_select.
pc_status pc_launch_select_batch(pc_ctx *ctx, int n, const float *const *W, const float *const *G, const int32_t *F,
                                 const int32_t *C, const LibArg &la, pc_keep_mode km, const int64_t *n_keep, pc_score_mode sm,
                                 uint8_t *const *pid, uint8_t *const *keep)
{
    static pc_per_device_once attr;
    if (pc_once_pending(attr, ctx->device)) {
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_select_rows_batch_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)(sizeof(uint32_t) * PC_TOPN_MAX + 2 * sizeof(float) * 9 * 512)));
        pc_once_done(attr, ctx->device);
    }
    SelBatchArg b;
    memset(&b, 0, sizeof(b));
    b.score_mode = (int)sm;
    int cmax = 0;
    auto flush = [&]() -> pc_status {
        if (b.n == 0) return PC_OK;
        const int T = cmax <= 256 ? 256 : 512;
        const size_t lds = sizeof(uint32_t) * (size_t)cmax + 2 * sizeof(float) * 9 * (size_t)T;
        hipLaunchKernelGGL(pc_select_rows_batch_kernel, dim3((unsigned)b.row0[b.n]), dim3((unsigned)T), lds, ctx->stream, b, la);
        b.n = 0;
        cmax = 0;
        return pc_hip_check(ctx, hipGetLastError(), "select (several layers) launch");
    };
    for (int l = 0; l < n; ++l) {
        if (km != PC_KEEP_PER_FILTER || C[l] > PC_TOPN_MAX) {
            pc_status s = pc_launch_select(ctx, W[l], G ? G[l] : nullptr, F[l], C[l], la, km, n_keep[l], sm, pid[l], keep[l]);
            if (s != PC_OK) return s;
            continue;
        }
        const int i = b.n;
        b.W[i] = W[l]; b.G[i] = G ? G[l] : nullptr; b.C[i] = C[l];
        b.n_keep[i] = (int32_t)(n_keep[l] < C[l] ? n_keep[l] : C[l]);
        b.pid[i] = pid[l]; b.keep[i] = keep[l];
        b.row0[i + 1] = b.row0[i] + F[l];
        if (C[l] > cmax) cmax = C[l];
        if (++b.n == PC_BATCH_MAX) {
            pc_status s = flush();
            if (s != PC_OK) return s;
        }
    }
    return flush();
}

// ------------------------------------------------------------------ packing
// Table rows are filters (row stride C, element stride 1 in the [F][C] maps) for the
// filter-major table, channels (row stride 1, element stride C) for the channel-major one.
//
// A pack is two launches. The first counts the kept kernels of every table row per pattern id and, for the
// matrix-core variant, writes the operand tiles (they depend on W and the masks only). The second places the
// kernels: every workgroup adds up the totals of the rows before its own, so no separate scan is needed.

// Kept kernels of one row, per pattern id, and their total.
__device__ __forceinline__ void pc_pack_count_row(const uint8_t *__restrict__ pid, const uint8_t *__restrict__ keep, int row,
                                                  int len, int64_t row_stride, int64_t elem_stride, int P,
                                                  int32_t *__restrict__ grp, int32_t *__restrict__ rowtot)
{
    __shared__ int hist[PC_MAX_P + 1];
    for (int p = threadIdx.x; p <= PC_MAX_P; p += blockDim.x) hist[p] = 0;
    __syncthreads();
    for (int e = threadIdx.x; e < len; e += blockDim.x) {
        int64_t k = row * row_stride + e * elem_stride;
        const int kp = keep[k], pd = pid[k];                      // both loads at once, not one behind the other
        if (kp && pd < P) atomicAdd(&hist[pd], 1);                // integer counts: order does not matter
    }
    __syncthreads();
    for (int p = threadIdx.x; p < P; p += blockDim.x) grp[(int64_t)row * (PC_MAX_P + 1) + p] = hist[p];
    if (threadIdx.x < 64) {
        int tot = 0;
        for (int p = threadIdx.x; p < P; p += 64) tot += hist[p];
        for (int off = 32; off > 0; off >>= 1) tot += __shfl_down(tot, off);
        if (threadIdx.x == 0) rowtot[row] = tot;
    }
}

// Operand tiles of one 32-filter x 32-channel block, all 9 taps.
// wz_fwd[mt][tap][ks][lane][8]: mt = filter/32, ks = channel/16; element i of lane l is
// w[f = 32*mt + l%32][c = 16*ks + 8*(l/32) + i][tap] as bf16, zero when pruned or padded.
// wz_bwd has the roles of filter and channel exchanged (rows = channels, k = filters).
// The pattern mask of a kernel comes from pid/keep, or (FROM_KINFO) from the kinfo table of an earlier pack.
#define PC_TILE_PITCH 40   // bf16 elements per LDS row: 32 + 8 keeps 16-byte alignment and spreads the banks

// 16 consecutive reduction entries of one row (bf16 bit patterns) as operands of the structured-sparse matrix
// instruction: for each of the 4 groups of 4 entries, part 1 stores the first two nonzeros and part 2 the third and
// fourth (stored value 2g + m of a part belongs to group g; an unused place holds zero), idx their 2-bit positions in
// the group: bits [4g+1:4g] and [4g+3:4g+2] for part 1, the same 16 bits higher for part 2. A place without a
// nonzero points at a position none of the part's nonzeros uses.
// ovf_pos / ovf_val (may be null): the up to 8 overflow weights (third and fourth nonzeros of a group) with their
// positions 0..15, *n_ovf their count.
__device__ __forceinline__ void pc_sparse_compress16(const uint16_t *src, uint4 *part1, uint4 *part2, uint32_t *idx,
                                                     uint32_t *ovf_pos, uint32_t *ovf_val, int *n_ovf)
{
    int no = 0;
    uint32_t w1[4] = {0u, 0u, 0u, 0u}, w2[4] = {0u, 0u, 0u, 0u};
    uint32_t ix = 0u;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        // values and positions of the nonzeros of the group, in ascending position
        uint32_t val[4] = {0u, 0u, 0u, 0u}, pos[4] = {0u, 0u, 0u, 0u};
        int n = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint32_t u = src[4 * g + e];
            if (u & 0x7FFFu) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (k == n) { val[k] = u; pos[k] = (uint32_t)e; }
                ++n;
            }
        }
#pragma unroll
        for (int k = 2; k < 4; ++k)
            if (k < n) {
#pragma unroll
                for (int q = 0; q < 8; ++q)
                    if (q == no) { ovf_pos[q] = 4u * g + pos[k]; ovf_val[q] = val[k]; }
                ++no;
            }
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            const int m = n - 2 * part;                 // nonzeros left for this part
            uint32_t a = 0u, b = 0u, pa = 0u, pb = 1u;  // none: zeros at positions 0 and 1
            if (m >= 2) { a = val[2 * part]; b = val[2 * part + 1]; pa = pos[2 * part]; pb = pos[2 * part + 1]; }
            else if (m == 1) {
                const uint32_t p = pos[2 * part], x = val[2 * part];
                if (p < 3u) { a = x; pa = p; pb = 3u; } else { b = x; pa = 0u; pb = 3u; }
            }
            (part ? w2 : w1)[g] = a | (b << 16);
            ix |= (pa | (pb << 2)) << (4 * g + 16 * part);
        }
    }
    *part1 = make_uint4(w1[0], w1[1], w1[2], w1[3]);
    *part2 = make_uint4(w2[0], w2[1], w2[2], w2[3]);
    *idx = ix;
    *n_ovf = no;
}
template <bool FROM_KINFO>
__device__ __forceinline__ void pc_pack_tile_block(const float *__restrict__ W, const uint8_t *__restrict__ pid,
                                                   const uint8_t *__restrict__ keep, const LibArg &la, const PackView &v,
                                                   int fb, int cb)
{
    __shared__ __align__(16) uint16_t tA[9][32][PC_TILE_PITCH];   // [tap][filter][channel]
    __shared__ __align__(16) uint16_t tB[9][32][PC_TILE_PITCH];   // [tap][channel][filter]
    __shared__ uint16_t tm[32][32];                               // pattern mask of kernel (f,c), 0 = pruned / outside
    __shared__ uint16_t lm[PC_MAX_P + 2];                         // the pool's masks
    const int tid = threadIdx.x, f0 = fb * 32, c0 = cb * 32;
    if (!FROM_KINFO) {
        if (tid < la.P) lm[tid] = la.mask[tid];
        uint8_t kp[4], pd[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = j * 256 + tid, f = f0 + (i >> 5), c = c0 + (i & 31);
            const bool in = f < v.F && c < v.C;
            const int64_t k = in ? (int64_t)f * v.C + c : 0;
            kp[j] = in ? keep[k] : (uint8_t)0;
            pd[j] = pid[k];
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = j * 256 + tid;
            tm[i >> 5][i & 31] = (kp[j] && pd[j] < la.P) ? lm[pd[j]] : (uint16_t)0;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int i = j * 256 + tid, f = f0 + (i >> 5), c = c0 + (i & 31);
            uint32_t u = 0xFFFFFFFFu;
            if (f < v.F && c < v.C) u = v.kinfo[(int64_t)f * v.C + c];
            tm[i >> 5][i & 31] = u == 0xFFFFFFFFu ? (uint16_t)0 : (uint16_t)(u & 511u);
        }
    }
    __syncthreads();
    const int ncols = v.C - c0 < 32 ? (v.C - c0 > 0 ? v.C - c0 : 0) : 32;
    if ((v.C & 3) == 0 && (reinterpret_cast<uintptr_t>(W) & 15) == 0) {
        // a filter row of the block is ncols*9 contiguous floats starting on a 16-byte boundary
        const int nq = ncols * 9 / 4;
        // all 9 loads of the thread are issued before the first value is used: one memory round trip, not nine
        float4 wq[9];
#pragma unroll
        for (int it = 0; it < 9; ++it) {
            const int q = it * 256 + tid;            // 32 rows x 72 quads
            const int r = q / 72, jq = q - r * 72;
            wq[it] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (f0 + r < v.F && jq < nq)
                wq[it] = *reinterpret_cast<const float4 *>(W + ((int64_t)(f0 + r) * v.C + c0) * 9 + jq * 4);
        }
#pragma unroll
        for (int it = 0; it < 9; ++it) {
            const int q = it * 256 + tid;
            const int r = q / 72, jq = q - r * 72;
            const float4 w4 = wq[it];
            const float wv[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = jq * 4 + e, cl = j / 9, tap = j - cl * 9;
                const uint16_t val = ((tm[r][cl] >> tap) & 1u) ? pc_f32_to_bf16(wv[e]) : (uint16_t)0;
                tA[tap][r][cl] = val;
                tB[tap][cl][r] = val;
            }
        }
    } else {
        for (int idx = tid; idx < 32 * 288; idx += 256) {
            const int r = idx / 288, j = idx - r * 288, cl = j / 9, tap = j - cl * 9;
            uint16_t val = 0;
            if (f0 + r < v.F && cl < ncols && ((tm[r][cl] >> tap) & 1u))
                val = pc_f32_to_bf16(W[((int64_t)(f0 + r) * v.C + c0 + cl) * 9 + tap]);
            tA[tap][r][cl] = val;
            tB[tap][cl][r] = val;
        }
    }
    __shared__ uint32_t lflag[2];
    __shared__ uint32_t ocnt[2];                     // overflow weights of this block, forward / backward-data orientation
    __shared__ uint2 oent[2][PC_OV_SUB];
    if (tid < 2) { lflag[tid] = 0u; ocnt[tid] = 0u; }
    __syncthreads();
    const int KSf = v.Ck / 16, KSb = v.Fk / 16;
    uint4 *of = reinterpret_cast<uint4 *>(v.wz_fwd), *ob = reinterpret_cast<uint4 *>(v.wz_bwd);
    for (int o = tid; o < 9 * 2 * 64; o += 256) {
        const int lane = o & 63, q = o >> 6, tap = q >> 1, sl = q & 1;
        const int row = lane & 31, col = 16 * sl + 8 * (lane >> 5);
        if (2 * cb + sl < KSf)
            of[((int64_t)(fb * 9 + tap) * KSf + 2 * cb + sl) * 64 + lane] = *reinterpret_cast<const uint4 *>(&tA[tap][row][col]);
        if (2 * fb + sl < KSb)
            ob[((int64_t)(cb * 9 + tap) * KSb + 2 * fb + sl) * 64 + lane] = *reinterpret_cast<const uint4 *>(&tB[tap][row][col]);
    }
    // The operands of the structured-sparse instruction: this block is one step of 32 reduction entries of row tile fb
    // (forward) and of row tile cb (backward-data). Lane l of a fragment holds row l % 32 and the entries
    // 16 * (l / 32) .. + 15 of the step.
    if (!v.ws_fwd_val) return;            // uniform: only packs made for the structured-sparse kernel hold these
    const int KS32f = v.Ck / 32, KS32b = v.Fk / 32;
    for (int o = tid; o < 2 * 9 * 64; o += 256) {
        const int lane = o & 63, q = o >> 6, tap = q % 9, bwd = q / 9;
        const int rt = bwd ? cb : fb, ss = bwd ? fb : cb;
        if (ss >= (bwd ? KS32b : KS32f)) continue;
        const uint16_t *src = bwd ? &tB[tap][lane & 31][16 * (lane >> 5)] : &tA[tap][lane & 31][16 * (lane >> 5)];
        uint4 p1, p2;
        uint32_t idx, opos[8], oval[8];
        int no;
        pc_sparse_compress16(src, &p1, &p2, &idx, opos, oval, &no);
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (q < no) {
                const uint32_t at = atomicAdd(&ocnt[bwd], 1u);
                if (at < PC_OV_SUB)
                    oent[bwd][at] = make_uint2(((uint32_t)tap << 11) | ((uint32_t)(lane & 31) << 6) | (16u * (lane >> 5) + opos[q]), oval[q]);
            }
        const int64_t fr = (int64_t)(rt * 9 + tap) * (bwd ? KS32b : KS32f) + ss;
        uint4 *ov = reinterpret_cast<uint4 *>(bwd ? v.ws_bwd_val : v.ws_fwd_val);
        ov[(fr * 2 + 0) * 64 + lane] = p1;
        ov[(fr * 2 + 1) * 64 + lane] = p2;
        (bwd ? v.ws_bwd_idx : v.ws_fwd_idx)[fr * 64 + lane] = idx;
        if (p2.x | p2.y | p2.z | p2.w) atomicOr(&lflag[bwd], 1u << tap);
    }
    __syncthreads();
    if (tid == 0 && cb < KS32f) v.ws_fwd_flag[(int64_t)fb * KS32f + cb] = (uint16_t)lflag[0];
    if (tid == 1 && fb < KS32b) v.ws_bwd_flag[(int64_t)cb * KS32b + fb] = (uint16_t)lflag[1];
    // The block's overflow weights, in the order of their keys (tap, row, entry): the order the atomic counter gave
    // them is not reproducible, their rank among the keys is. A list that does not fit only leaves its count.
    if (tid < 2 * PC_OV_SUB) {
        const int bwd = tid / PC_OV_SUB, e = tid % PC_OV_SUB;
        const int rt = bwd ? cb : fb, ss = bwd ? fb : cb;
        const int n = (int)ocnt[bwd];
        if (ss < (bwd ? KS32b : KS32f)) {
            const int64_t sub = (int64_t)rt * (bwd ? KS32b : KS32f) + ss;
            if (e == 0) (bwd ? v.ov_bwd_sub_cnt : v.ov_fwd_sub_cnt)[sub] = (uint32_t)n;
            if (e < n && n <= PC_OV_SUB) {
                const uint2 mine = oent[bwd][e];
                int rank = 0;
                for (int q = 0; q < n; ++q) rank += oent[bwd][q].x < mine.x;
                (bwd ? v.ov_bwd_sub_ent : v.ov_fwd_sub_ent)[sub * PC_OV_SUB + rank] = mine;
            }
        }
    }
}

// Merges the overflow lists of the two 32 x 32 blocks of a (row tile, 64-entry chunk) pair into the steps the
// structured-sparse kernel multiplies: list = blockIdx (forward lists first), 64 threads.
__device__ __forceinline__ void pc_pack_ovf_merge_body(const PackView &v, int list)
{
    __shared__ uint2 ent[2 * PC_OV_SUB];
    const int nf = (v.Fp / 32) * (v.Ck / 64);
    const bool bwd = list >= nf;
    const int l = bwd ? list - nf : list;
    const uint32_t *scnt = bwd ? v.ov_bwd_sub_cnt : v.ov_fwd_sub_cnt;
    const uint2 *sent = bwd ? v.ov_bwd_sub_ent : v.ov_fwd_sub_ent;
    uint32_t *cnt = bwd ? v.ov_bwd_cnt : v.ov_fwd_cnt;
    uint4 *oa = reinterpret_cast<uint4 *>(bwd ? v.ov_bwd_a : v.ov_fwd_a);
    uint32_t *ocol = bwd ? v.ov_bwd_col : v.ov_fwd_col;
    // sub-lists 2l and 2l + 1: the chunk's two steps of 32 entries ([rt][ss] with ss = 2 * chunk + half)
    const uint32_t n0 = scnt[2 * (int64_t)l], n1 = scnt[2 * (int64_t)l + 1];
    const int tid = threadIdx.x;
    if (n0 > PC_OV_SUB || n1 > PC_OV_SUB) {
        if (tid == 0) cnt[l] = PC_OV_BAD;
        return;
    }
    const int n = (int)(n0 + n1);
    if (tid < n) {
        const int half = tid >= (int)n0;
        uint2 e = sent[(2 * (int64_t)l + half) * PC_OV_SUB + (half ? tid - (int)n0 : tid)];
        e.x += half ? 32u : 0u;                      // entry inside the chunk
        ent[tid] = e;
    }
    __syncthreads();
    const int steps = (n + 15) / 16;
    if (tid == 0) cnt[l] = (uint32_t)steps;
    const int row = tid & 31, g = tid >> 5;
    // (the first step is always written: the kernel multiplies it without looking at the count)
    for (int s = 0; s < (steps > 1 ? steps : 1); ++s) {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int q = s * 16 + 8 * g + e;
            if (q < n) {
                const uint2 en = ent[q];
                if ((int)((en.x >> 6) & 31u) == row) w[e >> 1] |= (en.y & 0xFFFFu) << ((e & 1) * 16);
            }
        }
        oa[((int64_t)l * PC_OV_STEPS + s) * 64 + tid] = make_uint4(w[0], w[1], w[2], w[3]);
        if (tid < 16) {
            const int q = s * 16 + tid;
            uint32_t c = 0u;                         // unused columns: tap 0, entry 0 (a valid address; their weights are 0)
            if (q < n) {
                const uint32_t key = ent[q].x, tap = key >> 11;
                c = ((tap / 3u) << 12) | ((tap % 3u) << 8) | (key & 63u);
            }
            ocol[((int64_t)l * PC_OV_STEPS + s) * 16 + tid] = c;
        }
    }
}

__global__ void __launch_bounds__(64) pc_pack_ovf_merge_kernel(PackView v) { pc_pack_ovf_merge_body(v, (int)blockIdx.x); }


// First launch of a pack: workgroups [0, F) count the filter rows, [F, F + ncm) the channel rows (ncm = C for the
// gather variant, else 0), the rest write the operand tiles (matrix-core variant), one 32 x 32 block each.
__device__ __forceinline__ void pc_pack_stage1_body(const float *__restrict__ W, const uint8_t *__restrict__ pid,
                                                    const uint8_t *__restrict__ keep, const LibArg &la, const PackView &v, int ncm,
                                                    int tiles_c, int b)
{
    if (b < v.F) {
        pc_pack_count_row(pid, keep, b, v.C, (int64_t)v.C, 1, v.P, v.fm_grp, v.fm_rowtot);
        return;
    }
    b -= v.F;
    if (b < ncm) {
        pc_pack_count_row(pid, keep, b, v.F, 1, (int64_t)v.C, v.P, v.cm_grp, v.cm_rowtot);
        return;
    }
    b -= ncm;
    pc_pack_tile_block<false>(W, pid, keep, la, v, b / tiles_c, b % tiles_c);
}

__global__ void __launch_bounds__(256)
pc_pack_stage1_kernel(const float *__restrict__ W, const uint8_t *__restrict__ pid, const uint8_t *__restrict__ keep,
                      LibArg la, PackView v, int ncm, int tiles_c)
{
    pc_pack_stage1_body(W, pid, keep, la, v, ncm, tiles_c, (int)blockIdx.x);
}

// Several packs per launch: workgroup b serves block b - blk0[l] of pack l. The packs' views are read from their
// device copies (the pool is the launch's, so its size replaces the view's).
struct PackBatchArg {
    int32_t n;
    int32_t blk0[PC_BATCH_MAX + 1];
    const float *W[PC_BATCH_MAX];
    const uint8_t *pid[PC_BATCH_MAX], *keep[PC_BATCH_MAX];
    const PackView *view[PC_BATCH_MAX];
    int32_t ncm[PC_BATCH_MAX], tiles_c[PC_BATCH_MAX], bf16[PC_BATCH_MAX];
};

__global__ void __launch_bounds__(256) pc_pack_stage1_batch_kernel(PackBatchArg b, LibArg la)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    PackView v = *b.view[l];
    v.P = la.P;
    pc_pack_stage1_body(b.W[l], b.pid[l], b.keep[l], la, v, b.ncm[l], b.tiles_c[l], (int)blockIdx.x - b.blk0[l]);
}

// The 4 kept weights of kernel k; taps holds the 4 tap indices, one per byte, ascending from the low byte.
__device__ __forceinline__ float4 pc_gather_taps(const float *__restrict__ W, int64_t k, uint32_t taps, bool bf16)
{
    float v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float w = W[k * 9 + ((taps >> (8 * j)) & 255u)];
        v[j] = bf16 ? pc_bf16_to_f32(pc_f32_to_bf16(w)) : w;
    }
    return make_float4(v[0], v[1], v[2], v[3]);
}

__device__ __forceinline__ uint32_t pc_taps_word(const LibArg &la, int p)
{
    return (uint32_t)la.taps[p][0] | ((uint32_t)la.taps[p][1] << 8) | ((uint32_t)la.taps[p][2] << 16) | ((uint32_t)la.taps[p][3] << 24);
}

// Values again from new weights with unchanged tables, one launch for the matrix-core variant: workgroups
// [0, ntiles) rebuild the operand tiles (masks from the kinfo table), the others re-gather the compact values.
__device__ __forceinline__ void pc_pack_revalue_body(const float *__restrict__ W, const LibArg &la, int bf16, const PackView &v,
                                                     int tiles_c, int ntiles, int b)
{
    if (b < ntiles) {
        pc_pack_tile_block<true>(W, nullptr, nullptr, la, v, b / tiles_c, b % tiles_c);
        return;
    }
    const int64_t k = (int64_t)(b - ntiles) * 256 + threadIdx.x;
    if (k >= (int64_t)v.F * v.C) return;
    const uint32_t u = v.kinfo[k];
    if (u == 0xFFFFFFFFu) return;
    const int slot = (int)(u >> 9);
    v.fm_val[slot] = pc_gather_taps(W, k, pc_taps_word(la, v.fm_pid[slot]), bf16 != 0);
}

__global__ void __launch_bounds__(256)
pc_pack_revalue_kernel(const float *__restrict__ W, LibArg la, int bf16, PackView v, int tiles_c, int ntiles)
{
    pc_pack_revalue_body(W, la, bf16, v, tiles_c, ntiles, (int)blockIdx.x);
}

// Value update of several matrix-core packs (ncm holds the tile count of pack l here; the pool's tap lists are
// those of the pool the packs were made with).
__global__ void __launch_bounds__(256) pc_pack_revalue_batch_kernel(PackBatchArg b, LibArg la)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    PackView v = *b.view[l];
    v.P = la.P;
    pc_pack_revalue_body(b.W[l], la, b.bf16[l], v, b.tiles_c[l], b.ncm[l], (int)blockIdx.x - b.blk0[l]);
}

// Places the kept kernels of one row at (kept kernels of the rows before) + (pattern group start) + (rank inside
// the group); the rank of an element is the number of earlier members of its group in the row, so the order
// inside a group is ascending. The row is walked 256 elements at a time: every wave ballots each pattern id,
// the per-wave counts go through LDS. All counts are integers, so no result depends on an execution order.
template <bool FM>
__device__ __forceinline__ void pc_pack_place_body(const float *__restrict__ W, const uint8_t *__restrict__ pid,
                                                   const uint8_t *__restrict__ keep, int rows, int len, int64_t row_stride,
                                                   int64_t elem_stride, const LibArg &la, int bf16, const PackView &v, int row)
{
    __shared__ int start[PC_MAX_P + 1];          // next free slot of every pattern group
    __shared__ int wcnt[4][PC_MAX_P + 2];        // members of every group in the current 256 elements, per wave
    __shared__ int red[4];
    __shared__ uint32_t ltaps[PC_MAX_P + 2];      // tap lists and masks of the pool
    __shared__ uint16_t lmask[PC_MAX_P + 2];
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int P = la.P;
    if (tid < P) { ltaps[tid] = pc_taps_word(la, tid); lmask[tid] = la.mask[tid]; }
    int32_t *grp = (FM ? v.fm_grp : v.cm_grp) + (int64_t)row * (PC_MAX_P + 1);
    int32_t *rowptr = FM ? v.fm_rowptr : v.cm_rowptr;
    const int32_t *rowtot = FM ? v.fm_rowtot : v.cm_rowtot;
    // kept kernels in the rows before this one
    int part = 0;
    for (int i = tid; i < row; i += 256) part += rowtot[i];
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off);
    if (lane == 0) red[wave] = part;
    if (tid < P) start[tid] = grp[tid];          // counts for now
    __syncthreads();
    const int base = red[0] + red[1] + red[2] + red[3];
    if (tid == 0) {
        rowptr[row] = base;
        if (row == rows - 1) rowptr[rows] = base + rowtot[row];
        int run = base;
        for (int p = 0; p < P; ++p) {
            const int cnt = start[p];
            start[p] = run;
            run += cnt;
        }
        start[P] = run;
    }
    __syncthreads();
    if (tid <= P) grp[tid] = start[tid];         // group starts, [P] = row end
    for (int e0 = 0; e0 < len; e0 += 256) {
        const int e = e0 + tid;
        const int64_t k = row * row_stride + e * elem_stride;
        int code = 255;
        if (e < len) {
            const int kp = keep[k], pd = pid[k];
            if (kp && pd < P) code = pd;
        }
        int my_rank = 0, c0 = 0, c1 = 0;
        for (int p = 0; p < P; ++p) {
            const unsigned long long b = __ballot(code == p);
            if (code == p) my_rank = __popcll(b & ((1ull << lane) - 1ull));
            const int n = __popcll(b);
            if (lane == (p & 63)) { if (p < 64) c0 = n; else c1 = n; }
        }
        if (lane < P) wcnt[wave][lane] = c0;
        if (lane + 64 < P) wcnt[wave][lane + 64] = c1;
        __syncthreads();
        if (code != 255) {
            int slot = start[code] + my_rank;
            for (int w2 = 0; w2 < wave; ++w2) slot += wcnt[w2][code];
            const float4 val = pc_gather_taps(W, k, ltaps[code], bf16 != 0);
            if (FM) {
                v.fm_c[slot] = (uint16_t)e;
                v.fm_pid[slot] = (uint8_t)code;
                v.slot_f[slot] = (uint16_t)row;
                v.fm_val[slot] = val;
                v.slot_of[k] = slot;
                if (v.kinfo) v.kinfo[k] = ((uint32_t)slot << 9) | lmask[code];
            } else {
                v.cm_f[slot] = (uint16_t)e;
                v.cm_slot[slot] = v.slot_of[k];
                v.cm_val[slot] = val;
            }
        } else if (FM && e < len) {
            v.slot_of[k] = -1;
            if (v.kinfo) v.kinfo[k] = 0xFFFFFFFFu;
        }
        __syncthreads();
        if (tid < P) start[tid] += wcnt[0][tid] + wcnt[1][tid] + wcnt[2][tid] + wcnt[3][tid];
        __syncthreads();
    }
}

template <bool FM>
__global__ void __launch_bounds__(256)
pc_pack_place_kernel(const float *__restrict__ W, const uint8_t *__restrict__ pid, const uint8_t *__restrict__ keep,
                     int rows, int len, int64_t row_stride, int64_t elem_stride, LibArg la, int bf16, PackView v)
{
    pc_pack_place_body<FM>(W, pid, keep, rows, len, row_stride, elem_stride, la, bf16, v, (int)blockIdx.x);
}

template <bool FM> __global__ void __launch_bounds__(256) pc_pack_place_batch_kernel(PackBatchArg b, LibArg la)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    PackView v = *b.view[l];
    v.P = la.P;
    const int row = (int)blockIdx.x - b.blk0[l];
    if constexpr (FM) pc_pack_place_body<true>(b.W[l], b.pid[l], b.keep[l], v.F, v.C, (int64_t)v.C, (int64_t)1, la, b.bf16[l], v, row);
    else pc_pack_place_body<false>(b.W[l], b.pid[l], b.keep[l], v.C, v.F, (int64_t)1, (int64_t)v.C, la, b.bf16[l], v, row);
}

// Re-gathers values with unchanged tables (one thread per kernel (f,c)).
__global__ void __launch_bounds__(256)
pc_pack_regather_fm_kernel(const float *__restrict__ W, LibArg la, int bf16, PackView v)
{
    int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= (int64_t)v.F * v.C) return;
    int slot = v.slot_of[k];
    if (slot < 0) return;
    v.fm_val[slot] = pc_gather_taps(W, k, pc_taps_word(la, v.fm_pid[slot]), bf16 != 0);
}

__global__ void __launch_bounds__(256) pc_pack_regather_cm_kernel(PackView v)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= v.cm_rowptr[v.C]) return;
    v.cm_val[i] = v.fm_val[v.cm_slot[i]];
}

// The overflow lists of a pack made for the structured-sparse kernel (no-op for other packs).
static int pc_ovf_lists(const PackView &v) { return v.ov_fwd_cnt ? (v.Fp / 32) * (v.Ck / 64) + (v.Cp / 32) * (v.Fk / 64) : 0; }
static void pc_launch_ovf_merge(pc_ctx *ctx, const PackView &v)
{
    const int n = pc_ovf_lists(v);
    if (n > 0) hipLaunchKernelGGL(pc_pack_ovf_merge_kernel, dim3((unsigned)n), dim3(64), 0, ctx->stream, v);
}

// The same for several packs in one launch.
__global__ void __launch_bounds__(64) pc_pack_ovf_merge_batch_kernel(PackBatchArg b)
{
    const int l = pc_batch_find(b.blk0, b.n, (int)blockIdx.x);
    pc_pack_ovf_merge_body(*b.view[l], (int)blockIdx.x - b.blk0[l]);
}

static void pc_launch_ovf_merge_batch(pc_ctx *ctx, int m, pc_packed *const *pk)
{
    PackBatchArg a;
    memset(&a, 0, sizeof(a));
    a.n = m;
    for (int i = 0; i < m; ++i) {
        a.view[i] = pk[i]->v_dev;
        a.blk0[i + 1] = a.blk0[i] + pc_ovf_lists(pk[i]->v);
    }
    if (a.blk0[m] > 0) hipLaunchKernelGGL(pc_pack_ovf_merge_batch_kernel, dim3((unsigned)a.blk0[m]), dim3(64), 0, ctx->stream, a);
}

pc_status pc_launch_pack(pc_ctx *ctx, pc_packed *pk, const float *W, const uint8_t *pid, const uint8_t *keep)
{
    PackView v = pk->v;
    LibArg la;
    pc_fill_lib(&la, pk->lib, v.P);
    int bf16 = pk->dtype == PC_BF16;
    hipStream_t st = ctx->stream;
    const bool mfma = pk->variant == PC_VARIANT_MFMA;
    // the channel-major table serves the gather kernels' backward-data pass (the matrix-core kernels read operand tiles)
    const int ncm = mfma ? 0 : v.C;
    const int tiles_c = v.Cp / 32, ntiles = mfma ? (v.Fp / 32) * tiles_c : 0;
    hipLaunchKernelGGL(pc_pack_stage1_kernel, dim3((unsigned)(v.F + ncm + ntiles)), dim3(256), 0, st, W, pid, keep, la, v, ncm,
                       tiles_c);
    hipLaunchKernelGGL(pc_pack_place_kernel<true>, dim3(v.F), dim3(256), 0, st, W, pid, keep, v.F, v.C, (int64_t)v.C,
                       (int64_t)1, la, bf16, v);
    if (!mfma)
        hipLaunchKernelGGL(pc_pack_place_kernel<false>, dim3(v.C), dim3(256), 0, st, W, pid, keep, v.C, v.F, (int64_t)1,
                           (int64_t)v.C, la, bf16, v);
    pc_launch_ovf_merge(ctx, v);
    return pc_hip_check(ctx, hipGetLastError(), "pack launch");
}

// Re-packs several handles with one pool: three launches per group of up to PC_BATCH_MAX packs (two when none uses
// the gather kernels).
pc_status pc_launch_pack_batch(pc_ctx *ctx, int n, pc_packed *const *pk, const float *const *W, const uint8_t *const *pid,
                               const uint8_t *const *keep, const LibArg &la)
{
    for (int l0 = 0; l0 < n; l0 += PC_BATCH_MAX) {
        const int m = n - l0 < PC_BATCH_MAX ? n - l0 : PC_BATCH_MAX;
        PackBatchArg s1, fm, cm;
        memset(&s1, 0, sizeof(s1));
        s1.n = m;
        for (int i = 0; i < m; ++i) {
            const pc_packed *p = pk[l0 + i];
            const bool mfma = p->variant == PC_VARIANT_MFMA;
            s1.W[i] = W[l0 + i]; s1.pid[i] = pid[l0 + i]; s1.keep[i] = keep[l0 + i];
            s1.view[i] = p->v_dev;
            s1.ncm[i] = mfma ? 0 : p->v.C;
            s1.tiles_c[i] = p->v.Cp / 32;
            s1.bf16[i] = p->dtype == PC_BF16;
        }
        fm = s1;
        cm = s1;
        for (int i = 0; i < m; ++i) {
            const pc_packed *p = pk[l0 + i];
            const bool mfma = p->variant == PC_VARIANT_MFMA;
            s1.blk0[i + 1] = s1.blk0[i] + p->v.F + s1.ncm[i] + (mfma ? (p->v.Fp / 32) * s1.tiles_c[i] : 0);
            fm.blk0[i + 1] = fm.blk0[i] + p->v.F;
            cm.blk0[i + 1] = cm.blk0[i] + (mfma ? 0 : p->v.C);
        }
        hipLaunchKernelGGL(pc_pack_stage1_batch_kernel, dim3((unsigned)s1.blk0[m]), dim3(256), 0, ctx->stream, s1, la);
        hipLaunchKernelGGL(pc_pack_place_batch_kernel<true>, dim3((unsigned)fm.blk0[m]), dim3(256), 0, ctx->stream, fm, la);
        if (cm.blk0[m] > 0)
            hipLaunchKernelGGL(pc_pack_place_batch_kernel<false>, dim3((unsigned)cm.blk0[m]), dim3(256), 0, ctx->stream, cm, la);
        pc_launch_ovf_merge_batch(ctx, m, pk + l0);
        pc_status s = pc_hip_check(ctx, hipGetLastError(), "pack (several layers) launch");
        if (s != PC_OK) return s;
    }
    return PC_OK;
}

// Matrix-core packs made with the pool of the first such pack share launches of up to PC_BATCH_MAX; the others
// (gather-kernel packs, other pools) are updated one by one.
pc_status pc_launch_update_values_batch(pc_ctx *ctx, int n, pc_packed *const *pk, const float *const *W)
{
    PackBatchArg b;
    memset(&b, 0, sizeof(b));
    pc_packed *bpk[PC_BATCH_MAX];
    LibArg la;
    const pc_packed *first = nullptr;
    auto flush = [&]() -> pc_status {
        if (b.n == 0) return PC_OK;
        hipLaunchKernelGGL(pc_pack_revalue_batch_kernel, dim3((unsigned)b.blk0[b.n]), dim3(256), 0, ctx->stream, b, la);
        pc_launch_ovf_merge_batch(ctx, b.n, bpk);
        b.n = 0;
        return pc_hip_check(ctx, hipGetLastError(), "update_values (several layers) launch");
    };
    for (int l = 0; l < n; ++l) {
        pc_packed *p = pk[l];
        bool same = p->variant == PC_VARIANT_MFMA;
        if (same && !first) {
            first = p;
            pc_fill_lib(&la, p->lib, p->v.P);
        }
        if (same && (p->v.P != first->v.P || memcmp(p->lib, first->lib, sizeof(uint16_t) * p->v.P) != 0)) same = false;
        const int64_t nblk = ((int64_t)p->v.F * p->v.C + 255) / 256;
        if (!same) {
            pc_status s = pc_launch_update_values(ctx, p, W[l]);
            if (s != PC_OK) return s;
            continue;
        }
        const int i = b.n;
        bpk[i] = p;
        b.W[i] = W[l];
        b.view[i] = p->v_dev;
        b.tiles_c[i] = p->v.Cp / 32;
        b.ncm[i] = (p->v.Fp / 32) * b.tiles_c[i];
        b.bf16[i] = p->dtype == PC_BF16;
        b.blk0[i + 1] = b.blk0[i] + b.ncm[i] + (int32_t)nblk;
        if (++b.n == PC_BATCH_MAX) {
            pc_status s = flush();
            if (s != PC_OK) return s;
        }
    }
    return flush();
}

pc_status pc_launch_update_values(pc_ctx *ctx, pc_packed *pk, const float *W)
{
    PackView v = pk->v;
    LibArg la;
    pc_fill_lib(&la, pk->lib, v.P);
    int bf16 = pk->dtype == PC_BF16;
    int64_t nk = (int64_t)v.F * v.C;
    unsigned blocks = (unsigned)((nk + 255) / 256);
    if (pk->variant == PC_VARIANT_MFMA) {
        const int tiles_c = v.Cp / 32, ntiles = (v.Fp / 32) * tiles_c;
        hipLaunchKernelGGL(pc_pack_revalue_kernel, dim3((unsigned)ntiles + blocks), dim3(256), 0, ctx->stream, W, la, bf16, v,
                           tiles_c, ntiles);
        pc_launch_ovf_merge(ctx, v);
    } else {
        hipLaunchKernelGGL(pc_pack_regather_fm_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, la, bf16, v);
        hipLaunchKernelGGL(pc_pack_regather_cm_kernel, dim3(blocks), dim3(256), 0, ctx->stream, v);
    }
    return pc_hip_check(ctx, hipGetLastError(), "update_values launch");
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

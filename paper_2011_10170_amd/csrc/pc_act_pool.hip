// The step between two convolution layers of a chained network (Section 5.2, "Backward Phase Acceleration":
// a = sigma(z) forward, the error times sigma'(z) backward), for the networks of Section 6: sigma = ReLU,
// optionally followed by a 2x2 max pooling of stride 2. NHWC tensors, float32 or bfloat16.
//
// Both passes only compare and copy: results are exact, and bound by HBM traffic. One thread serves VEC
// consecutive channels of one pooled output element with 16-byte accesses (VEC = 8 bfloat16 / 4 float32) when the
// channel count and the pointers allow it, else VEC = 1. The forward pass leaves one byte per output element for
// the backward pass: the window position 2*dr + dc of the maximum, 255 when no error passes (maximum not
// positive). Among equal maxima the first position in row-major order wins (strict > while scanning).
#include "pc_internal.h"

#define AP_BLOCK 256
#define AP_NONE 255u

template <typename T, int VEC> struct alignas(sizeof(T) * VEC) ApVec { T e[VEC]; };
template <int VEC> struct alignas(VEC) ApSel { uint8_t e[VEC]; };

// i -> (n, oh, ow, cv) of a [..][Hn][Wn][Cv] index space; 32-bit divisions when the space allows (uniform branch)
__device__ __forceinline__ void ap_decompose(int64_t i, int64_t total, int Hn, int Wn, int Cv, int64_t &n, int &oh, int &ow, int &cv)
{
    if (total <= 0x7FFFFFFFLL) {
        uint32_t p = (uint32_t)i;
        cv = (int)(p % (uint32_t)Cv);
        p /= (uint32_t)Cv;
        ow = (int)(p % (uint32_t)Wn);
        p /= (uint32_t)Wn;
        oh = (int)(p % (uint32_t)Hn);
        n = p / (uint32_t)Hn;
    } else {
        cv = (int)(i % Cv);
        int64_t p = i / Cv;
        ow = (int)(p % Wn);
        p /= Wn;
        oh = (int)(p % Hn);
        n = p / Hn;
    }
}

__device__ __forceinline__ float ap_value(float v) { return v; }
__device__ __forceinline__ float ap_value(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// z [N][H][W][C] -> a, sel [N][Ho][Wo][C], Ho = H / POOL, Wo = W / POOL. Cv = C / VEC; total = N*Ho*Wo*Cv.
template <typename T, int VEC, int POOL>
__global__ void __launch_bounds__(AP_BLOCK)
pc_act_pool_fwd_kernel(const T *__restrict__ z, T *__restrict__ a, uint8_t *__restrict__ sel,
                       int H, int W, int Cv, int Ho, int Wo, int64_t total)
{
    typedef ApVec<T, VEC> V;
    const int64_t i = (int64_t)blockIdx.x * AP_BLOCK + threadIdx.x;
    if (i >= total) return;
    int cv, ow, oh;
    int64_t n;
    ap_decompose(i, total, Ho, Wo, Cv, n, oh, ow, cv);
    const V *zv = reinterpret_cast<const V *>(z);
    const int64_t base = ((n * H + (int64_t)oh * POOL) * W + (int64_t)ow * POOL) * Cv + cv;
    V v[POOL * POOL];
#pragma unroll
    for (int dr = 0; dr < POOL; ++dr)
#pragma unroll
        for (int dc = 0; dc < POOL; ++dc)
            v[dr * POOL + dc] = zv[base + ((int64_t)dr * W + dc) * Cv];
    V out;
    ApSel<VEC> so;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        T bt = v[0].e[j];
        float best = ap_value(bt);
        unsigned arg = 0;
#pragma unroll
        for (int k = 1; k < POOL * POOL; ++k) {
            const float x = ap_value(v[k].e[j]);
            if (x > best) { best = x; bt = v[k].e[j]; arg = k; }
        }
        const bool pos = best > 0.0f;
        out.e[j] = pos ? bt : (T)0;
        so.e[j] = (uint8_t)(pos ? arg : AP_NONE);
    }
    reinterpret_cast<V *>(a)[i] = out;
    reinterpret_cast<ApSel<VEC> *>(sel)[i] = so;
}

// da, sel [N][Ho][Wo][C] -> dz [N][H][W][C]. One thread per window of the grid that covers the whole map
// (Hc = ceil(H / POOL), Wc likewise): an odd last row / column belongs to no pooled element and gets zeros.
template <typename T, int VEC, int POOL>
__global__ void __launch_bounds__(AP_BLOCK)
pc_act_pool_bwd_kernel(const T *__restrict__ da, const uint8_t *__restrict__ sel, T *__restrict__ dz,
                       int H, int W, int Cv, int Ho, int Wo, int Hc, int Wc, int64_t total)
{
    typedef ApVec<T, VEC> V;
    const int64_t i = (int64_t)blockIdx.x * AP_BLOCK + threadIdx.x;
    if (i >= total) return;
    int cv, ow, oh;
    int64_t n;
    ap_decompose(i, total, Hc, Wc, Cv, n, oh, ow, cv);
    const bool whole = oh < Ho && ow < Wo;
    // clamped index: the loads are unconditional, a window outside the pooled map ignores what it read
    const int64_t src = ((n * Ho + (oh < Ho ? oh : Ho - 1)) * Wo + (ow < Wo ? ow : Wo - 1)) * Cv + cv;
    const V g = reinterpret_cast<const V *>(da)[src];
    const ApSel<VEC> s = reinterpret_cast<const ApSel<VEC> *>(sel)[src];
    V *dzv = reinterpret_cast<V *>(dz);
#pragma unroll
    for (int dr = 0; dr < POOL; ++dr)
#pragma unroll
        for (int dc = 0; dc < POOL; ++dc) {
            const int h = oh * POOL + dr, w = ow * POOL + dc;
            if (h >= H || w >= W) continue;
            V out;
#pragma unroll
            for (int j = 0; j < VEC; ++j)
                out.e[j] = (whole && s.e[j] == dr * POOL + dc) ? g.e[j] : (T)0;
            dzv[((n * H + h) * W + w) * Cv + cv] = out;
        }
}

static pc_status ap_check(pc_ctx *ctx, const char *who, const void *p0, const void *p1, const void *p2,
                          int32_t N, int32_t H, int32_t W, int32_t C, pc_dtype dtype, int32_t pool)
{
    if (!p0 || !p1 || !p2) return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: null pointer", who);
    if (dtype != PC_F32 && dtype != PC_BF16) return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (pool != 1 && pool != 2) return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: pool=%d, must be 1 or 2", who, pool);
    if (N < 1 || H < 1 || W < 1 || C < 1 || C > 65535) return pc_fail(ctx, PC_ERR_BAD_SHAPE, "%s: N=%d H=%d W=%d C=%d out of range", who, N, H, W, C);
    if (H < pool || W < pool) return pc_fail(ctx, PC_ERR_BAD_SHAPE, "%s: a %dx%d map has no %dx%d window", who, H, W, pool, pool);
    return PC_OK;
}

static bool ap_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <typename T, int VEC>
static void ap_launch_fwd(pc_ctx *ctx, const void *z, void *a, uint8_t *sel, int N, int H, int W, int C, int pool)
{
    const int Ho = H / pool, Wo = W / pool, Cv = C / VEC;
    const int64_t total = (int64_t)N * Ho * Wo * Cv;
    const dim3 grid((unsigned)((total + AP_BLOCK - 1) / AP_BLOCK));
    if (pool == 2)
        hipLaunchKernelGGL((pc_act_pool_fwd_kernel<T, VEC, 2>), grid, dim3(AP_BLOCK), 0, ctx->stream,
                           (const T *)z, (T *)a, sel, H, W, Cv, Ho, Wo, total);
    else
        hipLaunchKernelGGL((pc_act_pool_fwd_kernel<T, VEC, 1>), grid, dim3(AP_BLOCK), 0, ctx->stream,
                           (const T *)z, (T *)a, sel, H, W, Cv, Ho, Wo, total);
}

template <typename T, int VEC>
static void ap_launch_bwd(pc_ctx *ctx, const void *da, const uint8_t *sel, void *dz, int N, int H, int W, int C, int pool)
{
    const int Ho = H / pool, Wo = W / pool, Cv = C / VEC;
    const int Hc = (H + pool - 1) / pool, Wc = (W + pool - 1) / pool;
    const int64_t total = (int64_t)N * Hc * Wc * Cv;
    const dim3 grid((unsigned)((total + AP_BLOCK - 1) / AP_BLOCK));
    if (pool == 2)
        hipLaunchKernelGGL((pc_act_pool_bwd_kernel<T, VEC, 2>), grid, dim3(AP_BLOCK), 0, ctx->stream,
                           (const T *)da, sel, (T *)dz, H, W, Cv, Ho, Wo, Hc, Wc, total);
    else
        hipLaunchKernelGGL((pc_act_pool_bwd_kernel<T, VEC, 1>), grid, dim3(AP_BLOCK), 0, ctx->stream,
                           (const T *)da, sel, (T *)dz, H, W, Cv, Ho, Wo, Hc, Wc, total);
}

// The largest grid: one thread per element at VEC = 1 must still fit 2^31 - 1 blocks of 256 threads.
static bool ap_too_large(int64_t elements) { return (elements + AP_BLOCK - 1) / AP_BLOCK > 0x7FFFFFFFLL; }

extern "C" pc_status pc_act_pool_fwd(pc_ctx *ctx, const void *z, int32_t N, int32_t H, int32_t W, int32_t C,
                                     pc_dtype dtype, int32_t pool, void *a, uint8_t *sel)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = ap_check(ctx, "pc_act_pool_fwd", z, a, sel, N, H, W, C, dtype, pool);
    if (s != PC_OK) return s;
    if (ap_too_large((int64_t)N * H * W * C)) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "pc_act_pool_fwd: tensor too large");
    PC_HIP(ctx, hipSetDevice(ctx->device));
    const int vec = dtype == PC_BF16 ? 8 : 4;
    // sel is accessed vec bytes at a time: its alignment matters as well (vec <= 8)
    const bool wide = C % vec == 0 && ap_aligned16(z) && ap_aligned16(a) && (reinterpret_cast<uintptr_t>(sel) & 7u) == 0;
    if (dtype == PC_BF16) {
        if (wide) ap_launch_fwd<uint16_t, 8>(ctx, z, a, sel, N, H, W, C, pool);
        else ap_launch_fwd<uint16_t, 1>(ctx, z, a, sel, N, H, W, C, pool);
    } else {
        if (wide) ap_launch_fwd<float, 4>(ctx, z, a, sel, N, H, W, C, pool);
        else ap_launch_fwd<float, 1>(ctx, z, a, sel, N, H, W, C, pool);
    }
    return pc_hip_check(ctx, hipGetLastError(), "activation + pooling forward launch");
}

extern "C" pc_status pc_act_pool_bwd(pc_ctx *ctx, const void *da, const uint8_t *sel, int32_t N, int32_t H, int32_t W,
                                     int32_t C, pc_dtype dtype, int32_t pool, void *dz)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = ap_check(ctx, "pc_act_pool_bwd", da, sel, dz, N, H, W, C, dtype, pool);
    if (s != PC_OK) return s;
    if (ap_too_large((int64_t)N * H * W * C)) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "pc_act_pool_bwd: tensor too large");
    PC_HIP(ctx, hipSetDevice(ctx->device));
    const int vec = dtype == PC_BF16 ? 8 : 4;
    const bool wide = C % vec == 0 && ap_aligned16(da) && ap_aligned16(dz) && (reinterpret_cast<uintptr_t>(sel) & 7u) == 0;
    if (dtype == PC_BF16) {
        if (wide) ap_launch_bwd<uint16_t, 8>(ctx, da, sel, dz, N, H, W, C, pool);
        else ap_launch_bwd<uint16_t, 1>(ctx, da, sel, dz, N, H, W, C, pool);
    } else {
        if (wide) ap_launch_bwd<float, 4>(ctx, da, sel, dz, N, H, W, C, pool);
        else ap_launch_bwd<float, 1>(ctx, da, sel, dz, N, H, W, C, pool);
    }
    return pc_hip_check(ctx, hipGetLastError(), "activation + pooling backward launch");
}

// ------------------------------------------------------------------ ReLU alone, in place
// z = relu(z); and dz = dz where a > 0, else +0 (the ReLU derivative read from the activation itself: a > 0 exactly
// where z > 0). Used where a conv launch cannot apply the step itself.
template <typename T, int VEC, bool MASK>
__global__ void __launch_bounds__(AP_BLOCK) pc_relu_kernel(T *__restrict__ z, const T *__restrict__ a, int64_t nv)
{
    typedef ApVec<T, VEC> V;
    const int64_t i = (int64_t)blockIdx.x * AP_BLOCK + threadIdx.x;
    if (i >= nv) return;
    V v = reinterpret_cast<V *>(z)[i];
    V m = v;
    if (MASK) m = reinterpret_cast<const V *>(a)[i];
#pragma unroll
    for (int j = 0; j < VEC; ++j) v.e[j] = ap_value(m.e[j]) > 0.0f ? v.e[j] : (T)0;
    reinterpret_cast<V *>(z)[i] = v;
}

template <bool MASK>
static pc_status ap_launch_relu(pc_ctx *ctx, void *z, const void *a, int64_t n, pc_dtype dtype)
{
    if (n <= 0) return PC_OK;
    if (ap_too_large(n)) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "ReLU: tensor too large");
    const int vec = dtype == PC_BF16 ? 8 : 4;
    const bool wide = n % vec == 0 && ap_aligned16(z) && (!MASK || ap_aligned16(a));
    const int64_t nv = wide ? n / vec : n;
    const dim3 grid((unsigned)((nv + AP_BLOCK - 1) / AP_BLOCK));
    if (dtype == PC_BF16) {
        if (wide) hipLaunchKernelGGL((pc_relu_kernel<uint16_t, 8, MASK>), grid, dim3(AP_BLOCK), 0, ctx->stream, (uint16_t *)z, (const uint16_t *)a, nv);
        else hipLaunchKernelGGL((pc_relu_kernel<uint16_t, 1, MASK>), grid, dim3(AP_BLOCK), 0, ctx->stream, (uint16_t *)z, (const uint16_t *)a, nv);
    } else {
        if (wide) hipLaunchKernelGGL((pc_relu_kernel<float, 4, MASK>), grid, dim3(AP_BLOCK), 0, ctx->stream, (float *)z, (const float *)a, nv);
        else hipLaunchKernelGGL((pc_relu_kernel<float, 1, MASK>), grid, dim3(AP_BLOCK), 0, ctx->stream, (float *)z, (const float *)a, nv);
    }
    return pc_hip_check(ctx, hipGetLastError(), "ReLU launch");
}

pc_status pc_launch_relu(pc_ctx *ctx, void *z, int64_t n, pc_dtype dtype) { return ap_launch_relu<false>(ctx, z, nullptr, n, dtype); }
pc_status pc_launch_relu_mask(pc_ctx *ctx, void *dz, const void *a, int64_t n, pc_dtype dtype) { return ap_launch_relu<true>(ctx, dz, a, n, dtype); }

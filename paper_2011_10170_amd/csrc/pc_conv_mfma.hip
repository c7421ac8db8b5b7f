// Matrix-core (MFMA) variant of the passes for bf16 layers (Section 5.2; the per-layer choice
// between the sparse kernel and a dense contraction of Section 5.2/5.4, re-made for CDNA4).
//
// The layer is computed as an implicit GEMM over a tap list,
//     out[pixel, m] = sum_taps sum_k  A_tap[m, k] * in[pixel shifted by tap, k],
// with v_mfma_f32_32x32x16_bf16. A_tap is the hard-pruned weight matrix of one tap (zero at every
// pruned position), pre-arranged at pack time in the register order of the instruction's A operand,
// so wavefronts load it straight from global memory/L2 with one 16-byte load per lane. The input
// halo tile of 16 to 128 channels is staged in LDS (pixel-major, pitch 2*channels + 16 bytes: conflict-free
// 16-byte reads) and every tap is a constant LDS offset.
//   forward        : in = x,  m = filter,  k = channel, 9 taps at (r, s)
//   backward-data  : in = dy, m = channel, k = filter; stride 1: 9 taps at (2-r, 2-s) (rot180);
//                    stride 2: four parity classes of input pixels with 1, 2, 2 and 4 taps, one launch
//   backward-weight: pc_wgrad_mfma.hip
// This file holds the cooperative kernel (every wavefront stages and multiplies; output split over the
// wavefronts), the channel-padding copies and the planner (the operand tiles are written at pack time, in
// pc_select_pack.hip); the persistent wave-specialised kernel that takes
// most full 3x3 launches is in pc_conv_mfma_ws.hip.
//
// Operand layout of v_mfma_f32_32x32x16_bf16 used here: lane l holds row (A) / column (B) l%32 and
// the 8 consecutive k values 8*(l/32)..+7; accumulator register r of lane l is row
// 8*(r/4) + 4*(l/32) + r%4, column l%32.
#include "pc_mfma.h"

#define MF_LDS_MAX 65536

bool pc_mfma_supports(int F, int C) { return (int64_t)F * C < (1 << 23); }   // kinfo packs the slot in 23 bits

// Depth of the A-fragment prefetch ring: the smallest divisor of the steps per chunk that keeps the loads
// about 1000 cycles (an L2 round trip) ahead of their MFMAs; small tiles prefetch a whole chunk ahead.
constexpr int pc_prefetch_depth(int ns, int step_cycles)
{
    int want = (1024 + step_cycles - 1) / step_cycles;
    if (want > ns) want = ns;
    for (int d = want; d <= ns; ++d)
        if (ns % d == 0) return d;
    return ns;
}

// KC channels are staged per pass (LDS pixel pitch 2*KC + 16 bytes: conflict-free 16-byte reads).
// A fragments are prefetched PF steps ahead from global memory, B fragments one step ahead from LDS.
// With gridDim.z > 1 every split reduces its own range of channel chunks and writes float32 partial
// sums [split][pixel][m] that pc_mfma_splitk_reduce_kernel adds in a fixed order.
// MC: the launch covers the four parity classes of a stride-2 backward-data pass (NTAPS = 4 is then the longest
// tap list; a class with fewer taps skips the other steps, uniformly for the workgroup).
template <int A_T, int B_T, int WAVES_M, int WAVES_N, int NTAPS, int KC, bool MC = false>
__global__ void __launch_bounds__(256, 2)
pc_mfma_conv_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out, const uint16_t *__restrict__ wz,
                    float *__restrict__ partial, MfmaArgs g)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int BM = 32 * A_T * WAVES_M;
    constexpr int KSC = KC / 16;
    constexpr int NS = NTAPS * KSC;
    constexpr int PF = pc_prefetch_depth(NS, A_T * B_T * 32);
    constexpr int PITCH = 2 * KC + 16;
    constexpr int PARTS = KC / 8;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    int bt = blockIdx.x;
    int GH = g.GH, GW = g.GW, ooff_y = g.ooff_y, ooff_x = g.ooff_x, ntaps = NTAPS;
    int tapw[NTAPS], tapo[NTAPS];
    if constexpr (MC) {
        const int cl = bt / g.cls_tiles;
        bt -= cl * g.cls_tiles;
        GH = g.cls_GH[cl]; GW = g.cls_GW[cl]; ooff_y = g.cls_ooy[cl]; ooff_x = g.cls_oox[cl]; ntaps = g.cls_ntaps[cl];
#pragma unroll
        for (int t = 0; t < NTAPS; ++t) { tapw[t] = g.cls_tap_w[cl][t]; tapo[t] = g.cls_tap_off[cl][t]; }
    } else {
#pragma unroll
        for (int t = 0; t < NTAPS; ++t) { tapw[t] = g.tap_w[t]; tapo[t] = g.tap_off[t]; }
    }
    const int tx = bt % g.tiles_x; bt /= g.tiles_x;
    const int ty = bt % g.tiles_y; bt /= g.tiles_y;
    const int tn = bt;
    const int gy0 = ty * g.TH, gx0 = tx * g.TW;
    const int in_y0 = gy0 * g.iscale + g.ioff_y, in_x0 = gx0 * g.iscale + g.ioff_x;
    const int m0 = blockIdx.y * BM + wm * (32 * A_T);
    const int mt0 = m0 >> 5;
    const int npix = g.TI * g.TH * g.TW;
    const int ch0 = blockIdx.z * g.cps;
    const int ch1 = min(ch0 + g.cps, g.nchunks);

    int base[B_T];
#pragma unroll
    for (int j = 0; j < B_T; ++j) {
        int q = (wn * B_T + j) * 32 + (lane & 31);
        if (q >= npix) q = npix - 1;
        int ti = q / (g.TH * g.TW);
        int rem = q - ti * g.TH * g.TW;
        int y = rem / g.TW, x = rem - y * g.TW;
        base[j] = ((ti * g.IH + y * g.lstep) * g.IW + x * g.lstep) * PITCH + (lane >> 5) * 16;
    }

    f32x16 acc[A_T][B_T];
#pragma unroll
    for (int i = 0; i < A_T; ++i)
#pragma unroll
        for (int j = 0; j < B_T; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const uint16_t *wzl = wz + (int64_t)mt0 * 9 * g.KS * 512 + lane * 8;
    // fragment of row tile i for step st of chunk ch (past the last chunk: re-read the last one, unused)
    auto a_load = [&](int ch, int st, int i) -> bf16x8 {
        const int t = st / KSC, ks = st % KSC;
        const int chc = ch < ch1 ? ch : ch1 - 1;
        return *reinterpret_cast<const bf16x8 *>(wzl + (int64_t)((i * 9 + tapw[t]) * g.KS + chc * KSC + ks) * 512);
    };
    bf16x8 aring[PF][A_T];
#pragma unroll
    for (int d = 0; d < PF; ++d)
#pragma unroll
        for (int i = 0; i < A_T; ++i) aring[d][i] = a_load(ch0, d, i);

    // element offset of every staged pixel in the input tensor (-1 = zero padding), computed once
    const int HP = g.TI * g.IH * g.IW;
    int64_t *pixoff = reinterpret_cast<int64_t *>(lds + (size_t)HP * PITCH);
    for (int q = threadIdx.x; q < HP; q += 256) {
        int ix = q % g.IW;
        int t2 = q / g.IW;
        int iy = t2 % g.IH;
        int ti = t2 / g.IH;
        int n = tn * g.TI + ti, y = in_y0 + iy, x = in_x0 + ix;
        bool ok = n < g.N && y >= 0 && y < g.in_H && x >= 0 && x < g.in_W;
        pixoff[q] = ok ? (((int64_t)n * g.in_H + y) * g.in_W + x) * g.in_CH : (int64_t)-1;
    }
    for (int ch = ch0; ch < ch1; ++ch) {
        __syncthreads();
        if ((g.in_CH & 7) == 0) {
            // four elements per thread and round: the loads are unconditional (address clamped to the tensor's
            // start, value masked afterwards) and all issued before the first LDS write, so a round costs one
            // memory round trip instead of four
            constexpr int U = 4;
            const int total = HP * PARTS;
            for (int e0 = threadIdx.x; e0 < total; e0 += 256 * U) {
                uint4 vv[U];
                bool okv[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = e0 + 256 * u, ec = e < total ? e : total - 1;
                    const int q = ec / PARTS, part = ec - q * PARTS;
                    const int c = ch * KC + part * 8;
                    const int64_t po = pixoff[q];
                    okv[u] = po >= 0 && c < g.in_CH;
                    vv[u] = *reinterpret_cast<const uint4 *>(in + (okv[u] ? po + c : 0));
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e = e0 + 256 * u;
                    if (e < total) {
                        const int q = e / PARTS, part = e - q * PARTS;
                        *reinterpret_cast<uint4 *>(lds + q * PITCH + part * 16) = okv[u] ? vv[u] : make_uint4(0u, 0u, 0u, 0u);
                    }
                }
            }
        } else {
            for (int e = threadIdx.x; e < HP * PARTS; e += 256) {
                const int q = e / PARTS, part = e - q * PARTS;
                const int c = ch * KC + part * 8;
                const int64_t po = pixoff[q];
                uint4 v = make_uint4(0u, 0u, 0u, 0u);
                if (po >= 0 && c < g.in_CH) {   // channel count not a multiple of 8: rows are not 16-byte aligned, load by element
                    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (c + i < g.in_CH) w[i >> 1] |= (uint32_t)in[po + c + i] << ((i & 1) * 16);
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
                *reinterpret_cast<uint4 *>(lds + q * PITCH + part * 16) = v;
            }
        }
        __syncthreads();
        // B fragments are read DB steps ahead of their MFMAs (LDS latency is longer than one small step);
        // scheduling barriers keep the compiler from sinking the loads back next to their uses
        constexpr int DB = (A_T * B_T >= 4) ? 1 : (NS >= 4 ? 4 : NS);
        constexpr int RB = DB + 1;
        bf16x8 bring[RB][B_T];
#pragma unroll
        for (int d = 0; d < DB; ++d) {
            const int t1 = d / KSC, k1 = d % KSC;
#pragma unroll
            for (int j = 0; j < B_T; ++j)
                bring[d % RB][j] = *reinterpret_cast<const bf16x8 *>(lds + base[j] + tapo[t1] + k1 * 32);
        }
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            if (st + DB < NS) {
                const int t1 = (st + DB) / KSC, k1 = (st + DB) % KSC;
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    bring[(st + DB) % RB][j] = *reinterpret_cast<const bf16x8 *>(lds + base[j] + tapo[t1] + k1 * 32);
            }
            bf16x8 anow[A_T];
#pragma unroll
            for (int i = 0; i < A_T; ++i) anow[i] = aring[st % PF][i];
            {
                const int nst = st + PF;
                const int nch = nst >= NS ? ch + 1 : ch;
                const int nss = nst >= NS ? nst - NS : nst;
#pragma unroll
                for (int i = 0; i < A_T; ++i) aring[st % PF][i] = a_load(nch, nss, i);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (!MC || st / KSC < ntaps) {
#pragma unroll
                for (int i = 0; i < A_T; ++i)
#pragma unroll
                    for (int j = 0; j < B_T; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(anow[i], bring[st % RB][j], acc[i][j], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // epilogue: lane holds, for its pixel, 4 consecutive output channels per accumulator quad
#pragma unroll
    for (int j = 0; j < B_T; ++j) {
        int q = (wn * B_T + j) * 32 + (lane & 31);
        if (q >= npix) continue;
        int ti = q / (g.TH * g.TW);
        int rem = q - ti * g.TH * g.TW;
        int y = rem / g.TW, x = rem - y * g.TW;
        int n = tn * g.TI + ti, gy = gy0 + y, gx = gx0 + x;
        if (n >= g.N || gy >= GH || gx >= GW) continue;
        int oy = gy * g.oscale + ooff_y, ox = gx * g.oscale + ooff_x;
        const int64_t opix = ((int64_t)n * g.out_H + oy) * g.out_W + ox;
        if (gridDim.z == 1) {
            uint16_t *op = out + opix * g.out_CH;
#pragma unroll
            for (int i = 0; i < A_T; ++i)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    int m = m0 + i * 32 + r4 * 8 + (lane >> 5) * 4;
                    if ((g.out_CH & 3) == 0) {
                        if (m < g.out_CH) {
                            uint2 pk;
                            pk.x = (uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 0]) | ((uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 1]) << 16);
                            pk.y = (uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 2]) | ((uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 3]) << 16);
                            *reinterpret_cast<uint2 *>(op + m) = pk;
                        }
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (m + e < g.out_CH) op[m + e] = pc_f32_to_bf16(acc[i][j][r4 * 4 + e]);
                    }
                }
        } else {
            const int64_t npx_all = (int64_t)g.N * g.out_H * g.out_W;
            float *pp = partial + ((int64_t)blockIdx.z * npx_all + opix) * g.out_CH;
#pragma unroll
            for (int i = 0; i < A_T; ++i)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    int m = m0 + i * 32 + r4 * 8 + (lane >> 5) * 4;
                    if ((g.out_CH & 3) == 0) {
                        if (m < g.out_CH)
                            *reinterpret_cast<float4 *>(pp + m) = make_float4(acc[i][j][r4 * 4 + 0], acc[i][j][r4 * 4 + 1],
                                                                              acc[i][j][r4 * 4 + 2], acc[i][j][r4 * 4 + 3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (m + e < g.out_CH) pp[m + e] = acc[i][j][r4 * 4 + e];
                    }
                }
        }
    }
}

// out[e] = bf16(partial[0][e] + partial[1][e] + ...), 4 elements per thread
__global__ void __launch_bounds__(256)
pc_mfma_splitk_reduce_kernel(const float4 *__restrict__ partial, int64_t n4, int splits, uint2 *__restrict__ out)
{
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n4) return;
    float4 s = partial[e];
    for (int z = 1; z < splits; ++z) {
        float4 p = partial[(int64_t)z * n4 + e];
        s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
    }
    uint2 pk;
    pk.x = (uint32_t)pc_f32_to_bf16(s.x) | ((uint32_t)pc_f32_to_bf16(s.y) << 16);
    pk.y = (uint32_t)pc_f32_to_bf16(s.z) | ((uint32_t)pc_f32_to_bf16(s.w) << 16);
    out[e] = pk;
}


// ------------------------------------------------------------------ channel padding copies
// xp[pixel][0..Cp) = x[pixel][0..C), zero above: a copy whose pixel rows are 16-byte aligned groups of 8 channels
__global__ void __launch_bounds__(256)
pc_pad_channels_kernel(const uint16_t *__restrict__ x, uint4 *__restrict__ xp, int64_t npix, int C, int Cp)
{
    const int gpp = Cp / 8;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= npix * gpp) return;
    const int64_t p = i / gpp;
    const int c0 = (int)(i - p * gpp) * 8;
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (c0 + e < C) w[e >> 1] |= (uint32_t)x[p * C + c0 + e] << ((e & 1) * 16);
    xp[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

void pc_launch_pad_channels(pc_ctx *ctx, const uint16_t *x, void *xp, int64_t npix, int C, int Cp)
{
    const int64_t n16 = npix * (Cp / 8);
    hipLaunchKernelGGL(pc_pad_channels_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, ctx->stream, x,
                       reinterpret_cast<uint4 *>(xp), npix, C, Cp);
}

// y[pixel][0..C) = yp[pixel][0..C) for rows of Cp = 8 channels (C < 8): the inverse of the copy above
__global__ void __launch_bounds__(256)
pc_unpad_channels_kernel(const uint4 *__restrict__ yp, uint16_t *__restrict__ y, int64_t npix, int C)
{
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= npix) return;
    const uint4 v = yp[p];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (e < C) y[p * C + e] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
}

void pc_launch_unpad_channels(pc_ctx *ctx, const void *yp, uint16_t *y, int64_t npix, int C)
{
    hipLaunchKernelGGL(pc_unpad_channels_kernel, dim3((unsigned)((npix + 255) / 256)), dim3(256), 0, ctx->stream,
                       reinterpret_cast<const uint4 *>(yp), y, npix, C);
}

// ------------------------------------------------------------------ planning and launch
struct MfmaCfg { int a, b, wm, wn, kc; };
static const MfmaCfg kCfgs[] = {
    {2, 4, 1, 4, 32}, {2, 4, 2, 2, 32}, {2, 2, 2, 2, 32}, {2, 2, 2, 2, 64}, {1, 2, 2, 2, 64}, {1, 1, 2, 2, 64},
    {1, 2, 2, 2, 16},
};
// automatic choice tries these in order and keeps the first that yields enough workgroups (else the last)
static const int kAutoOrder[] = {4, 5};
// the same for a launch over the four parity classes (four times the workgroups: the 128-row tiles pay off earlier)
static const int kAutoOrderClasses[] = {1, 3, 4, 5};
static const int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);

void pc_plan_mfma_tiles(MfmaArgs *g, int BN, int ext)
{
    int ntx = (g->GW + 31) / 32;
    g->TW = (g->GW + ntx - 1) / ntx;
    int thmax = BN / g->TW;
    if (thmax < 1) thmax = 1;
    int nty = (g->GH + thmax - 1) / thmax;
    g->TH = (g->GH + nty - 1) / nty;
    g->TI = BN / (g->TH * g->TW);
    if (g->TI > g->N) g->TI = g->N;
    if (g->TI < 1) g->TI = 1;
    g->IH = (g->TH - 1) * g->lstep + ext;
    g->IW = (g->TW - 1) * g->lstep + ext;
    g->tiles_y = (g->GH + g->TH - 1) / g->TH;
    g->tiles_x = (g->GW + g->TW - 1) / g->TW;
}

// The four parity classes of a stride-2 backward-data pass: extent, output offset and tap list of each.
struct ParityClasses {
    int GH[4], GW[4], ooy[4], oox[4], ntaps[4];
    int tap_w[4][4], tr[4][4], tc[4][4];
};

template <int A_T, int B_T, int WM, int WN, int KC>
static void launch_cfg(hipStream_t st, dim3 grid, size_t lds, bool classes, const uint16_t *in, uint16_t *out,
                       const uint16_t *wz, float *partial, const MfmaArgs &g)
{
    if (classes)
        hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 4, KC, true>), grid, dim3(256), lds, st, in, out, wz, partial, g);
    else
        hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 9, KC, false>), grid, dim3(256), lds, st, in, out, wz, partial, g);
}


// g holds everything but the tile plan; ext = reach of the tap offsets (3 or 2); tap rows/cols in tr/tc.
// With pcl (stride-2 backward-data) the launch covers the four parity classes: g.GH/GW are the largest class
// extents, ntaps = 4, and tr/tc are unused.
// act / act_mask / fused: a fused activation step (PC_ACT_*) is applied when the wave-specialised kernel takes the
// launch and writes the output tensor itself; *fused then becomes true. Otherwise the plain conv runs and the caller
// applies the step.
static pc_status run_mfma_conv(pc_ctx *ctx, MfmaArgs g, int ext, int ntaps, const int *tr, const int *tc,
                               const uint16_t *in, uint16_t *out, const uint16_t *wz, const SparseOperand &sp,
                               const ParityClasses *pcl = nullptr, int act = PC_ACT_NONE, const uint16_t *act_mask = nullptr,
                               bool *fused = nullptr)
{
    g.act_mask = nullptr;
    int plan_cfg = (ctx->plan_cfg >= 10 && ctx->plan_cfg < 13) ? -1 : ctx->plan_cfg;   // 10 and 11 select a backward-weight kernel
    if (ntaps == 9 && (plan_cfg < 0 || plan_cfg >= 7) && ctx->plan_split == 0) {
        // The wave-specialised kernel reads and writes whole groups of 8 channels. The first layer's few channels
        // (input of the forward pass, output of the backward-data pass) go through a copy with 8-channel rows.
        MfmaArgs gw = g;
        const uint16_t *inw = in;
        uint16_t *outw = out;
        const int64_t in_pix = (int64_t)g.N * g.in_H * g.in_W, out_pix = (int64_t)g.N * g.out_H * g.out_W;
        // (for the input the copy pays off on large images only: on 32x32 inputs the cooperative kernel's element-wise
        // staging of 3 channels is as fast as copy + kernel)
        const bool pad_in = g.in_CH < 8 && (in_pix >= 300000 || plan_cfg >= 7), pad_out = g.out_CH < 8 && g.oscale == 1;
        if (pad_in || pad_out) {
            void *scr = nullptr;
            pc_status s = pc_scratch(ctx, (size_t)16 * (size_t)((pad_in ? in_pix : 0) + (pad_out ? out_pix : 0)), &scr);
            if (s != PC_OK) return s;
            if (pad_in) {
                pc_launch_pad_channels(ctx, in, scr, in_pix, g.in_CH, 8);
                inw = static_cast<const uint16_t *>(scr);
                gw.in_CH = 8;
            }
            if (pad_out) {
                outw = reinterpret_cast<uint16_t *>(static_cast<unsigned char *>(scr) + (pad_in ? 16 * in_pix : 0));
                gw.out_CH = 8;
            }
        }
        if ((gw.in_CH & 7) == 0 && (gw.in_CH >= 32 || pad_in)) {
            bool launched = false;
            const int act_here = (fused && !pad_out) ? act : PC_ACT_NONE;
            gw.act_mask = act_here == PC_ACT_RELU_MASK ? act_mask : nullptr;
            pc_status s = pc_run_mfma_conv_ws(ctx, plan_cfg, gw, ext, tr, tc, inw, outw, wz, sp, &launched, act_here);
            if (s != PC_OK) return s;
            if (launched) {
                if (fused) *fused = act_here != PC_ACT_NONE;
                if (pad_out) pc_launch_unpad_channels(ctx, outw, out, out_pix, g.out_CH);
                return pc_hip_check(ctx, hipGetLastError(), "channel copy launch");
            }
        }
    }
    if (plan_cfg >= 7) {   // forced wave-specialised kernel: launches it cannot take (tap subsets) use the automatic choice
        if (ntaps == 9) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: the wave-specialised kernel does not fit this launch");
        plan_cfg = -1;
    }
    int pick = -1, pick_split = 1;
    MfmaArgs best = g;
    const int64_t want = 2 * (int64_t)ctx->num_cu;
    const int *order = pcl ? kAutoOrderClasses : kAutoOrder;
    const int n_order = pcl ? (int)(sizeof(kAutoOrderClasses) / sizeof(int)) : (int)(sizeof(kAutoOrder) / sizeof(int));
    const int n_try = plan_cfg >= 0 ? 1 : n_order;
    for (int k = 0; k < n_try; ++k) {
        int ci = plan_cfg >= 0 ? plan_cfg : order[k];
        if (plan_cfg < 0 && g.in_CH <= 16) ci = 6;   // a handful of input channels: one 16-channel k-step per tap
        const MfmaCfg &c = kCfgs[ci];
        int BM = 32 * c.a * c.wm, BN = 32 * c.b * c.wn;
        if (plan_cfg < 0 && k + 1 < n_try && BM > (g.out_CH + 63) / 64 * 64) continue;   // row tile mostly padding
        MfmaArgs t = g;
        pc_plan_mfma_tiles(&t, BN, ext);
        // too large for LDS (strided or tiny images): fewer images, then fewer rows per tile (idle lanes)
        while ((size_t)t.TI * t.IH * t.IW * (2 * c.kc + 16 + 8) > MF_LDS_MAX) {
            if (t.TI > 1) --t.TI;
            else if (t.TH > 1) {
                t.TH = (t.TH + 1) / 2;
                t.IH = (t.TH - 1) * t.lstep + ext;
                t.tiles_y = (t.GH + t.TH - 1) / t.TH;
            } else break;
        }
        size_t lds = (size_t)t.TI * t.IH * t.IW * (2 * c.kc + 16 + 8);
        if (lds > MF_LDS_MAX) continue;
        t.nchunks = (g.in_CH + c.kc - 1) / c.kc;
        int64_t blocks = (int64_t)((t.N + t.TI - 1) / t.TI) * t.tiles_y * t.tiles_x * ((g.out_CH + BM - 1) / BM) * (pcl ? 4 : 1);
        int split = 1;
        if (ctx->plan_split > 0) split = ctx->plan_split;
        else if (k == n_try - 1 && blocks <= ctx->num_cu && t.nchunks >= 8) split = 4;
        if (g.oscale != 1 || (g.out_CH & 3)) split = 1;   // parity-class launches share the output; the reduce is 4-wide
        if (split > t.nchunks) split = t.nchunks;
        t.cps = (t.nchunks + split - 1) / split;
        split = (t.nchunks + t.cps - 1) / t.cps;
        pick = ci;
        pick_split = split;
        best = t;
        if (blocks >= want) break;   // enough workgroups to fill the chip: keep the bigger tile
    }
    if (pick < 0) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: no tile configuration fits in LDS");
    g = best;
    const MfmaCfg &c = kCfgs[pick];
    const int pix_tiles = ((g.N + g.TI - 1) / g.TI) * g.tiles_y * g.tiles_x;
    if (pcl) {
        g.cls_tiles = pix_tiles;
        for (int cl = 0; cl < 4; ++cl) {
            g.cls_GH[cl] = pcl->GH[cl]; g.cls_GW[cl] = pcl->GW[cl];
            g.cls_ooy[cl] = pcl->ooy[cl]; g.cls_oox[cl] = pcl->oox[cl];
            g.cls_ntaps[cl] = pcl->ntaps[cl];
            for (int t = 0; t < 4; ++t) {
                const int u = t < pcl->ntaps[cl] ? t : 0;   // unused entries repeat the first: valid addresses, never multiplied
                g.cls_tap_w[cl][t] = pcl->tap_w[cl][u];
                g.cls_tap_off[cl][t] = (pcl->tr[cl][u] * g.IW + pcl->tc[cl][u]) * (2 * c.kc + 16);
            }
        }
    } else {
        for (int t = 0; t < ntaps; ++t) g.tap_off[t] = (tr[t] * g.IW + tc[t]) * (2 * c.kc + 16);
    }
    int BM = 32 * c.a * c.wm;
    dim3 grid((unsigned)(pix_tiles * (pcl ? 4 : 1)), (unsigned)((g.out_CH + BM - 1) / BM), (unsigned)pick_split);
    size_t lds = (size_t)g.TI * g.IH * g.IW * (2 * c.kc + 16 + 8);
    float *partial = nullptr;
    const int64_t n_out = (int64_t)g.N * g.out_H * g.out_W * g.out_CH;
    if (pick_split > 1) {
        void *scr = nullptr;
        pc_status s = pc_scratch(ctx, sizeof(float) * (size_t)pick_split * (size_t)n_out, &scr);
        if (s != PC_OK) return s;
        partial = (float *)scr;
    }
    switch (pick) {
    case 0: launch_cfg<2, 4, 1, 4, 32>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    case 1: launch_cfg<2, 4, 2, 2, 32>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    case 2: launch_cfg<2, 2, 2, 2, 32>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    case 3: launch_cfg<2, 2, 2, 2, 64>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    case 4: launch_cfg<1, 2, 2, 2, 64>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    case 5: launch_cfg<1, 1, 2, 2, 64>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    default: launch_cfg<1, 2, 2, 2, 16>(ctx->stream, grid, lds, pcl != nullptr, in, out, wz, partial, g); break;
    }
    pc_note_kernel(ctx, "pc_mfma_conv_kernel<%d, %d, %d, %d, %d, %d, %s>", c.a, c.b, c.wm, c.wn, pcl ? 4 : 9, c.kc, pcl ? "true" : "false");
    pc_status s = pc_hip_check(ctx, hipGetLastError(), "MFMA conv launch");
    if (s != PC_OK || pick_split == 1) return s;
    int64_t n4 = n_out / 4;
    hipLaunchKernelGGL(pc_mfma_splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, ctx->stream,
                       (const float4 *)partial, n4, pick_split, (uint2 *)out);
    return pc_hip_check(ctx, hipGetLastError(), "split-K reduce launch");
}

// The first-layer kernels take a launch under the automatic choice or override code 23. A requested ReLU is fused
// into the forward launch; the mask of the backward pass is left to the caller (*fused = false).
static pc_status try_thin(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *in, void *out, bool fwd, int act,
                          bool *fused, bool *taken)
{
    *taken = false;
    if ((ctx->plan_cfg >= 0 && ctx->plan_cfg != 23) || ctx->plan_split != 0) return PC_OK;
    const int act_here = (fwd && fused && act == PC_ACT_RELU) ? PC_ACT_RELU : PC_ACT_NONE;
    const pc_status s = fwd ? pc_thin_fwd(ctx, d, pk, in, out, act_here, taken) : pc_thin_bwd_data(ctx, d, pk, in, out, taken);
    if (s != PC_OK) return s;
    if (*taken && fused) *fused = act != PC_ACT_NONE && act_here == act;
    if (!*taken && ctx->plan_cfg == 23) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: the first-layer kernels do not take this layer");
    return PC_OK;
}

pc_status pc_mfma_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y, int act, bool *fused)
{
    {
        bool taken = false;
        const pc_status s = try_thin(ctx, d, pk, x, y, true, act, fused, &taken);
        if (s != PC_OK || taken) return s;
    }
    MfmaArgs g;
    memset(&g, 0, sizeof(g));
    const int st = d->stride;
    g.N = d->N; g.in_H = d->H; g.in_W = d->W; g.in_CH = d->C;
    g.out_H = (d->H - 1) / st + 1; g.out_W = (d->W - 1) / st + 1; g.out_CH = d->F;
    g.GH = g.out_H; g.GW = g.out_W; g.oscale = 1;
    g.iscale = st; g.ioff_y = g.ioff_x = -1; g.lstep = st;
    g.KS = pk->v.Ck / 16;
    int tr[9], tc[9];
    for (int t = 0; t < 9; ++t) { g.tap_w[t] = t; tr[t] = t / 3; tc[t] = t % 3; }
    const SparseOperand sp = {pk->v.ws_fwd_val, pk->v.ws_fwd_idx, pk->v.ws_fwd_flag, pk->v.ov_fwd_cnt, pk->v.ov_fwd_a, pk->v.ov_fwd_col};
    return run_mfma_conv(ctx, g, 3, 9, tr, tc, (const uint16_t *)x, (uint16_t *)y, pk->v.wz_fwd, sp, nullptr, act, nullptr, fused);
}

pc_status pc_mfma_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx, int act,
                           const void *act_mask, bool *fused)
{
    {
        bool taken = false;
        const pc_status s = try_thin(ctx, d, pk, dy, dx, false, act, fused, &taken);
        if (s != PC_OK || taken) return s;
    }
    MfmaArgs g;
    memset(&g, 0, sizeof(g));
    const int st = d->stride;
    g.N = d->N; g.in_H = (d->H - 1) / st + 1; g.in_W = (d->W - 1) / st + 1; g.in_CH = d->F;
    g.out_H = d->H; g.out_W = d->W; g.out_CH = d->C;
    g.KS = pk->v.Fk / 16;
    g.lstep = 1; g.iscale = 1;
    int tr[9], tc[9];
    const SparseOperand sp = {pk->v.ws_bwd_val, pk->v.ws_bwd_idx, pk->v.ws_bwd_flag, pk->v.ov_bwd_cnt, pk->v.ov_bwd_a, pk->v.ov_bwd_col};
    if (st == 1) {
        g.GH = d->H; g.GW = d->W; g.oscale = 1; g.ioff_y = g.ioff_x = -1;
        for (int t = 0; t < 9; ++t) { g.tap_w[t] = t; tr[t] = 2 - t / 3; tc[t] = 2 - t % 3; }
        return run_mfma_conv(ctx, g, 3, 9, tr, tc, (const uint16_t *)dy, (uint16_t *)dx, pk->v.wz_bwd, sp, nullptr, act,
                             (const uint16_t *)act_mask, fused);
    }
    // stride 2: input pixel (iy, ix) of parity class (py, px) = (iy % 2, ix % 2) receives the taps (r, s) with
    // (py + 1 - r) and (px + 1 - s) even, from output pixel ((iy + 1 - r) / 2, (ix + 1 - s) / 2). One launch takes
    // all four classes, the one with 4 taps first.
    ParityClasses pcl;
    memset(&pcl, 0, sizeof(pcl));
    static const int order[4][2] = {{1, 1}, {1, 0}, {0, 1}, {0, 0}};
    for (int cl = 0; cl < 4; ++cl) {
        const int py = order[cl][0], px = order[cl][1];
        pcl.GH[cl] = (d->H - py + 1) / 2;
        pcl.GW[cl] = (d->W - px + 1) / 2;
        pcl.ooy[cl] = py; pcl.oox[cl] = px;
        int nt = 0;
        for (int t = 0; t < 9; ++t) {
            const int r = t / 3, s = t % 3;
            if ((py + 1 - r) % 2 == 0 && (px + 1 - s) % 2 == 0) {
                pcl.tap_w[cl][nt] = t; pcl.tr[cl][nt] = (py + 1 - r) / 2; pcl.tc[cl][nt] = (px + 1 - s) / 2;
                ++nt;
            }
        }
        pcl.ntaps[cl] = nt;
    }
    g.GH = (d->H + 1) / 2; g.GW = (d->W + 1) / 2;
    g.oscale = 2; g.ioff_y = g.ioff_x = 0;
    return run_mfma_conv(ctx, g, 2, 4, nullptr, nullptr, (const uint16_t *)dy, (uint16_t *)dx, pk->v.wz_bwd, sp, &pcl);
}

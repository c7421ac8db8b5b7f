// Vector-ALU variant of the three passes (Section 5.2): only the kept taps are multiplied.
//
// Forward and backward-data share one kernel: a workgroup stages an input halo tile in LDS
// (channel-planar, float32), every wavefront owns one output channel at a time, every lane a strip
// of 4 output pixels. The kept kernels of that output channel are walked pattern group by pattern
// group: inside a group the 4 LDS tap offsets are wave-uniform scalars, channel index and weights
// come from scalar loads, so all 64 lanes do identical work on different pixels.
// Backward-data is the same gather over the channel-major table with the taps rotated by 180
// degrees (delta (*) rot180(W)); for stride 2 the input pixels are split in 4 parity classes,
// each with the subset of taps that reaches it.
//
// Backward-weight assigns one lane to one kept kernel (4 private float32 sums, no cross-lane
// reduction), walks pixel tiles staged in LDS, writes per-tile-group partial sums and reduces
// them in a fixed order (deterministic, no float atomics).
#include "pc_internal.h"

#define VS 4          // output pixels per lane strip
#define VOB 16        // output channels per workgroup
#define VTILE_FLOATS 11776   // LDS floats available for the input tile (the rest holds the output tile)

struct GatherArgs {
    int32_t N;
    int32_t in_H, in_W, in_CH;
    int32_t out_H, out_W, out_CH;
    int32_t GH, GW;                    // extent of the pixel grid this launch covers
    int32_t oscale, ooff_y, ooff_x;    // output pixel = grid * oscale + ooff
    int32_t iscale, ioff_y, ioff_x;    // input tile origin = tile grid origin * iscale + ioff
    int32_t TI, TH, TSX;               // tile: images, rows, strips per row
    int32_t IH, IW, IWp, plane;        // input tile rows, cols, padded row pitch, padded channel plane
    int32_t CC;                        // channels staged per pass
    int32_t tiles_y, tiles_x;
    int32_t P;
    int16_t tapoff[PC_MAX_P][4];       // LDS offset of each kept tap of a pattern, -1 = tap does not apply
};

template <typename T, int LSTEP>
__global__ void __launch_bounds__(256)
pc_gather_conv_kernel(const T *__restrict__ in, T *__restrict__ out, GatherArgs g, const int32_t *__restrict__ grp,
                      const uint16_t *__restrict__ idx, const float4 *__restrict__ val)
{
    extern __shared__ float smem[];
    float *tile = smem;
    float *otile = smem + VTILE_FLOATS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    int bt = blockIdx.x;
    const int tx = bt % g.tiles_x; bt /= g.tiles_x;
    const int ty = bt % g.tiles_y; bt /= g.tiles_y;
    const int tn = bt;
    const int ob0 = blockIdx.y * VOB;
    const int TW = g.TSX * VS;
    const int gy0 = ty * g.TH, gx0 = tx * TW;
    const int in_y0 = gy0 * g.iscale + g.ioff_y, in_x0 = gx0 * g.iscale + g.ioff_x;

    const int nstrips = g.TI * g.TH * g.TSX;
    const bool lane_on = lane < nstrips;
    int rem = lane_on ? lane : 0;
    const int l_ti = rem / (g.TH * g.TSX); rem -= l_ti * g.TH * g.TSX;
    const int l_ty = rem / g.TSX;
    const int l_sx = rem - l_ty * g.TSX;
    const int lbase = (l_ti * g.IH + l_ty * LSTEP) * g.IWp + l_sx * VS * LSTEP;

    float acc[VOB / 4][VS];
#pragma unroll
    for (int a = 0; a < VOB / 4; ++a)
#pragma unroll
        for (int i = 0; i < VS; ++i) acc[a][i] = 0.0f;

    const int tile_px = g.TI * g.IH * g.IW;
    for (int c0 = 0; c0 < g.in_CH; c0 += g.CC) {
        const int cc = min(g.CC, g.in_CH - c0);
        __syncthreads();
        for (int e = threadIdx.x; e < tile_px * cc; e += 256) {
            int cl = e % cc;
            int q = e / cc;
            int ix = q % g.IW; q /= g.IW;
            int iy = q % g.IH;
            int ti = q / g.IH;
            int n = tn * g.TI + ti, y = in_y0 + iy, x = in_x0 + ix;
            float v = 0.0f;
            if (n < g.N && y >= 0 && y < g.in_H && x >= 0 && x < g.in_W)
                v = pc_load<T>(in + (((int64_t)n * g.in_H + y) * g.in_W + x) * g.in_CH + c0 + cl);
            tile[cl * g.plane + (ti * g.IH + iy) * g.IWp + ix] = v;
        }
        __syncthreads();
        if (lane_on) {
#pragma unroll
            for (int a = 0; a < VOB / 4; ++a) {
                const int o = ob0 + wave + 4 * a;
                if (o >= g.out_CH) break;
                const int32_t *gr = grp + (int64_t)o * (PC_MAX_P + 1);
                int s_begin = gr[0];
                for (int p = 0; p < g.P; ++p) {
                    const int s_end = gr[p + 1];
                    if (s_end > s_begin) {
                        const int o0 = g.tapoff[p][0], o1 = g.tapoff[p][1], o2 = g.tapoff[p][2], o3 = g.tapoff[p][3];
                        // The slots of a pattern group are ordered by channel: with several channel chunks, start at
                        // the first slot of this chunk (binary search) and stop at the first one past it, instead of
                        // walking the whole group once per chunk.
                        int first = s_begin;
                        if (c0 > 0) {
                            int hi = s_end;
                            while (first < hi) {
                                const int mid = (first + hi) >> 1;
                                if ((int)idx[mid] < c0) first = mid + 1; else hi = mid;
                            }
                        }
                        for (int slot = first; slot < s_end; ++slot) {
                            const int c = idx[slot];
                            if (c >= c0 + cc) break;
                            const float4 w = val[slot];
                            const float *t = tile + (c - c0) * g.plane + lbase;
                            if (o0 >= 0) {
#pragma unroll
                                for (int i = 0; i < VS; ++i) acc[a][i] = fmaf(t[o0 + i * LSTEP], w.x, acc[a][i]);
                            }
                            if (o1 >= 0) {
#pragma unroll
                                for (int i = 0; i < VS; ++i) acc[a][i] = fmaf(t[o1 + i * LSTEP], w.y, acc[a][i]);
                            }
                            if (o2 >= 0) {
#pragma unroll
                                for (int i = 0; i < VS; ++i) acc[a][i] = fmaf(t[o2 + i * LSTEP], w.z, acc[a][i]);
                            }
                            if (o3 >= 0) {
#pragma unroll
                                for (int i = 0; i < VS; ++i) acc[a][i] = fmaf(t[o3 + i * LSTEP], w.w, acc[a][i]);
                            }
                        }
                    }
                    s_begin = s_end;
                }
            }
        }
    }
    // transpose through LDS so that the NHWC store is contiguous over output channels
    if (lane_on) {
#pragma unroll
        for (int a = 0; a < VOB / 4; ++a)
#pragma unroll
            for (int i = 0; i < VS; ++i) otile[(lane * VS + i) * (VOB + 1) + wave + 4 * a] = acc[a][i];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < nstrips * VS * VOB; e += 256) {
        int ol = e % VOB;
        int pl = e / VOB;
        int i = pl % VS;
        int strip = pl / VS;
        int s_ti = strip / (g.TH * g.TSX);
        int r2 = strip - s_ti * g.TH * g.TSX;
        int s_ty = r2 / g.TSX;
        int s_sx = r2 - s_ty * g.TSX;
        int n = tn * g.TI + s_ti, gy = gy0 + s_ty, gx = gx0 + s_sx * VS + i, o = ob0 + ol;
        if (n < g.N && gy < g.GH && gx < g.GW && o < g.out_CH) {
            int oy = gy * g.oscale + g.ooff_y, ox = gx * g.oscale + g.ooff_x;
            pc_store<T>(out + (((int64_t)n * g.out_H + oy) * g.out_W + ox) * g.out_CH + o, otile[pl * (VOB + 1) + ol]);
        }
    }
}

// Tile geometry for a pixel grid of GH x GW, lane step lstep, halo extent ext (3 = full 3x3 reach).
static void plan_tiles(GatherArgs *g, int lstep, int ext)
{
    int TW = (g->GW + VS - 1) / VS * VS;
    if (TW > 32) TW = 32;
    g->TSX = TW / VS;
    g->TH = 64 / g->TSX;
    if (g->TH > g->GH) g->TH = g->GH;
    g->TI = 64 / (g->TSX * g->TH);
    if (g->TI > g->N) g->TI = g->N;
    if (g->TI < 1) g->TI = 1;
    g->IH = (g->TH - 1) * lstep + ext;
    g->IW = (TW - 1) * lstep + ext;
    g->IWp = g->IW;
    while (g->IWp % 4 != 1) ++g->IWp;   // rows of lanes then spread over all LDS banks
    g->plane = (g->TI * g->IH * g->IWp) | 1;
    g->CC = VTILE_FLOATS / g->plane;
    if (g->CC > g->in_CH) g->CC = g->in_CH;
    g->tiles_y = (g->GH + g->TH - 1) / g->TH;
    g->tiles_x = (g->GW + TW - 1) / TW;
}

template <int LSTEP>
static pc_status launch_gather(pc_ctx *ctx, pc_dtype dt, const void *in, void *out, const GatherArgs &g,
                               const int32_t *grp, const uint16_t *idx, const float4 *val)
{
    if (g.CC < 1) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "VALU conv: tile does not fit in LDS");
    int tiles_n = (g.N + g.TI - 1) / g.TI;
    dim3 grid((unsigned)(tiles_n * g.tiles_y * g.tiles_x), (unsigned)((g.out_CH + VOB - 1) / VOB));
    size_t lds = sizeof(float) * (VTILE_FLOATS + 256 * (VOB + 1));
    if (dt == PC_F32)
        hipLaunchKernelGGL((pc_gather_conv_kernel<float, LSTEP>), grid, dim3(256), lds, ctx->stream, (const float *)in,
                           (float *)out, g, grp, idx, val);
    else
        hipLaunchKernelGGL((pc_gather_conv_kernel<uint16_t, LSTEP>), grid, dim3(256), lds, ctx->stream,
                           (const uint16_t *)in, (uint16_t *)out, g, grp, idx, val);
    pc_note_kernel(ctx, "pc_gather_conv_kernel<%s, %d>", dt == PC_F32 ? "float" : "unsigned short", LSTEP);
    return pc_hip_check(ctx, hipGetLastError(), "VALU conv launch");
}

pc_status pc_valu_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y)
{
    GatherArgs g;
    memset(&g, 0, sizeof(g));
    const int st = d->stride;
    const int Ho = (d->H - 1) / st + 1, Wo = (d->W - 1) / st + 1;
    g.N = d->N; g.in_H = d->H; g.in_W = d->W; g.in_CH = d->C;
    g.out_H = Ho; g.out_W = Wo; g.out_CH = d->F;
    g.GH = Ho; g.GW = Wo; g.oscale = 1; g.ooff_y = g.ooff_x = 0;
    g.iscale = st; g.ioff_y = g.ioff_x = -1;
    g.P = pk->v.P;
    plan_tiles(&g, st, 3);
    for (int p = 0; p < g.P; ++p)
        for (int j = 0; j < 4; ++j) {
            int t = pk->taps[p][j];
            g.tapoff[p][j] = (int16_t)((t / 3) * g.IWp + (t % 3));
        }
    const PackView &v = pk->v;
    return st == 1 ? launch_gather<1>(ctx, d->dtype, x, y, g, v.fm_grp, v.fm_c, v.fm_val)
                   : launch_gather<2>(ctx, d->dtype, x, y, g, v.fm_grp, v.fm_c, v.fm_val);
}

pc_status pc_valu_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx)
{
    const int st = d->stride;
    const int Ho = (d->H - 1) / st + 1, Wo = (d->W - 1) / st + 1;
    const PackView &v = pk->v;
    GatherArgs g;
    memset(&g, 0, sizeof(g));
    g.N = d->N; g.in_H = Ho; g.in_W = Wo; g.in_CH = d->F;
    g.out_H = d->H; g.out_W = d->W; g.out_CH = d->C;
    g.P = v.P;
    if (st == 1) {
        // dx[iy,ix] reads dy[iy+1-r, ix+1-s]: tile origin (-1,-1), tap (r,s) at tile offset (2-r, 2-s)
        g.GH = d->H; g.GW = d->W; g.oscale = 1; g.ooff_y = g.ooff_x = 0;
        g.iscale = 1; g.ioff_y = g.ioff_x = -1;
        plan_tiles(&g, 1, 3);
        for (int p = 0; p < g.P; ++p)
            for (int j = 0; j < 4; ++j) {
                int t = pk->taps[p][j];
                g.tapoff[p][j] = (int16_t)((2 - t / 3) * g.IWp + (2 - t % 3));
            }
        return launch_gather<1>(ctx, d->dtype, dy, dx, g, v.cm_grp, v.cm_f, v.cm_val);
    }
    // stride 2: input pixel (2a+py, 2b+px) is reached by tap (r,s) iff py+1-r and px+1-s are even;
    // it then reads dy[a + (py+1-r)/2, b + (px+1-s)/2]. One launch per parity class.
    for (int py = 0; py < 2; ++py)
        for (int px = 0; px < 2; ++px) {
            g.GH = (d->H - py + 1) / 2;
            g.GW = (d->W - px + 1) / 2;
            if (g.GH < 1 || g.GW < 1) continue;
            g.oscale = 2; g.ooff_y = py; g.ooff_x = px;
            g.iscale = 1; g.ioff_y = g.ioff_x = 0;
            plan_tiles(&g, 1, 2);
            for (int p = 0; p < g.P; ++p)
                for (int j = 0; j < 4; ++j) {
                    int t = pk->taps[p][j], r = t / 3, s = t % 3;
                    bool ok = ((py + 1 - r) % 2 == 0) && ((px + 1 - s) % 2 == 0);
                    g.tapoff[p][j] = ok ? (int16_t)(((py + 1 - r) / 2) * g.IWp + (px + 1 - s) / 2) : (int16_t)-1;
                }
            pc_status s = launch_gather<1>(ctx, d->dtype, dy, dx, g, v.cm_grp, v.cm_f, v.cm_val);
            if (s != PC_OK) return s;
        }
    return PC_OK;
}

// ------------------------------------------------------------------ backward-weight
#define WB_TH 8
#define WB_TW 8
#define WB_NF 32               // filters of dy staged per pass
#define WB_X_FLOATS 9728       // LDS floats for the x tile

struct WgradArgs {
    int32_t N, H, W, C, F, Ho, Wo, stride;
    int32_t IH, IW, CC, CCp;
    int32_t tiles_y, tiles_x, n_tiles, G;
    uint8_t taps[PC_MAX_P][4];
};

template <typename T>
__global__ void __launch_bounds__(256)
pc_wgrad_valu_kernel(const T *__restrict__ x, const T *__restrict__ dy, WgradArgs a, PackView v,
                     float4 *__restrict__ partial, int64_t pstride)
{
    __shared__ float xs[WB_X_FLOATS];
    __shared__ float ds[WB_TH * WB_TW * (WB_NF + 1)];
    const int nnzk = v.fm_rowptr[v.F];
    const int s0 = blockIdx.x * 256;
    if (s0 >= nnzk) return;
    const int slot = s0 + threadIdx.x;
    const bool live = slot < nnzk;
    const int f = live ? v.slot_f[slot] : 0;
    const int c = live ? v.fm_c[slot] : 0;
    const int pidv = live ? v.fm_pid[slot] : 0;
    int toff[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int t = a.taps[pidv][j];
        toff[j] = ((t / 3) * a.IW + (t % 3)) * a.CCp;
    }
    const int f_lo = v.slot_f[s0];
    const int f_hi = v.slot_f[min(s0 + 255, nnzk - 1)];
    float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;

    for (int tile = blockIdx.y; tile < a.n_tiles; tile += a.G) {
        int q = tile;
        const int tx = q % a.tiles_x; q /= a.tiles_x;
        const int ty = q % a.tiles_y;
        const int n = q / a.tiles_y;
        const int oy0 = ty * WB_TH, ox0 = tx * WB_TW;
        const int iy0 = oy0 * a.stride - 1, ix0 = ox0 * a.stride - 1;
        for (int c0 = 0; c0 < a.C; c0 += a.CC) {
            const int cc = min(a.CC, a.C - c0);
            __syncthreads();
            for (int e = threadIdx.x; e < a.IH * a.IW * cc; e += 256) {
                int cl = e % cc;
                int qq = e / cc;
                int ix = qq % a.IW, iy = qq / a.IW;
                int yy = iy0 + iy, xx = ix0 + ix;
                float val = 0.0f;
                if (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W)
                    val = pc_load<T>(x + (((int64_t)n * a.H + yy) * a.W + xx) * a.C + c0 + cl);
                xs[qq * a.CCp + cl] = val;
            }
            const bool c_in = live && c >= c0 && c < c0 + cc;
            for (int fr0 = f_lo; fr0 <= f_hi; fr0 += WB_NF) {
                const int nf = min(WB_NF, f_hi - fr0 + 1);
                __syncthreads();
                for (int e = threadIdx.x; e < WB_TH * WB_TW * nf; e += 256) {
                    int fl = e % nf;
                    int pp = e / nf;
                    int oy = oy0 + pp / WB_TW, ox = ox0 + pp % WB_TW;
                    float val = 0.0f;
                    if (oy < a.Ho && ox < a.Wo)
                        val = pc_load<T>(dy + (((int64_t)n * a.Ho + oy) * a.Wo + ox) * a.F + fr0 + fl);
                    ds[pp * (WB_NF + 1) + fl] = val;
                }
                __syncthreads();
                if (c_in && f >= fr0 && f < fr0 + nf) {
                    const float *xb = xs + (c - c0);
                    const float *db = ds + (f - fr0);
                    for (int py = 0; py < WB_TH; ++py)
#pragma unroll
                        for (int px = 0; px < WB_TW; ++px) {
                            float g = db[(py * WB_TW + px) * (WB_NF + 1)];
                            const float *xp = xb + ((py * a.stride) * a.IW + px * a.stride) * a.CCp;
                            acc0 = fmaf(g, xp[toff[0]], acc0);
                            acc1 = fmaf(g, xp[toff[1]], acc1);
                            acc2 = fmaf(g, xp[toff[2]], acc2);
                            acc3 = fmaf(g, xp[toff[3]], acc3);
                        }
                }
            }
        }
    }
    if (live) partial[(int64_t)blockIdx.y * pstride + slot] = make_float4(acc0, acc1, acc2, acc3);
}

// dw[slot] = sum over g of partial[g][slot] in a fixed order: TPS threads per slot each add every TPS-th
// partial (ascending), then one thread adds the TPS sub-sums in order. 256 / TPS consecutive slots per workgroup.
// partial is [G][pstride] float4; the number of live slots is read on the device.
template <int TPS>
__device__ __forceinline__ void pc_wgrad_reduce_body(const float4 *__restrict__ partial, int G, int64_t pstride, int64_t nslots_exact,
                                                     const int32_t *__restrict__ nnzk_dev, float4 *__restrict__ dw, int blk)
{
    constexpr int SPB = 256 / TPS;
    __shared__ float4 sub[TPS > 1 ? TPS : 1][TPS > 1 ? SPB : 1];
    const int nnzk = *nnzk_dev;
    const int q = threadIdx.x % SPB, sg = threadIdx.x / SPB;
    const int64_t slot = (int64_t)blk * SPB + q;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    // A plane holds pstride slots. When that is the exact count the loads need not wait for the count read from
    // the device; when it is the pack's capacity they do, or they would fetch the unused part of every plane.
    if (slot < (pstride == nslots_exact ? pstride : (int64_t)nnzk)) {
        // loads run ahead in groups of 8, the additions keep their order
        int gi = sg;
        for (; gi + 7 * TPS < G; gi += 8 * TPS) {
            float4 p[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) p[u] = partial[(int64_t)(gi + u * TPS) * pstride + slot];
#pragma unroll
            for (int u = 0; u < 8; ++u) { s.x += p[u].x; s.y += p[u].y; s.z += p[u].z; s.w += p[u].w; }
        }
        for (; gi < G; gi += TPS) {
            float4 p = partial[(int64_t)gi * pstride + slot];
            s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w;
        }
    }
    if (TPS == 1) {
        if (slot < nnzk) dw[slot] = s;
        return;
    }
    sub[sg][q] = s;
    __syncthreads();
    if (sg == 0 && slot < nnzk) {
        float4 t = sub[0][q];
        for (int i = 1; i < TPS; ++i) {
            float4 p = sub[i][q];
            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
        }
        dw[slot] = t;
    }
}

template <int TPS>
__global__ void __launch_bounds__(256)
pc_wgrad_reduce_kernel(const float4 *__restrict__ partial, int G, int64_t pstride, int64_t nslots_exact, PackView v,
                       float4 *__restrict__ dw)
{
    pc_wgrad_reduce_body<TPS>(partial, G, pstride, nslots_exact, v.fm_rowptr + v.F, dw, (int)blockIdx.x);
}

// The reductions of several layers in one launch: workgroup b serves workgroup b - blk0[l] of layer l, with that
// layer's number of threads per slot.
struct WgradReduceGroup {
    int32_t n;
    int32_t blk0[PC_REDUCE_GROUP_MAX + 1];
    WgradReduceItem item[PC_REDUCE_GROUP_MAX];
};

__global__ void __launch_bounds__(256) pc_wgrad_reduce_group_kernel(WgradReduceGroup g)
{
    const int l = pc_batch_find(g.blk0, g.n, (int)blockIdx.x);
    const WgradReduceItem &y = g.item[l];
    const int blk = (int)blockIdx.x - g.blk0[l];
    const float4 *pp = reinterpret_cast<const float4 *>(y.partial);
    float4 *out = reinterpret_cast<float4 *>(y.dw);
    if (y.tps == 64) pc_wgrad_reduce_body<64>(pp, y.G, y.pstride, y.exact, y.nnzk_dev, out, blk);
    else if (y.tps == 16) pc_wgrad_reduce_body<16>(pp, y.G, y.pstride, y.exact, y.nnzk_dev, out, blk);
    else if (y.tps == 4) pc_wgrad_reduce_body<4>(pp, y.G, y.pstride, y.exact, y.nnzk_dev, out, blk);
    else pc_wgrad_reduce_body<1>(pp, y.G, y.pstride, y.exact, y.nnzk_dev, out, blk);
}

// items: partial planes, split count G, plane stride, upper bound of the live slots (nslots) per layer; tps and exact
// are filled here. One launch per PC_REDUCE_GROUP_MAX layers.
pc_status pc_launch_wgrad_reduce_group(pc_ctx *ctx, int n, WgradReduceItem *items, const int64_t *nslots, const pc_packed *const *pk)
{
    for (int l0 = 0; l0 < n; l0 += PC_REDUCE_GROUP_MAX) {
        const int m = n - l0 < PC_REDUCE_GROUP_MAX ? n - l0 : PC_REDUCE_GROUP_MAX;
        WgradReduceGroup g;
        memset(&g, 0, sizeof(g));
        g.n = m;
        for (int i = 0; i < m; ++i) {
            WgradReduceItem y = items[l0 + i];
            const pc_packed *p = pk[l0 + i];
            y.exact = p->nnzk >= 0 ? p->nnzk : -1;
            y.nnzk_dev = p->v.fm_rowptr + p->v.F;
            y.tps = y.G >= 128 ? 64 : y.G >= 32 ? 16 : y.G >= 8 ? 4 : 1;      // as in the launch of one layer
            const int spb = 256 / y.tps;
            g.item[i] = y;
            g.blk0[i + 1] = g.blk0[i] + (int32_t)((nslots[l0 + i] + spb - 1) / spb);
        }
        if (g.blk0[m] > 0)
            hipLaunchKernelGGL(pc_wgrad_reduce_group_kernel, dim3((unsigned)g.blk0[m]), dim3(256), 0, ctx->stream, g);
    }
    return pc_hip_check(ctx, hipGetLastError(), "bwd_weight reduce (several layers) launch");
}

// nslots bounds the live slots from above (the exact count when the host knows it, else the pack's capacity)
pc_status pc_launch_wgrad_reduce(pc_ctx *ctx, const float *partial, int G, int64_t pstride, int64_t nslots,
                                 const pc_packed *pk, float *dw)
{
    if (nslots <= 0) return PC_OK;
    const int64_t exact = pk->nnzk >= 0 ? pk->nnzk : -1;   // -1: not known on the host
    const float4 *pp = (const float4 *)partial;
    float4 *out = (float4 *)dw;
    if (G >= 128)
        hipLaunchKernelGGL(pc_wgrad_reduce_kernel<64>, dim3((unsigned)((nslots + 3) / 4)), dim3(256), 0, ctx->stream, pp, G,
                           pstride, exact, pk->v, out);
    else if (G >= 32)
        hipLaunchKernelGGL(pc_wgrad_reduce_kernel<16>, dim3((unsigned)((nslots + 15) / 16)), dim3(256), 0, ctx->stream, pp, G,
                           pstride, exact, pk->v, out);
    else if (G >= 8)
        hipLaunchKernelGGL(pc_wgrad_reduce_kernel<4>, dim3((unsigned)((nslots + 63) / 64)), dim3(256), 0, ctx->stream, pp, G,
                           pstride, exact, pk->v, out);
    else
        hipLaunchKernelGGL(pc_wgrad_reduce_kernel<1>, dim3((unsigned)((nslots + 255) / 256)), dim3(256), 0, ctx->stream, pp, G,
                           pstride, exact, pk->v, out);
    return pc_hip_check(ctx, hipGetLastError(), "bwd_weight reduce launch");
}

pc_status pc_valu_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, const void *dy,
                             float *dw)
{
    // No read-back of the kept-kernel count (the call stays asynchronous and can be captured): the kernels find the
    // live slots on the device; the host sizes the grid and strides the partial planes by the count when an earlier
    // pc_packed_info has it, else by the pack's capacity (workgroups past the live slots return at once).
    const int64_t nnzk = pk->nnzk >= 0 ? pk->nnzk : (int64_t)pk->v.F * pk->v.C;
    if (nnzk == 0) return PC_OK;
    pc_status s = PC_OK;
    WgradArgs a;
    memset(&a, 0, sizeof(a));
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.F = d->F; a.stride = d->stride;
    a.Ho = (d->H - 1) / d->stride + 1;
    a.Wo = (d->W - 1) / d->stride + 1;
    a.IH = (WB_TH - 1) * d->stride + 3;
    a.IW = (WB_TW - 1) * d->stride + 3;
    a.CC = WB_X_FLOATS / (a.IH * a.IW);
    if (a.CC > d->C) a.CC = d->C;
    if (a.CC > 1 && a.CC % 2 == 0 && a.CC * a.IH * a.IW + a.IH * a.IW <= WB_X_FLOATS) a.CCp = a.CC + 1;
    else a.CCp = a.CC;
    a.tiles_y = (a.Ho + WB_TH - 1) / WB_TH;
    a.tiles_x = (a.Wo + WB_TW - 1) / WB_TW;
    a.n_tiles = d->N * a.tiles_y * a.tiles_x;
    memcpy(a.taps, pk->taps, sizeof(a.taps));
    int bx = (int)((nnzk + 255) / 256);
    int G = (4 * ctx->num_cu + bx - 1) / bx;
    if (G > a.n_tiles) G = a.n_tiles;
    if (G < 1) G = 1;
    a.G = G;
    void *scr = nullptr;
    s = pc_scratch(ctx, sizeof(float4) * (size_t)G * (size_t)nnzk, &scr);
    if (s != PC_OK) return s;
    dim3 grid((unsigned)bx, (unsigned)G);
    if (d->dtype == PC_F32)
        hipLaunchKernelGGL((pc_wgrad_valu_kernel<float>), grid, dim3(256), 0, ctx->stream, (const float *)x,
                           (const float *)dy, a, pk->v, (float4 *)scr, nnzk);
    else
        hipLaunchKernelGGL((pc_wgrad_valu_kernel<uint16_t>), grid, dim3(256), 0, ctx->stream, (const uint16_t *)x,
                           (const uint16_t *)dy, a, pk->v, (float4 *)scr, nnzk);
    pc_note_kernel(ctx, "pc_wgrad_valu_kernel<%s>", d->dtype == PC_F32 ? "float" : "unsigned short");
    s = pc_hip_check(ctx, hipGetLastError(), "VALU bwd_weight launch");
    if (s != PC_OK) return s;
    return pc_launch_wgrad_reduce(ctx, (const float *)scr, G, nnzk, nnzk, pk, dw);
}

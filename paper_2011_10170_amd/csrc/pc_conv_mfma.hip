// Matrix-core (MFMA) variant of the passes for bf16 layers (Section 5.2; the per-layer choice
// between the sparse kernel and a dense contraction of Section 5.2/5.4, re-made for CDNA4).
//
// The layer is computed as an implicit GEMM over a tap list,
//     out[pixel, m] = sum_taps sum_k  A_tap[m, k] * in[pixel shifted by tap, k],
// with v_mfma_f32_32x32x16_bf16. A_tap is the hard-pruned weight matrix of one tap (zero at every
// pruned position), pre-arranged at pack time in the register order of the instruction's A operand,
// so wavefronts load it straight from global memory/L2 with one 16-byte load per lane. The input
// halo tile of 32 channels is staged in LDS (pixel-major, 80-byte pitch: conflict-free 16-byte reads)
// and every tap is a constant LDS offset.
//   forward        : in = x,  m = filter,  k = channel, 9 taps at (r, s)
//   backward-data  : in = dy, m = channel, k = filter; stride 1: 9 taps at (2-r, 2-s) (rot180);
//                    stride 2: four parity classes of input pixels with 1, 2, 2 and 4 taps
//   backward-weight: see the second half of this file
//
// Operand layout of v_mfma_f32_32x32x16_bf16 used here: lane l holds row (A) / column (B) l%32 and
// the 8 consecutive k values 8*(l/32)..+7; accumulator register r of lane l is row
// 8*(r/4) + 4*(l/32) + r%4, column l%32.
#include "pc_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define MF_PITCH 80          // LDS bytes per staged pixel: 32 channels of bf16 + 16 bytes of padding
#define MF_LDS_MAX 65536

bool pc_mfma_supports(int F, int C) { return F % 8 == 0 && C % 8 == 0; }

struct MfmaArgs {
    int32_t N, in_H, in_W, in_CH;
    int32_t out_H, out_W, out_CH;
    int32_t GH, GW, oscale, ooff_y, ooff_x;
    int32_t iscale, ioff_y, ioff_x, lstep;
    int32_t TI, TH, TW, IH, IW;
    int32_t tiles_y, tiles_x;
    int32_t KS;              // k-steps of 16 in the packed operand (padded reduction length / 16)
    int32_t tap_w[9];        // weight tap index of every list entry
    int32_t tap_off[9];      // LDS byte offset of every list entry
};

template <int A_T, int B_T, int WAVES_M, int WAVES_N, int NTAPS>
__global__ void __launch_bounds__(256)
pc_mfma_conv_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out, const uint16_t *__restrict__ wz,
                    MfmaArgs g)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int BM = 32 * A_T * WAVES_M;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    int bt = blockIdx.x;
    const int tx = bt % g.tiles_x; bt /= g.tiles_x;
    const int ty = bt % g.tiles_y; bt /= g.tiles_y;
    const int tn = bt;
    const int gy0 = ty * g.TH, gx0 = tx * g.TW;
    const int in_y0 = gy0 * g.iscale + g.ioff_y, in_x0 = gx0 * g.iscale + g.ioff_x;
    const int m0 = blockIdx.y * BM + wm * (32 * A_T);
    const int mt0 = m0 >> 5;
    const int npix = g.TI * g.TH * g.TW;

    int base[B_T];
#pragma unroll
    for (int j = 0; j < B_T; ++j) {
        int q = (wn * B_T + j) * 32 + (lane & 31);
        if (q >= npix) q = npix - 1;
        int ti = q / (g.TH * g.TW);
        int rem = q - ti * g.TH * g.TW;
        int y = rem / g.TW, x = rem - y * g.TW;
        base[j] = ((ti * g.IH + y * g.lstep) * g.IW + x * g.lstep) * MF_PITCH + (lane >> 5) * 16;
    }

    f32x16 acc[A_T][B_T];
#pragma unroll
    for (int i = 0; i < A_T; ++i)
#pragma unroll
        for (int j = 0; j < B_T; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    const int HP = g.TI * g.IH * g.IW;
    const int nchunks = g.KS >> 1;
    for (int ch = 0; ch < nchunks; ++ch) {
        __syncthreads();
        for (int e = threadIdx.x; e < HP * 4; e += 256) {
            int q = e >> 2, part = e & 3;
            int ix = q % g.IW;
            int t2 = q / g.IW;
            int iy = t2 % g.IH;
            int ti = t2 / g.IH;
            int n = tn * g.TI + ti, y = in_y0 + iy, x = in_x0 + ix, c = ch * 32 + part * 8;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (n < g.N && y >= 0 && y < g.in_H && x >= 0 && x < g.in_W && c < g.in_CH)
                v = *reinterpret_cast<const uint4 *>(in + (((int64_t)n * g.in_H + y) * g.in_W + x) * g.in_CH + c);
            *reinterpret_cast<uint4 *>(lds + q * MF_PITCH + part * 16) = v;
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < NTAPS; ++t) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                bf16x8 af[A_T], bfr[B_T];
#pragma unroll
                for (int i = 0; i < A_T; ++i)
                    af[i] = *reinterpret_cast<const bf16x8 *>(
                        wz + ((((int64_t)(mt0 + i) * 9 + g.tap_w[t]) * g.KS + ch * 2 + ks) * 64 + lane) * 8);
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    bfr[j] = *reinterpret_cast<const bf16x8 *>(lds + base[j] + g.tap_off[t] + ks * 32);
#pragma unroll
                for (int i = 0; i < A_T; ++i)
#pragma unroll
                    for (int j = 0; j < B_T; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
            }
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
        if (n >= g.N || gy >= g.GH || gx >= g.GW) continue;
        int oy = gy * g.oscale + g.ooff_y, ox = gx * g.oscale + g.ooff_x;
        uint16_t *op = out + (((int64_t)n * g.out_H + oy) * g.out_W + ox) * g.out_CH;
#pragma unroll
        for (int i = 0; i < A_T; ++i)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                int m = m0 + i * 32 + r4 * 8 + (lane >> 5) * 4;
                if (m < g.out_CH) {
                    uint2 pk;
                    pk.x = (uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 0]) | ((uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 1]) << 16);
                    pk.y = (uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 2]) | ((uint32_t)pc_f32_to_bf16(acc[i][j][r4 * 4 + 3]) << 16);
                    *reinterpret_cast<uint2 *>(op + m) = pk;
                }
            }
    }
}

// ------------------------------------------------------------------ operand tiles
// wz_fwd[mt][tap][ks][lane][8]: mt = filter/32, ks = channel/16; element i of lane l is
// w[f = 32*mt + l%32][c = 16*ks + 8*(l/32) + i][tap], zero when pruned or padded.
// wz_bwd has the roles of filter and channel exchanged (rows = channels, k = filters).
__global__ void __launch_bounds__(256)
pc_pack_tiles_kernel(const float *__restrict__ W, LibArg la, PackView v, int bwd)
{
    const int Mp = bwd ? v.Cp : v.Fp;          // padded row count (multiple of 128)
    const int KS = (bwd ? v.Fk : v.Ck) / 16;   // padded reduction length / 16
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t total = (int64_t)(Mp / 32) * 9 * KS * 64;
    if (idx >= total) return;
    int lane = (int)(idx & 63);
    int64_t r = idx >> 6;
    int ks = (int)(r % KS); r /= KS;
    int tap = (int)(r % 9);
    int mt = (int)(r / 9);
    int m = mt * 32 + (lane & 31);
    int k0 = ks * 16 + (lane >> 5) * 8;
    uint16_t o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int k = k0 + i;
        int f = bwd ? k : m, c = bwd ? m : k;
        uint16_t val = 0;
        if (f < v.F && c < v.C) {
            int slot = v.slot_of[(int64_t)f * v.C + c];
            if (slot >= 0 && (la.mask[v.fm_pid[slot]] >> tap) & 1u)
                val = pc_f32_to_bf16(W[((int64_t)f * v.C + c) * 9 + tap]);
        }
        o[i] = val;
    }
    uint4 pk;
    pk.x = o[0] | ((uint32_t)o[1] << 16);
    pk.y = o[2] | ((uint32_t)o[3] << 16);
    pk.z = o[4] | ((uint32_t)o[5] << 16);
    pk.w = o[6] | ((uint32_t)o[7] << 16);
    reinterpret_cast<uint4 *>(bwd ? v.wz_bwd : v.wz_fwd)[idx] = pk;
}

pc_status pc_launch_pack_tiles(pc_ctx *ctx, pc_packed *pk, const float *W)
{
    PackView v = pk->v;
    LibArg la;
    pc_fill_lib(&la, pk->lib, v.P);
    for (int bwd = 0; bwd < 2; ++bwd) {
        int Mp = bwd ? v.Cp : v.Fp, KS = (bwd ? v.Fk : v.Ck) / 16;
        int64_t total = (int64_t)(Mp / 32) * 9 * KS * 64;
        hipLaunchKernelGGL(pc_pack_tiles_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, ctx->stream, W, la,
                           v, bwd);
    }
    return pc_hip_check(ctx, hipGetLastError(), "pack tiles launch");
}

// ------------------------------------------------------------------ planning and launch
struct MfmaCfg { int a, b, wm, wn; };
static const MfmaCfg kCfgs[] = {{2, 4, 1, 4}, {2, 4, 2, 2}, {2, 2, 2, 2}, {1, 2, 2, 2}, {1, 1, 2, 2}};
static const int kNumCfgs = sizeof(kCfgs) / sizeof(kCfgs[0]);

static void plan_mfma_tiles(MfmaArgs *g, int BN, int ext)
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

template <int A_T, int B_T, int WM, int WN>
static void launch_cfg(hipStream_t st, dim3 grid, size_t lds, int ntaps, const uint16_t *in, uint16_t *out,
                       const uint16_t *wz, const MfmaArgs &g)
{
    switch (ntaps) {
    case 9: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 9>), grid, dim3(256), lds, st, in, out, wz, g); break;
    case 4: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 4>), grid, dim3(256), lds, st, in, out, wz, g); break;
    case 2: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 2>), grid, dim3(256), lds, st, in, out, wz, g); break;
    default: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 1>), grid, dim3(256), lds, st, in, out, wz, g); break;
    }
}

// g holds everything but the tile plan; ext = reach of the tap offsets (3 or 2); tap rows/cols in tr/tc.
static pc_status run_mfma_conv(pc_ctx *ctx, MfmaArgs g, int ext, int ntaps, const int *tr, const int *tc,
                               const uint16_t *in, uint16_t *out, const uint16_t *wz)
{
    int pick = -1;
    MfmaArgs best = g;
    for (int ci = 0; ci < kNumCfgs; ++ci) {
        const MfmaCfg &c = kCfgs[ci];
        int BM = 32 * c.a * c.wm, BN = 32 * c.b * c.wn;
        if (BM > 64 && g.out_CH <= 64) continue;
        MfmaArgs t = g;
        plan_mfma_tiles(&t, BN, ext);
        size_t lds = (size_t)t.TI * t.IH * t.IW * MF_PITCH;
        if (lds > MF_LDS_MAX) continue;
        int64_t blocks = (int64_t)((t.N + t.TI - 1) / t.TI) * t.tiles_y * t.tiles_x * ((g.out_CH + BM - 1) / BM);
        pick = ci;
        best = t;
        if (blocks >= 2 * (int64_t)ctx->num_cu) break;   // enough workgroups to fill the chip: keep the bigger tile
    }
    if (pick < 0) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: no tile configuration fits in LDS");
    g = best;
    for (int t = 0; t < ntaps; ++t) g.tap_off[t] = (tr[t] * g.IW + tc[t]) * MF_PITCH;
    const MfmaCfg &c = kCfgs[pick];
    int BM = 32 * c.a * c.wm;
    dim3 grid((unsigned)(((g.N + g.TI - 1) / g.TI) * g.tiles_y * g.tiles_x), (unsigned)((g.out_CH + BM - 1) / BM));
    size_t lds = (size_t)g.TI * g.IH * g.IW * MF_PITCH;
    switch (pick) {
    case 0: launch_cfg<2, 4, 1, 4>(ctx->stream, grid, lds, ntaps, in, out, wz, g); break;
    case 1: launch_cfg<2, 4, 2, 2>(ctx->stream, grid, lds, ntaps, in, out, wz, g); break;
    case 2: launch_cfg<2, 2, 2, 2>(ctx->stream, grid, lds, ntaps, in, out, wz, g); break;
    case 3: launch_cfg<1, 2, 2, 2>(ctx->stream, grid, lds, ntaps, in, out, wz, g); break;
    default: launch_cfg<1, 1, 2, 2>(ctx->stream, grid, lds, ntaps, in, out, wz, g); break;
    }
    return pc_hip_check(ctx, hipGetLastError(), "MFMA conv launch");
}

pc_status pc_mfma_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y)
{
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
    return run_mfma_conv(ctx, g, 3, 9, tr, tc, (const uint16_t *)x, (uint16_t *)y, pk->v.wz_fwd);
}

pc_status pc_mfma_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx)
{
    MfmaArgs g;
    memset(&g, 0, sizeof(g));
    const int st = d->stride;
    g.N = d->N; g.in_H = (d->H - 1) / st + 1; g.in_W = (d->W - 1) / st + 1; g.in_CH = d->F;
    g.out_H = d->H; g.out_W = d->W; g.out_CH = d->C;
    g.KS = pk->v.Fk / 16;
    g.lstep = 1; g.iscale = 1;
    int tr[9], tc[9];
    if (st == 1) {
        g.GH = d->H; g.GW = d->W; g.oscale = 1; g.ioff_y = g.ioff_x = -1;
        for (int t = 0; t < 9; ++t) { g.tap_w[t] = t; tr[t] = 2 - t / 3; tc[t] = 2 - t % 3; }
        return run_mfma_conv(ctx, g, 3, 9, tr, tc, (const uint16_t *)dy, (uint16_t *)dx, pk->v.wz_bwd);
    }
    for (int py = 0; py < 2; ++py)
        for (int px = 0; px < 2; ++px) {
            g.GH = (d->H - py + 1) / 2;
            g.GW = (d->W - px + 1) / 2;
            if (g.GH < 1 || g.GW < 1) continue;
            g.oscale = 2; g.ooff_y = py; g.ooff_x = px; g.ioff_y = g.ioff_x = 0;
            int nt = 0;
            for (int t = 0; t < 9; ++t) {
                int r = t / 3, s = t % 3;
                if ((py + 1 - r) % 2 == 0 && (px + 1 - s) % 2 == 0) {
                    g.tap_w[nt] = t; tr[nt] = (py + 1 - r) / 2; tc[nt] = (px + 1 - s) / 2;
                    ++nt;
                }
            }
            pc_status s = run_mfma_conv(ctx, g, 2, nt, tr, tc, (const uint16_t *)dy, (uint16_t *)dx, pk->v.wz_bwd);
            if (s != PC_OK) return s;
        }
    return PC_OK;
}

// ------------------------------------------------------------------ backward-weight
// dW[t][f][c] = sum over output pixels of dy[pixel][f] * x[pixel shifted by tap t][c]: for every tap a
// GEMM with M = filters, N = channels and the pixels as the reduction. Both operands need the pixels
// contiguous per lane, while NHWC memory has the channels contiguous, so the staging transposes:
// LDS holds dyT[filter][pixel] and xT[channel][row][column] (bf16). One workgroup owns a 64x64 tile of
// (filter, channel) for all 9 taps (each wave 32x32x9: 144 accumulator registers) and walks pixel tiles
// of R rows x TWp columns of one image. The three horizontal taps of a kernel row come from ONE aligned
// LDS read plus its two neighbouring dwords, re-aligned in registers with v_alignbit. Pixel tiles are
// split over blockIdx.z; every split writes only the kept taps, in compact slot order, to its own
// partial buffer, and a second kernel adds the partials in a fixed order (no float atomics).
#define WG_T 64                // filters and channels per workgroup
#define WG_DY_PITCH 144        // bytes per filter row of dyT: 64 pixels of bf16 + 16 bytes of padding

struct WgradMfmaArgs {
    int32_t N, H, W, C, F, Ho, Wo;
    int32_t TWp, R;            // pixel tile: R rows x TWp columns (TWp % 8 == 0, R*TWp % 16 == 0, <= 64)
    int32_t xrow;              // elements per xT row: TWp + 16 (column index = halo column + 7)
    int32_t xplane;            // bytes per xT channel plane
    int32_t tiles_r, tiles_c, n_ktiles, ksplit;
    int32_t nnzk;
    uint8_t taps[PC_MAX_P][4];
};

__device__ __forceinline__ bf16x8 pc_as_bf16x8(uint32_t a, uint32_t b, uint32_t c, uint32_t d)
{
    uint4 v = make_uint4(a, b, c, d);
    return __builtin_bit_cast(bf16x8, v);
}

__global__ void __launch_bounds__(256)
pc_mfma_wgrad_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dy, WgradMfmaArgs a, PackView v,
                     float *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *dyT = lds;
    unsigned char *xT = lds + WG_T * WG_DY_PITCH;
    __shared__ int8_t jmap[PC_MAX_P][9];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int fh = wave & 1, chh = wave >> 1;
    const int c0 = blockIdx.x * WG_T, f0 = blockIdx.y * WG_T;
    const int g = lane >> 5;

    for (int e = threadIdx.x; e < v.P * 9; e += 256) (&jmap[0][0])[e] = -1;
    __syncthreads();
    for (int e = threadIdx.x; e < v.P * 4; e += 256) jmap[e >> 2][a.taps[e >> 2][e & 3]] = (int8_t)(e & 3);

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    const int nks = (a.R * a.TWp) >> 4;
    const int hw = a.TWp + 2;
    const unsigned char *a_base = dyT + (fh * 32 + (lane & 31)) * WG_DY_PITCH + g * 16;
    const unsigned char *b_base = xT + (chh * 32 + (lane & 31)) * a.xplane;

    for (int kt = blockIdx.z; kt < a.n_ktiles; kt += a.ksplit) {
        int q = kt;
        const int tc = q % a.tiles_c; q /= a.tiles_c;
        const int tr = q % a.tiles_r;
        const int n = q / a.tiles_r;
        const int oy0 = tr * a.R, ox0 = tc * a.TWp;
        __syncthreads();
        // dy tile, transposed to [filter][pixel]
        for (int e = threadIdx.x; e < a.R * a.TWp * 8; e += 256) {
            int fg = e & 7, p = e >> 3;
            int prow = p / a.TWp, pcol = p - prow * a.TWp;
            int oy = oy0 + prow, ox = ox0 + pcol, f = f0 + fg * 8;
            uint4 val = make_uint4(0u, 0u, 0u, 0u);
            if (oy < a.Ho && ox < a.Wo && f < a.F)
                val = *reinterpret_cast<const uint4 *>(dy + (((int64_t)n * a.Ho + oy) * a.Wo + ox) * a.F + f);
            uint16_t *dst = reinterpret_cast<uint16_t *>(dyT + (fg * 8) * WG_DY_PITCH) + p;
            const uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                dst[(2 * j) * (WG_DY_PITCH / 2)] = (uint16_t)(w[j] & 0xFFFFu);
                dst[(2 * j + 1) * (WG_DY_PITCH / 2)] = (uint16_t)(w[j] >> 16);
            }
        }
        // x halo tile, transposed to [channel][row][column + 7]
        for (int e = threadIdx.x; e < (a.R + 2) * hw * 8; e += 256) {
            int cg = e & 7, p = e >> 3;
            int hy = p / hw, hx = p - hy * hw;
            int yy = oy0 - 1 + hy, xx = ox0 - 1 + hx, c = c0 + cg * 8;
            uint4 val = make_uint4(0u, 0u, 0u, 0u);
            if (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W && c < a.C)
                val = *reinterpret_cast<const uint4 *>(x + (((int64_t)n * a.H + yy) * a.W + xx) * a.C + c);
            unsigned char *dstb = xT + (cg * 8) * a.xplane + (hy * a.xrow + hx + 7) * 2;
            const uint32_t w[4] = {val.x, val.y, val.z, val.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                *reinterpret_cast<uint16_t *>(dstb + (2 * j) * a.xplane) = (uint16_t)(w[j] & 0xFFFFu);
                *reinterpret_cast<uint16_t *>(dstb + (2 * j + 1) * a.xplane) = (uint16_t)(w[j] >> 16);
            }
        }
        __syncthreads();
        for (int kk = 0; kk < nks; ++kk) {
            const bf16x8 af = *reinterpret_cast<const bf16x8 *>(a_base + kk * 32);
            const int p = kk * 16 + g * 8;
            const int prow = p / a.TWp, pcol = p - prow * a.TWp;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const unsigned char *bp = b_base + ((prow + r) * a.xrow + pcol + 8) * 2;
                const uint32_t dm = *reinterpret_cast<const uint32_t *>(bp - 4);
                const uint4 d = *reinterpret_cast<const uint4 *>(bp);
                const uint32_t dp = *reinterpret_cast<const uint32_t *>(bp + 16);
                const uint32_t s01 = __builtin_amdgcn_alignbit(d.y, d.x, 16);
                const uint32_t s12 = __builtin_amdgcn_alignbit(d.z, d.y, 16);
                const uint32_t s23 = __builtin_amdgcn_alignbit(d.w, d.z, 16);
                const bf16x8 b0 = pc_as_bf16x8(__builtin_amdgcn_alignbit(d.x, dm, 16), s01, s12, s23);
                const bf16x8 b1 = pc_as_bf16x8(d.x, d.y, d.z, d.w);
                const bf16x8 b2 = pc_as_bf16x8(s01, s12, s23, __builtin_amdgcn_alignbit(dp, d.w, 16));
                acc[3 * r + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b0, acc[3 * r + 0], 0, 0, 0);
                acc[3 * r + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b1, acc[3 * r + 1], 0, 0, 0);
                acc[3 * r + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b2, acc[3 * r + 2], 0, 0, 0);
            }
        }
    }
    // kept taps only, compact slot order
    const int c = c0 + chh * 32 + (lane & 31);
    float *pout = partial + (int64_t)blockIdx.z * a.nnzk * 4;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int f = f0 + fh * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
        if (f < a.F && c < a.C) {
            const int slot = v.slot_of[(int64_t)f * a.C + c];
            if (slot >= 0) {
                const int8_t *jm = jmap[v.fm_pid[slot]];
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int j = jm[t];
                    if (j >= 0) pout[(int64_t)slot * 4 + j] = acc[t][i];
                }
            }
        }
    }
}

pc_status pc_mfma_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, const void *dy,
                             float *dw)
{
    if (d->stride != 1) return pc_valu_bwd_weight(ctx, d, pk, x, dy, dw);   // stride-2 contraction not built yet
    int64_t nnzk = 0;
    pc_status s = pc_packed_info(ctx, pk, &nnzk, nullptr);
    if (s != PC_OK) return s;
    if (nnzk == 0) return PC_OK;
    WgradMfmaArgs a;
    memset(&a, 0, sizeof(a));
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.F = d->F; a.Ho = d->H; a.Wo = d->W;
    int ntc = (a.Wo + 31) / 32;
    int tw = (a.Wo + ntc - 1) / ntc;
    a.TWp = (tw + 7) / 8 * 8;
    a.R = (64 / a.TWp) & ~1;
    int ho2 = (a.Ho + 1) & ~1;
    if (a.R > ho2) a.R = ho2;
    a.xrow = a.TWp + 16;
    a.xplane = (a.R + 2) * a.xrow * 2 + 16;
    a.tiles_c = (a.Wo + a.TWp - 1) / a.TWp;
    a.tiles_r = (a.Ho + a.R - 1) / a.R;
    a.n_ktiles = d->N * a.tiles_r * a.tiles_c;
    a.nnzk = (int32_t)nnzk;
    memcpy(a.taps, pk->taps, sizeof(a.taps));
    int ft = (a.F + WG_T - 1) / WG_T, ct = (a.C + WG_T - 1) / WG_T;
    int ks = (2 * ctx->num_cu + ft * ct - 1) / (ft * ct);
    if (ks > a.n_ktiles) ks = a.n_ktiles;
    if (ks < 1) ks = 1;
    a.ksplit = ks;
    void *scr = nullptr;
    s = pc_scratch(ctx, sizeof(float) * 4 * (size_t)ks * (size_t)nnzk, &scr);
    if (s != PC_OK) return s;
    size_t lds = (size_t)WG_T * WG_DY_PITCH + (size_t)WG_T * a.xplane;
    hipLaunchKernelGGL(pc_mfma_wgrad_kernel, dim3((unsigned)ct, (unsigned)ft, (unsigned)ks), dim3(256), lds, ctx->stream,
                       (const uint16_t *)x, (const uint16_t *)dy, a, pk->v, (float *)scr);
    s = pc_hip_check(ctx, hipGetLastError(), "MFMA bwd_weight launch");
    if (s != PC_OK) return s;
    return pc_launch_wgrad_reduce(ctx, (const float *)scr, ks, pk, dw);
}

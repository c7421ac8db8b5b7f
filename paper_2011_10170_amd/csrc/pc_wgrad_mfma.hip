// Backward-weight on the matrix cores (bf16 layers): dW at the kept taps only, in compact slot order
// (Section 5.3: only the kept positions are needed).
#include "pc_mfma.h"

// ------------------------------------------------------------------ backward-weight
// dW[t][f][c] = sum over output pixels of dy[pixel][f] * x[pixel shifted by tap t][c]: for every tap a
// GEMM with M = filters, N = channels and the pixels as the reduction. Both MFMA operands need 8
// reduction indices contiguous per lane, while NHWC memory has the channels contiguous. The reduction
// is therefore ordered (spatial position, image) with the image index fastest in groups of 8: a lane's
// 8 values are the same pixel and channel of 8 consecutive images, every tap is just another spatial
// position (a different 16-byte slot, always aligned), and the zero padding is a zero slot.
// LDS holds dyT[filter][slot][8 images] and xT[channel][slot][8 images] (bf16); the staging loads the
// 8 images of a (position, 8 channels) task with eight 16-byte loads, transposes 8x8 in registers
// (v_perm) and writes eight 16-byte rows. Every group of 8 channel planes is shifted by 16 bytes so that
// both the transposing writes and the fragment reads are free of bank conflicts while every fragment
// address stays (per-lane base) + (wave-uniform offset).
// One workgroup owns a 64x64 tile of (filter, channel) for all 9 taps (each wave 32x32x9: 144
// accumulator registers) and walks pixel tiles; pixel tiles are split over blockIdx.z; every split
// writes only the kept taps, in compact slot order, to its own partial buffer, and a second kernel adds
// the partials in a fixed order (no float atomics).
#define WG_T 64                // filters and channels per workgroup
#define WG_NSLOT 32            // dy slots per pixel tile (16 MFMA k-steps)
#define WG_XTASKS 3            // x staging tasks per thread at most (x slots <= 96)
#define WG_DY_PLANE (WG_NSLOT * 16 + 16)
#define WG_LDS_MAX (144 * 1024)

struct WgradMfmaArgs {
    int32_t N, H, W, C, F, Ho, Wo, stride;
    int32_t TR, TC, npos, ng;  // pixel tile: ng groups of 8 images x (TR x TC output positions)
    int32_t IR, IC, xs_per_g;  // x region per image group: IR x IC positions
    int32_t xslots;            // ng * xs_per_g rounded up to a multiple of 8
    int32_t xplane;            // bytes per xT channel plane
    int32_t nks;               // MFMA k-steps per pixel tile: ceil(ng * npos / 2)
    int32_t tiles_r, tiles_c, tiles_n, n_ktiles, ksplit;
    int32_t pstride;       // slots per partial plane
    // decode tables built on the host (no integer divisions in the kernel); 0xFFFFFFFF = unused entry
    int16_t xb_tab[WG_NSLOT];              // x slot read by dy slot s for tap (0,0)
    uint32_t dy_tab[WG_NSLOT];             // dy slot -> (image group << 16) | (row << 8) | column of the output position
    uint32_t x_tab[32 * WG_XTASKS];        // x slot  -> (image group << 16) | (row << 8) | column inside the x region
};

// 8 rows (images) of 8 bf16 (channels) -> 8 rows (channels) of 8 bf16 (images), row j stored at dst + j*pitch
__device__ __forceinline__ void pc_transpose8x8_store(const uint4 (&r)[8], unsigned char *dst, int pitch)
{
    const uint32_t in[8][4] = {{r[0].x, r[0].y, r[0].z, r[0].w}, {r[1].x, r[1].y, r[1].z, r[1].w},
                               {r[2].x, r[2].y, r[2].z, r[2].w}, {r[3].x, r[3].y, r[3].z, r[3].w},
                               {r[4].x, r[4].y, r[4].z, r[4].w}, {r[5].x, r[5].y, r[5].z, r[5].w},
                               {r[6].x, r[6].y, r[6].z, r[6].w}, {r[7].x, r[7].y, r[7].z, r[7].w}};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint4 lo, hi;
        lo.x = __builtin_amdgcn_perm(in[1][d], in[0][d], 0x05040100u);
        lo.y = __builtin_amdgcn_perm(in[3][d], in[2][d], 0x05040100u);
        lo.z = __builtin_amdgcn_perm(in[5][d], in[4][d], 0x05040100u);
        lo.w = __builtin_amdgcn_perm(in[7][d], in[6][d], 0x05040100u);
        *reinterpret_cast<uint4 *>(dst + (2 * d) * pitch) = lo;
        hi.x = __builtin_amdgcn_perm(in[1][d], in[0][d], 0x07060302u);
        hi.y = __builtin_amdgcn_perm(in[3][d], in[2][d], 0x07060302u);
        hi.z = __builtin_amdgcn_perm(in[5][d], in[4][d], 0x07060302u);
        hi.w = __builtin_amdgcn_perm(in[7][d], in[6][d], 0x07060302u);
        *reinterpret_cast<uint4 *>(dst + (2 * d + 1) * pitch) = hi;
    }
}

// 8 consecutive channels starting at channel c of a pixel row with nch channels; rows whose channel count
// is not a multiple of 8 are not 16-byte aligned and are read by element (zero past the last channel).
__device__ __forceinline__ uint4 pc_load8(const uint16_t *p, int nch, int c)
{
    if ((nch & 7) == 0) return *reinterpret_cast<const uint4 *>(p);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (c + i < nch) w[i >> 1] |= (uint32_t)p[i] << ((i & 1) * 16);
    return make_uint4(w[0], w[1], w[2], w[3]);
}

// One workgroup per CU (up to 512 registers per lane): the global loads of the NEXT pixel tile are in
// flight in registers while the MFMAs of the current one run, and the fragments of the next k-step are
// read from LDS while the 9 MFMAs of the current k-step issue.
template <int NKS>   // MFMA k-steps per pixel tile (dy slots / 2, rounded up to a multiple of 4; unused slots are zero)
__global__ void __launch_bounds__(256, 1)
pc_mfma_wgrad_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dy, WgradMfmaArgs a, PackView v,
                     float *__restrict__ partial)
{
    extern __shared__ __align__(16) unsigned char lds[];
    unsigned char *dyT = lds;
    unsigned char *xT = lds + WG_T * WG_DY_PLANE + 128;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // wave = (channel half, tap group). The 18 (filter half, tap) units of the 64x64x9 tile are split 9/9:
    // tap group 0 holds taps 0..4 of filter half 0 and taps 0..3 of half 1; tap group 1 holds taps 8..4 of
    // half 1 and taps 8..5 of half 0. In both groups unit u < 5 is ("first" half, tap slot u) and unit
    // u >= 5 is ("second" half, tap slot u-5), so a wave reads 2 A and 5 B fragments for 9 MFMAs per k-step.
    const int chh = wave & 1, tg = wave >> 1;
    const int c0 = blockIdx.x * WG_T, f0 = blockIdx.y * WG_T;
    const int g = lane >> 5;

    const int first_half = tg;                                    // filter half of units 0..4
    const int fl = lane & 31, cl = chh * 32 + (lane & 31);
    // (compact slot, pattern mask) of the 16 kernels this thread writes in the epilogue: loaded now so that
    // the look-up latency hides behind the main loop
    uint32_t kinf[2][8];
#pragma unroll
    for (int fh = 0; fh < 2; ++fh)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int p = threadIdx.x + 256 * k;
            const int f = f0 + fh * 32 + (p >> 6), c = c0 + (p & 63);
            kinf[fh][k] = (f < a.F && c < a.C) ? v.kinfo[(int64_t)f * a.C + c] : 0xFFFFFFFFu;
        }

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;

    // plane p (a filter of dyT, a channel of xT) starts at p * plane + (p >> 3) * 16
    const unsigned char *b_col = xT + cl * a.xplane + (cl >> 3) * 16;
    int xb[NKS];
#pragma unroll
    for (int kk = 0; kk < NKS; ++kk) xb[kk] = a.xb_tab[2 * kk + g];
    int toff[5];                                                  // x slot offset of this wave's 5 tap slots
#pragma unroll
    for (int b = 0; b < 5; ++b) {
        const int tap = tg ? 8 - b : b;
        toff[b] = (tap / 3) * a.IC + (tap % 3);
    }
    const int f_first = fl + (first_half ? 32 : 0), f_second = fl + (first_half ? 0 : 32);
    const unsigned char *a_row0 = dyT + f_first * WG_DY_PLANE + (f_first >> 3) * 16;    // rows of units 0..4
    const unsigned char *a_row1 = dyT + f_second * WG_DY_PLANE + (f_second >> 3) * 16;  // rows of units 5..8

    // staging tasks of this thread: the (slot, channel group) of a task is the same for every pixel tile
    const int tcg = threadIdx.x & 7;                      // group of 8 filters (dy) / channels (x)
    const int d_slot = threadIdx.x >> 3;                  // WG_NSLOT * 8 == 256: one dy task per thread
    const uint32_t d_tab = a.dy_tab[d_slot];
    const bool d_ok = d_tab != 0xFFFFFFFFu;
    const int d_ig = (int)(d_tab >> 16), d_py = (int)((d_tab >> 8) & 255), d_px = (int)(d_tab & 255);
    bool has_x[WG_XTASKS], x_ok[WG_XTASKS];
    int x_slot[WG_XTASKS], x_ig[WG_XTASKS], x_iy[WG_XTASKS], x_ix[WG_XTASKS];
#pragma unroll
    for (int k = 0; k < WG_XTASKS; ++k) {
        const int e = threadIdx.x + 256 * k;
        has_x[k] = e < a.xslots * 8;
        x_slot[k] = e >> 3;
        const uint32_t xt = has_x[k] ? a.x_tab[x_slot[k]] : 0xFFFFFFFFu;
        x_ok[k] = xt != 0xFFFFFFFFu;
        x_ig[k] = (int)(xt >> 16) & 255; x_iy[k] = (int)((xt >> 8) & 255); x_ix[k] = (int)(xt & 255);
    }
    const int64_t dy_img = (int64_t)a.Ho * a.Wo * a.F, x_img = (int64_t)a.H * a.W * a.C;

    uint4 rd[8], rx[WG_XTASKS][8];
    // 8 images of one (position, 8 channels) task: one branch per task, not per load, in the common case
    auto load_task = [&](uint4 (&r)[8], const uint16_t *src, int64_t img, int nch, int ch, bool ok, int nb) {
        if (ok && nb + 8 <= a.N && (nch & 7) == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) r[i] = *reinterpret_cast<const uint4 *>(src + i * img);
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                r[i] = make_uint4(0u, 0u, 0u, 0u);
                if (ok && nb + i < a.N) r[i] = pc_load8(src + i * img, nch, ch);
            }
        }
    };
    auto issue = [&](int kt) {
        int q = kt;
        const int tc = q % a.tiles_c; q /= a.tiles_c;
        const int tr = q % a.tiles_r;
        const int tn = q / a.tiles_r;
        const int oy0 = tr * a.TR, ox0 = tc * a.TC, n0 = tn * a.ng * 8;
        {
            const int oy = oy0 + d_py, ox = ox0 + d_px, f = f0 + tcg * 8, nb = n0 + d_ig * 8;
            const bool ok = d_ok && oy < a.Ho && ox < a.Wo && f < a.F;
            load_task(rd, dy + (int64_t)nb * dy_img + ((int64_t)oy * a.Wo + ox) * a.F + f, dy_img, a.F, f, ok, nb);
        }
#pragma unroll
        for (int k = 0; k < WG_XTASKS; ++k) {
            if (has_x[k]) {
                const int yy = oy0 * a.stride - 1 + x_iy[k], xx = ox0 * a.stride - 1 + x_ix[k];
                const int c = c0 + tcg * 8, nb = n0 + x_ig[k] * 8;
                const bool ok = x_ok[k] && yy >= 0 && yy < a.H && xx >= 0 && xx < a.W && c < a.C;
                load_task(rx[k], x + (int64_t)nb * x_img + ((int64_t)yy * a.W + xx) * a.C + c, x_img, a.C, c, ok, nb);
            }
        }
    };

    int kt = blockIdx.z;
    if (kt < a.n_ktiles) issue(kt);
    for (; kt < a.n_ktiles; kt += a.ksplit) {
        __syncthreads();
        pc_transpose8x8_store(rd, dyT + (tcg * 8) * WG_DY_PLANE + tcg * 16 + (d_slot << 4), WG_DY_PLANE);
#pragma unroll
        for (int k = 0; k < WG_XTASKS; ++k)
            if (has_x[k]) pc_transpose8x8_store(rx[k], xT + (tcg * 8) * a.xplane + tcg * 16 + (x_slot[k] << 4), a.xplane);
        __syncthreads();
        if (kt + a.ksplit < a.n_ktiles) issue(kt + a.ksplit);

        // fragment addresses are recomputed per pixel tile from two opaque per-lane bases: keeping all of
        // them live across the loop would take more registers than the prefetched tile leaves
        int o_a0 = (int)(a_row0 - lds) + g * 16, o_a1 = (int)(a_row1 - lds) + g * 16, o_b = (int)(b_col - lds);
        asm volatile("" : "+v"(o_a0), "+v"(o_a1), "+v"(o_b));
        const unsigned char *ar0 = lds + o_a0, *ar1 = lds + o_a1, *bc = lds + o_b;
        bf16x8 aq[2][2], bq[2][5];
        aq[0][0] = *reinterpret_cast<const bf16x8 *>(ar0);
        aq[0][1] = *reinterpret_cast<const bf16x8 *>(ar1);
#pragma unroll
        for (int b = 0; b < 5; ++b)
            bq[0][b] = *reinterpret_cast<const bf16x8 *>(bc + ((xb[0] + toff[b]) << 4));
#pragma unroll
        for (int kk = 0; kk < NKS; ++kk) {
            const int cur = kk & 1, nxt = cur ^ 1;
            if (kk + 1 < NKS) {
                aq[nxt][0] = *reinterpret_cast<const bf16x8 *>(ar0 + (kk + 1) * 32);
                aq[nxt][1] = *reinterpret_cast<const bf16x8 *>(ar1 + (kk + 1) * 32);
                const unsigned char *bk = bc + (xb[kk + 1 < NKS ? kk + 1 : 0] << 4);
#pragma unroll
                for (int b = 0; b < 5; ++b)
                    bq[nxt][b] = *reinterpret_cast<const bf16x8 *>(bk + (toff[b] << 4));
            }
#pragma unroll
            for (int u = 0; u < 9; ++u)
                acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[cur][u < 5 ? 0 : 1], bq[cur][u < 5 ? u : u - 5],
                                                                 acc[u], 0, 0, 0);
        }
    }
    // Epilogue, one filter half (32 filters) at a time: the waves park their tiles of that half in LDS as
    // out[tap][filter][channel] (float32, 72 KiB), then every thread walks 8 kernels (f, c) of the half and,
    // for the kept ones, gathers the 4 kept taps and writes them as one 16-byte entry in compact slot order.
    float *pout = partial + (int64_t)blockIdx.z * a.pstride * 4;
    float *ot = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int fh = 0; fh < 2; ++fh) {
        __syncthreads();
        const int h = fh == first_half ? 0 : 1;   // this wave's unit range holding filter half fh
#pragma unroll
        for (int b = 0; b < 5; ++b) {
            if (h == 0 || b < 4) {
                const int tap = tg ? 8 - b : b;
                float *tp = ot + (tap * 32) * WG_T + cl;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int fr = 8 * (i >> 2) + 4 * g + (i & 3);
                    // units 0..4 and 5..8 are distinct registers: select without dynamic indexing
                    tp[fr * WG_T] = h == 0 ? acc[b][i] : acc[5 + (b < 4 ? b : 0)][i];
                }
            }
        }
        __syncthreads();
        const uint32_t (&info)[8] = kinf[fh];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int p = threadIdx.x + 256 * k;
            const int fr = p >> 6, cc = p & 63;
            // entry j of a slot is the j-th set bit of the pattern mask: peel the 4 set bits and read those taps
            if (info[k] != 0xFFFFFFFFu) {
                uint32_t m = info[k] & 0x1FFu;
                const float *ob = ot + fr * WG_T + cc;
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = __builtin_ctz(m);
                    m &= m - 1u;
                    o[j] = ob[t * (32 * WG_T)];
                }
                *reinterpret_cast<float4 *>(pout + (int64_t)(info[k] >> 9) * 4) = make_float4(o[0], o[1], o[2], o[3]);
            }
        }
    }
}


// ------------------------------------------------------------------ backward-weight, wave-specialised
// Same arithmetic and LDS planes as the kernel above, re-organised like the forward kernel: wavefronts
// 4..7 load, transpose and write the NEXT pixel tile (16 dy slots: 8 MFMA k-steps) into the other of two
// LDS buffers while wavefronts 0..3 issue the 72 MFMAs of the current one; the loaders' global loads are
// two pixel tiles ahead in registers. All loads are buffer loads whose offset is out of range for
// everything that must read as zero (padding, tile edges, unused slots), so the loader has no branches.
// Every split writes its partial sums in compact slot order; pc_wgrad_reduce_kernel adds them in split
// order. (Letting the last workgroup of a tile add them inside this kernel was slower: data crossing
// the XCDs within a kernel needs device-scope write-through stores and read-through loads, and one
// workgroup waits for those round trips in series.)
#define WS_NSLOT 16
#define WS_NKS (WS_NSLOT / 2)
#define WS_XSLOTS 48
#define WS_DY_PLANE (WS_NSLOT * 16 + 16)
#define WS_LDS_MAX (160 * 1024 - 256)   // dynamic part; the kernel has a few bytes of static LDS too

struct WgradWsArgs {
    int32_t N, H, W, C, F, Ho, Wo, stride;   // C: channels of the x tensor the kernel reads (padded to a multiple of 8)
    int32_t Creal;                           // channels of the layer (row length of the kinfo table)
    int32_t thin;                            // at most 3 channels: the (tap, channel) pairs are the 32 columns of one MFMA tile
    int32_t TR, TC, npos, ng, IR, IC, xs_per_g, xslots, xplane;
    int32_t tiles_r, tiles_c, n_ktiles, ksplit, pstride;
    int32_t buf_bytes;                     // one LDS buffer: dyT planes, then xT planes
    uint32_t x_bytes, dy_bytes;            // tensor sizes (bounds of the buffer loads)
    uint32_t mg_tc, mg_tr;                 // multiply-high constants of the divisions by tiles_c and tiles_r
    uint32_t mg_npos, mg_TC, mg_xs, mg_IC; // and by npos, TC, xs_per_g, IC (slot tables below)
};

// dy slot -> (image group << 16) | (row << 8) | column of the pixel tile; 0xFFFFFFFF = unused
__device__ __forceinline__ uint32_t ws_dy_tab(const WgradWsArgs &a, int sl)
{
    const int ig = (int)pc_udiv((uint32_t)sl, a.mg_npos), pos = sl - ig * a.npos;
    const int py = (int)pc_udiv((uint32_t)pos, a.mg_TC), px = pos - py * a.TC;
    return ig < a.ng ? ((uint32_t)ig << 16) | ((uint32_t)py << 8) | (uint32_t)px : 0xFFFFFFFFu;
}

// x slot read by dy slot sl for tap (0,0)
__device__ __forceinline__ int ws_xb_tab(const WgradWsArgs &a, int sl)
{
    const int ig = (int)pc_udiv((uint32_t)sl, a.mg_npos), pos = sl - ig * a.npos;
    const int py = (int)pc_udiv((uint32_t)pos, a.mg_TC), px = pos - py * a.TC;
    return ig < a.ng ? ig * a.xs_per_g + py * a.stride * a.IC + px * a.stride : 0;
}

// x slot -> (image group << 16) | (row << 8) | column inside the x region; 0xFFFFFFFF = unused
__device__ __forceinline__ uint32_t ws_x_tab(const WgradWsArgs &a, int xs)
{
    const int ig = (int)pc_udiv((uint32_t)xs, a.mg_xs), rem = xs - ig * a.xs_per_g;
    const int r = (int)pc_udiv((uint32_t)rem, a.mg_IC), q = rem - r * a.IC;
    return ig < a.ng ? ((uint32_t)ig << 16) | ((uint32_t)r << 8) | (uint32_t)q : 0xFFFFFFFFu;
}

// lin: index of the workgroup in the layer's grid of gx x gy tiles x ksplit splits (x fastest).
__device__ __forceinline__ void pc_mfma_wgrad_ws_body(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dy,
                                                      const WgradWsArgs &a, const uint32_t *__restrict__ kinfo,
                                                      float *__restrict__ partial, float *__restrict__ dw, int lin, int gx, int gy)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int XT_OFF = WG_T * WS_DY_PLANE + 128;   // xT planes inside a buffer
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups go to the XCDs round-robin by their linear index. The index is re-read so that the workgroups of
    // one XCD share as few pixel splits as possible: each XCD's L2 then fetches its own slice of x and dy once,
    // instead of every XCD fetching all of both.
    int bx = lin % gx, by = (lin / gx) % gy, bz = lin / (gx * gy);
    {
        const int T = gx * gy, ks = a.ksplit;
        const int xcd = lin & 7, r = lin >> 3;
        int tile = -1;
        if ((ks & 7) == 0) {                           // an XCD owns ks/8 splits, all tiles of each
            tile = r % T;
            bz = (r / T) * 8 + xcd;
        } else if (ks < 8 && (8 % ks) == 0 && (T % (8 / ks)) == 0) {   // 8/ks XCDs share a split
            bz = xcd % ks;
            tile = r * (8 / ks) + xcd / ks;
        }
        if (tile >= 0) { bx = tile % gx; by = tile / gx; }
    }
    const int c0 = bx * WG_T, f0 = by * WG_T;
    const int nt = (a.n_ktiles - bz + a.ksplit - 1) / a.ksplit;   // pixel tiles of this workgroup

    // (compact slot, pattern mask) of the 8 kernels this thread writes in the epilogue; requested early (the loaders
    // first request their pixel tiles) so that the look-up latency hides behind the main loop
    uint32_t kinf[2][4];
    auto load_kinfo = [&]() {
#pragma unroll
        for (int fh = 0; fh < 2; ++fh)
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int p = threadIdx.x + 512 * k;
                const int f = f0 + fh * 32 + (p >> 6), c = c0 + (p & 63);
                kinf[fh][k] = (f < a.F && c < a.Creal) ? kinfo[(int64_t)f * a.Creal + c] : 0xFFFFFFFFu;
            }
    };
    float *pout = a.ksplit > 1 ? partial + (int64_t)bz * a.pstride * 4 : dw;
    const float *ot = reinterpret_cast<const float *>(lds);
    // gathers the 4 kept taps of every kept kernel of filter half fh from the parked tiles (half fh at fh * 72 KiB)
    auto gather = [&](int fh) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int p = threadIdx.x + 512 * k;
            const uint32_t info = kinf[fh][k];
            if (info != 0xFFFFFFFFu) {
                uint32_t m = info & 0x1FFu;
                const float *ob = ot + fh * (9 * 32 * WG_T) + (p >> 6) * WG_T + (p & 63);
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = __builtin_ctz(m);
                    m &= m - 1u;
                    if (a.thin) {
                        // parked as [wavefront][filter half][column = tap * channels + channel][filter]: the four
                        // wavefronts' shares of the pixels, added in wavefront order
                        const float *q = ot + (fh * 32 + t * a.Creal + (p & 63)) * 32 + (p >> 6);
                        o[j] = ((q[0] + q[2 * 32 * 32]) + q[4 * 32 * 32]) + q[6 * 32 * 32];
                    } else {
                        o[j] = ob[t * (32 * WG_T)];
                    }
                }
                *reinterpret_cast<float4 *>(pout + (int64_t)(info >> 9) * 4) = make_float4(o[0], o[1], o[2], o[3]);
            }
        }
    };

    if (wave >= 4) {
        // ------------------------------------------------------------ loaders
        const int tl = threadIdx.x - 256;
        const int cg = tl & 7;
        const bool dy0 = wave < 6;                      // task 0 of wavefronts 4,5 is a dy task, of 6,7 an x task
        constexpr uint32_t OOB = 0x80000000u;
        const __amdgpu_buffer_rsrc_t xsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(x), 0, a.x_bytes, 0x00020000);
        const __amdgpu_buffer_rsrc_t src0 = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(dy0 ? dy : x), 0,
                                                                               dy0 ? a.dy_bytes : a.x_bytes, 0x00020000);
        const int dy_img = a.Ho * a.Wo * a.F * 2, x_img = a.H * a.W * a.C * 2;   // bytes per image
        // task 0: slot tl>>3 (dy) or (tl-128)>>3 (x slots 0..15); task 1: x slot 16 + tl>>3 (x slots 16..47)
        const int slot0 = dy0 ? tl >> 3 : (tl - 128) >> 3;
        const int slot1 = 16 + (tl >> 3);
        const uint32_t tab0 = dy0 ? ws_dy_tab(a, slot0) : (slot0 < a.xslots ? ws_x_tab(a, slot0) : 0xFFFFFFFFu);
        const uint32_t tab1 = slot1 < a.xslots ? ws_x_tab(a, slot1) : 0xFFFFFFFFu;
        const int ig0 = (int)(tab0 >> 16) & 255, r0 = (int)(tab0 >> 8) & 255, q0 = (int)tab0 & 255;
        const int ig1 = (int)(tab1 >> 16) & 255, r1 = (int)(tab1 >> 8) & 255, q1 = (int)tab1 & 255;
        const bool chan0 = dy0 ? f0 + cg * 8 < a.F : c0 + cg * 8 < a.C;
        const bool use0 = tab0 != 0xFFFFFFFFu && chan0;
        const bool use1 = tab1 != 0xFFFFFFFFu && c0 + cg * 8 < a.C;
        // byte offset of the task's first image relative to the pixel tile's origin
        const int rel0 = dy0 ? ig0 * 8 * dy_img + ((r0 * a.Wo + q0) * a.F + f0 + cg * 8) * 2
                             : ig0 * 8 * x_img + ((r0 * a.W + q0) * a.C + c0 + cg * 8) * 2;
        const int rel1 = ig1 * 8 * x_img + ((r1 * a.W + q1) * a.C + c0 + cg * 8) * 2;
        const int img0 = dy0 ? dy_img : x_img;
        const int pitch0 = dy0 ? WS_DY_PLANE : a.xplane;
        const int dst0 = (dy0 ? 0 : XT_OFF) + (cg * 8) * pitch0 + cg * 16 + (slot0 << 4);
        const int dst1 = XT_OFF + (cg * 8) * a.xplane + cg * 16 + (slot1 << 4);

        int kt = bz;                                     // next pixel tile to request
        auto issue = [&](uint4 (&A)[8], uint4 (&B)[8]) {
            const bool live = kt < a.n_ktiles;
            const uint32_t u = pc_udiv((uint32_t)kt, a.mg_tc);
            const int tc = kt - (int)u * a.tiles_c;
            const uint32_t tn = pc_udiv(u, a.mg_tr);
            const int tr = (int)u - (int)tn * a.tiles_r;
            const int oy0 = tr * a.TR, ox0 = tc * a.TC, n0 = (int)tn * a.ng * 8;
            const int xy0 = oy0 * a.stride - 1, xx0 = ox0 * a.stride - 1;
            const int org_d = n0 * dy_img + (oy0 * a.Wo + ox0) * a.F * 2;
            const int org_x = n0 * x_img + (xy0 * a.W + xx0) * a.C * 2;
            bool ok0, ok1;
            if (dy0) ok0 = oy0 + r0 < a.Ho && ox0 + q0 < a.Wo;
            else ok0 = (unsigned)(xy0 + r0) < (unsigned)a.H && (unsigned)(xx0 + q0) < (unsigned)a.W;
            ok0 = ok0 && live && use0 && n0 + ig0 * 8 < a.N;
            ok1 = (unsigned)(xy0 + r1) < (unsigned)a.H && (unsigned)(xx0 + q1) < (unsigned)a.W && live && use1 &&
                  n0 + ig1 * 8 < a.N;
            const uint32_t vo0 = ok0 ? (uint32_t)(rel0 + (dy0 ? org_d : org_x)) : OOB;
            const uint32_t vo1 = ok1 ? (uint32_t)(rel1 + org_x) : OOB;
            // images of the task's group that exist (the last group of a batch that is no multiple of 8 is short)
            const int nv0 = a.N - (n0 + ig0 * 8), nv1 = a.N - (n0 + ig1 * 8);
            // (the image offset sits in the scalar offset, which the range check of a buffer load does not see: a
            // short group needs its missing images switched off one by one; a batch of whole groups of 8 does not, and
            // saves a compare and a select per load on a SIMD whose vector issue the MFMA wavefront needs)
            if (a.N & 7) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const v4u32 t0 = __builtin_amdgcn_raw_buffer_load_b128(src0, (int)(i < nv0 ? vo0 : OOB), i * img0, 0);
                    A[i] = make_uint4(t0.x, t0.y, t0.z, t0.w);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const v4u32 t1 = __builtin_amdgcn_raw_buffer_load_b128(xsrc, (int)(i < nv1 ? vo1 : OOB), i * x_img, 0);
                    B[i] = make_uint4(t1.x, t1.y, t1.z, t1.w);
                }
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const v4u32 t0 = __builtin_amdgcn_raw_buffer_load_b128(src0, (int)vo0, i * img0, 0);
                    A[i] = make_uint4(t0.x, t0.y, t0.z, t0.w);
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const v4u32 t1 = __builtin_amdgcn_raw_buffer_load_b128(xsrc, (int)vo1, i * x_img, 0);
                    B[i] = make_uint4(t1.x, t1.y, t1.z, t1.w);
                }
            }
            kt += a.ksplit;
        };
        // a task whose slot lies past the x planes has nowhere to write (every slot inside them is written,
        // with zeros where nothing is loaded)
        const bool in0 = dy0 || slot0 < a.xslots, in1 = slot1 < a.xslots;
        auto put = [&](const uint4 (&A)[8], const uint4 (&B)[8], int bufoff) {
            if (in0) pc_transpose8x8_store(A, lds + bufoff + dst0, pitch0);
            if (in1) pc_transpose8x8_store(B, lds + bufoff + dst1, a.xplane);
        };
        uint4 A0[8], B0[8], A1[8], B1[8];
        issue(A0, B0); issue(A1, B1);
        load_kinfo();
        put(A0, B0, 0);
        __syncthreads();
        issue(A0, B0);
        // tile i: write tile i+1 (register set (i+1)&1) into buffer (i+1)&1, refill the set with tile i+3
        int i = 0;
        // (the scheduling barriers keep the transposes of the next tile, and with them the wait for its data,
        // from being hoisted in front of the workgroup barrier)
        auto sync = [&]() {
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
        };
        for (; i + 2 <= nt; i += 2) {
            put(A1, B1, a.buf_bytes); issue(A1, B1); sync();
            put(A0, B0, 0);           issue(A0, B0); sync();
        }
        if (i < nt) { put(A1, B1, a.buf_bytes); issue(A1, B1); sync(); }
        __syncthreads();
        __syncthreads();
        gather(0);
        gather(1);
    } else if (a.thin) {
        // ------------------------------------------------------------ MFMA wavefronts, at most 3 channels
        // The 9 * C <= 27 (tap, channel) pairs are the columns of ONE 32-column tile: column n of the x operand is
        // channel n % C at the slot of tap n / C, a per-lane slot offset instead of a per-instruction one. Two matrix
        // instructions (the two filter halves) per k-step instead of 36; wavefront w takes k-steps w and w + 4 of
        // every pixel tile and the four partial tiles are added in the epilogue.
        load_kinfo();
        const int g = lane >> 5, n = lane & 31;
        const int ncol = 9 * a.Creal;
        const int tapn = n < ncol ? n / a.Creal : 0, cn = n < ncol ? n - tapn * a.Creal : 0;   // columns past the last: any valid address
        const int toffn = (tapn / 3) * a.IC + (tapn % 3);
        f32x16 acc[2];
#pragma unroll
        for (int fh = 0; fh < 2; ++fh)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[fh][r] = 0.0f;
        int xbq[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) xbq[q] = ws_xb_tab(a, 2 * (wave + 4 * q) + g);
        const int fl = lane & 31;
        const int o_a0 = fl * WS_DY_PLANE + (fl >> 3) * 16 + g * 16;
        const int o_a1 = (fl + 32) * WS_DY_PLANE + ((fl + 32) >> 3) * 16 + g * 16;
        const int o_b = XT_OFF + cn * a.xplane + (cn >> 3) * 16;
        __syncthreads();
        for (int i = 0; i < nt; ++i) {
            const unsigned char *bufp = lds + (i & 1) * a.buf_bytes;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int kk = wave + 4 * q;
                const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(bufp + o_a0 + kk * 32);
                const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(bufp + o_a1 + kk * 32);
                const bf16x8 b = *reinterpret_cast<const bf16x8 *>(bufp + o_b + ((xbq[q] + toffn) << 4));
                acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[0], 0, 0, 0);
                acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[1], 0, 0, 0);
            }
            __syncthreads();
        }
        float *otw = reinterpret_cast<float *>(lds);
        __syncthreads();
#pragma unroll
        for (int fh = 0; fh < 2; ++fh)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int fr = 8 * (i >> 2) + 4 * g + (i & 3);
                otw[((wave * 2 + fh) * 32 + n) * 32 + fr] = acc[fh][i];
            }
        __syncthreads();
        gather(0);
        gather(1);
    } else {
        // ------------------------------------------------------------ MFMA wavefronts
        // wave = (channel half, tap group); the 18 (filter half, tap) units are split 9/9 as in the kernel above
        load_kinfo();
        const int chh = wave & 1, tg = wave >> 1;
        const int g = lane >> 5;
        const int first_half = tg;
        const int fl = lane & 31, cl = chh * 32 + (lane & 31);
        f32x16 acc[9];
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
        int xb[WS_NKS];
#pragma unroll
        for (int kk = 0; kk < WS_NKS; ++kk) xb[kk] = ws_xb_tab(a, 2 * kk + g);
        int toff[5];
#pragma unroll
        for (int b = 0; b < 5; ++b) {
            const int tap = tg ? 8 - b : b;
            toff[b] = (tap / 3) * a.IC + (tap % 3);
        }
        const int f_first = fl + (first_half ? 32 : 0), f_second = fl + (first_half ? 0 : 32);
        const int o_a0 = f_first * WS_DY_PLANE + (f_first >> 3) * 16 + g * 16;
        const int o_a1 = f_second * WS_DY_PLANE + (f_second >> 3) * 16 + g * 16;
        const int o_b = XT_OFF + cl * a.xplane + (cl >> 3) * 16;

        __syncthreads();
        // The fragments of a k-step are read one k-step ahead of its matrix instructions, also across the barrier
        // between two pixel tiles: the last k-step of a tile is multiplied after the barrier, behind the first reads
        // of the next tile, so that the LDS latency at the start of a tile is covered as well.
        bf16x8 aq[2][2], bq[2][5];
        auto read_frags = [&](int i, int kk, int slot) __attribute__((always_inline)) {
            const unsigned char *bufp = lds + (i & 1) * a.buf_bytes;
            aq[slot][0] = *reinterpret_cast<const bf16x8 *>(bufp + o_a0 + kk * 32);
            aq[slot][1] = *reinterpret_cast<const bf16x8 *>(bufp + o_a1 + kk * 32);
            const unsigned char *bk = bufp + o_b + (xb[kk] << 4);
#pragma unroll
            for (int b = 0; b < 5; ++b) bq[slot][b] = *reinterpret_cast<const bf16x8 *>(bk + (toff[b] << 4));
        };
        if (nt > 0) read_frags(0, 0, 0);
        for (int i = 0; i < nt; ++i) {
#pragma unroll
            for (int kk = 0; kk < WS_NKS; ++kk) {
                const int cur = kk & 1, nxt = cur ^ 1;
                if (kk + 1 < WS_NKS) {
                    read_frags(i, kk + 1, nxt);
                } else {
                    __syncthreads();        // the tile's buffer is free; the next tile's is complete
                    if (i + 1 < nt) read_frags(i + 1, 0, nxt);
                }
#pragma unroll
                for (int u = 0; u < 9; ++u)
                    acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[cur][u < 5 ? 0 : 1], bq[cur][u < 5 ? u : u - 5], acc[u], 0, 0, 0);
                // the 7 fragment reads of the next k-step go one by one into the shadow of the MFMAs
#pragma unroll
                for (int u = 0; u < 9; ++u) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                    if (u < 7) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // epilogue: park both filter halves' tiles as out[half][tap][filter][channel] (2 x 72 KiB), then gather
        float *otw = reinterpret_cast<float *>(lds);
        __syncthreads();
#pragma unroll
        for (int fh = 0; fh < 2; ++fh) {
            const int h = fh == first_half ? 0 : 1;
#pragma unroll
            for (int b = 0; b < 5; ++b) {
                if (h == 0 || b < 4) {
                    const int tap = tg ? 8 - b : b;
                    float *tp = otw + fh * (9 * 32 * WG_T) + (tap * 32) * WG_T + cl;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int fr = 8 * (i >> 2) + 4 * g + (i & 3);
                        tp[fr * WG_T] = h == 0 ? acc[b][i] : acc[5 + (b < 4 ? b : 0)][i];
                    }
                }
            }
        }
        __syncthreads();
        gather(0);
        gather(1);
    }
}

__global__ void __launch_bounds__(512, 1)
pc_mfma_wgrad_ws_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dy, WgradWsArgs a,
                        const uint32_t *__restrict__ kinfo, float *__restrict__ partial, float *__restrict__ dw)
{
    const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    pc_mfma_wgrad_ws_body(x, dy, a, kinfo, partial, dw, lin, (int)gridDim.x, (int)gridDim.y);
}

// The layers of a network in one launch (all of them independent once every x and dy exists): workgroup b serves
// workgroup b - blk0[l] of layer l. blk0 entries are multiples of 8, so a layer's workgroups meet the XCDs as
// they would in a launch of their own; the workgroups that pad a layer's count return at once.
#define WS_GROUP_MAX 20
// A grouped launch aims at one workgroup per CU while a workgroup's share stays below PC_GROUP_UNITS (tile,
// pixel tile) units (the prologue and epilogue of a workgroup cost as much as several), then at up to 4 per CU
// (long workgroups: balance matters more). Measured: vgg16_cifar 105 / 113 / 123 us and vgg16_imagenet
// 1017 / 1029 / 915 / 895 us at 1 / 2 / 3 / 4 workgroups per CU; with the threshold at 16 / 32 / 64 units:
// vgg16_cifar 112 / 105 / 106 us, resnet50_imagenet 312 / 312 / 300 us, vgg16_imagenet 910 / 914 / 1030 us.
#ifndef PC_GROUP_UNITS
#define PC_GROUP_UNITS 32
#endif
struct WgradWsLayer {
    WgradWsArgs a;
    const uint16_t *x, *dy;
    const uint32_t *kinfo;
    float *partial, *dw;
    int32_t gx, gy;
};
struct WgradWsGroup {
    int32_t n;
    int32_t blk0[WS_GROUP_MAX + 1];
    WgradWsLayer layer[WS_GROUP_MAX];
};

__global__ void __launch_bounds__(512, 1) pc_mfma_wgrad_ws_group_kernel(WgradWsGroup g)
{
    const int l = pc_batch_find(g.blk0, g.n, (int)blockIdx.x);
    const WgradWsLayer &y = g.layer[l];
    const int lin = (int)blockIdx.x - g.blk0[l];
    if (lin >= y.gx * y.gy * y.a.ksplit) return;
    pc_mfma_wgrad_ws_body(y.x, y.dy, y.a, y.kinfo, y.partial, y.dw, lin, y.gx, y.gy);
}

// Plan of the wave-specialised kernel for one layer; false when the layer is outside what that kernel takes (the
// caller then uses the cooperative kernel). nslots strides the partial planes. *xb = bytes of the channel-padded
// copy of x the kernel reads when *pad_x.
static bool ws_plan(const pc_ctx *ctx, const pc_conv_desc *d, int64_t nslots, WgradWsArgs *out, int *ct_out, int *ft_out,
                    size_t *lds_out, bool *pad_x_out, int64_t *xb_out)
{
    WgradWsArgs a;
    memset(&a, 0, sizeof(a));
    const int st = d->stride;
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = (d->C + 7) / 8 * 8; a.Creal = d->C; a.F = d->F; a.stride = st;
    a.Ho = (d->H - 1) / st + 1; a.Wo = (d->W - 1) / st + 1;
    // 16-byte buffer loads of 8 channels. An input whose channel count is no multiple of 8 (the first layer's 3)
    // is first copied to rows padded to 8 channels; an output-gradient with such a filter count is left to the
    // cooperative kernel, which reads by element.
    if (a.F & 7) return false;
    const bool pad_x = a.C != a.Creal;
    // (override code 11 keeps a first layer on the general form of the kernel)
    a.thin = d->C <= 3 && (ctx->plan_cfg < 0 || ctx->plan_cfg == 23);
    const int64_t xb = (int64_t)a.N * a.H * a.W * a.C * 2, db = (int64_t)a.N * a.Ho * a.Wo * a.F * 2;
    if (xb >= ((int64_t)1 << 31) || db >= ((int64_t)1 << 31)) return false;
    const int ft = (a.F + WG_T - 1) / WG_T, ct = (a.C + WG_T - 1) / WG_T;
    a.x_bytes = (uint32_t)xb; a.dy_bytes = (uint32_t)db;
    int best_tr = 0, best_tc = 0, best_ng = 0;
    double best_eff = -1.0;
    const int ngroups = (a.N + 7) / 8;
    for (int tr = 1; tr <= WS_NSLOT; ++tr)
        for (int tc = 1; tr * tc <= WS_NSLOT; ++tc) {
            if ((tr > a.Ho && tr > 1) || (tc > a.Wo && tc > 1)) continue;
            const int xs1 = ((tr - 1) * st + 3) * ((tc - 1) * st + 3);
            int ngc = WS_NSLOT / (tr * tc);
            if (ngc > ngroups) ngc = ngroups;
            while (ngc > 1 && ngc * xs1 > WS_XSLOTS) --ngc;
            if (ngc * xs1 > WS_XSLOTS) continue;
            const int nr = (a.Ho + tr - 1) / tr, nc = (a.Wo + tc - 1) / tc;
            const double cover = (double)a.Ho * a.Wo / ((double)nr * tr * nc * tc);
            const double fill = (double)(ngc * tr * tc) / WS_NSLOT;
            const double halo = (double)(tr * tc) / xs1;
            const double eff = cover * fill * (0.75 + 0.25 * halo);
            if (eff > best_eff) { best_eff = eff; best_tr = tr; best_tc = tc; best_ng = ngc; }
        }
    if (best_eff < 0.0) return false;
    a.TR = best_tr; a.TC = best_tc; a.npos = a.TR * a.TC; a.ng = best_ng;
    a.IR = (a.TR - 1) * st + 3; a.IC = (a.TC - 1) * st + 3;
    a.xs_per_g = a.IR * a.IC;
    a.xslots = (a.ng * a.xs_per_g + 7) / 8 * 8;
    if (a.xslots > WS_XSLOTS) return false;
    a.xplane = a.xslots * 16 + 16;
    a.tiles_r = (a.Ho + a.TR - 1) / a.TR;
    a.tiles_c = (a.Wo + a.TC - 1) / a.TC;
    const int tiles_n = (ngroups + a.ng - 1) / a.ng;
    const int64_t nkt = (int64_t)tiles_n * a.tiles_r * a.tiles_c;
    if (nkt * (a.tiles_r > a.tiles_c ? a.tiles_r : a.tiles_c) >= ((int64_t)1 << 31)) return false;
    a.n_ktiles = (int)nkt;
    a.pstride = (int32_t)nslots;
    auto magic = [](int dd) { return pc_udiv_magic(dd); };
    a.mg_tc = magic(a.tiles_c); a.mg_tr = magic(a.tiles_r);
    a.mg_npos = magic(a.npos); a.mg_TC = magic(a.TC); a.mg_xs = magic(a.xs_per_g); a.mg_IC = magic(a.IC);
    a.buf_bytes = (WG_T * WS_DY_PLANE + 128 + WG_T * a.xplane + 128 + 255) / 256 * 256;
    size_t lds = 2 * (size_t)a.buf_bytes;
    if (lds < (size_t)2 * 9 * 32 * WG_T * sizeof(float)) lds = (size_t)2 * 9 * 32 * WG_T * sizeof(float);   // the epilogue parks both filter halves
    if (lds > WS_LDS_MAX) return false;
    int ks = ctx->num_cu / (ft * ct);
    if (ks > a.n_ktiles) ks = a.n_ktiles;
    if (ks < 1) ks = 1;
    a.ksplit = ks;
    *out = a;
    *ct_out = ct; *ft_out = ft; *lds_out = lds; *pad_x_out = pad_x; *xb_out = xb;
    return true;
}

static pc_status ws_set_lds_attr(pc_ctx *ctx)
{
    static pc_per_device_once attr;
    if (pc_once_pending(attr, ctx->device)) {
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_ws_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_ws_group_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS_MAX));
        pc_once_done(attr, ctx->device);
    }
    return PC_OK;
}

// Wave-specialised backward-weight of one layer: plan and launch. *launched stays false when the layer is outside
// what that kernel takes.
static pc_status pc_mfma_bwd_weight_ws(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, const void *dy,
                                       float *dw, int64_t nslots, bool *launched)
{
    *launched = false;
    WgradWsArgs a;
    int ct, ft;
    size_t lds;
    bool pad_x;
    int64_t xb;
    if (!ws_plan(ctx, d, nslots, &a, &ct, &ft, &lds, &pad_x, &xb)) return PC_OK;
    const int ks = a.ksplit;
    void *scr = nullptr;
    const size_t part_bytes = ks > 1 ? (sizeof(float) * 4 * (size_t)ks * (size_t)nslots + 255) / 256 * 256 : 0;
    if (part_bytes || pad_x) {
        pc_status s = pc_scratch(ctx, part_bytes + (pad_x ? (size_t)xb : 0), &scr);
        if (s != PC_OK) return s;
    }
    if (pad_x) {
        void *xp = static_cast<unsigned char *>(scr) + part_bytes;
        pc_launch_pad_channels(ctx, (const uint16_t *)x, xp, (int64_t)a.N * a.H * a.W, a.Creal, a.C);
        x = xp;
    }
    pc_status s = ws_set_lds_attr(ctx);
    if (s != PC_OK) return s;
    hipLaunchKernelGGL(pc_mfma_wgrad_ws_kernel, dim3((unsigned)ct, (unsigned)ft, (unsigned)ks), dim3(512), lds, ctx->stream,
                       (const uint16_t *)x, (const uint16_t *)dy, a, pk->v.kinfo, (float *)scr, dw);
    *launched = true;
    pc_note_kernel(ctx, "pc_mfma_wgrad_ws_kernel");
    s = pc_hip_check(ctx, hipGetLastError(), "MFMA bwd_weight (wave-specialised) launch");
    if (s != PC_OK || ks == 1) return s;
    return pc_launch_wgrad_reduce(ctx, (const float *)scr, ks, nslots, nslots, pk, dw);
}

pc_status pc_mfma_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, const void *dy,
                             float *dw)
{
    // The kernels find the kept kernels and their slots on the device; the host only needs an upper bound of
    // the slot count to size and stride the partial planes: the exact count when a read-back has already
    // happened, else the capacity of the pack. No read-back is forced here, so a step that re-packs stays
    // asynchronous.
    const int64_t nslots = pk->nnzk >= 0 ? pk->nnzk : (int64_t)pk->v.F * pk->v.C;
    if (nslots == 0) return PC_OK;
    pc_status s = PC_OK;
    if (ctx->plan_cfg != 10) {   // 10 forces the cooperative kernel
        bool launched = false;
        s = pc_mfma_bwd_weight_ws(ctx, d, pk, x, dy, dw, nslots, &launched);
        if (launched || s != PC_OK) return s;
        if (ctx->plan_cfg == 11)
            return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA bwd_weight: the wave-specialised kernel does not take this layer");
    }
    WgradMfmaArgs a;
    memset(&a, 0, sizeof(a));
    const int st = d->stride;
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.F = d->F; a.stride = st;
    a.Ho = (d->H - 1) / st + 1; a.Wo = (d->W - 1) / st + 1;
    // output region per image group: up to 16 positions at stride 1, 8 at stride 2 (the x region grows 4x)
    const int maxpos = st == 1 ? WG_NSLOT / 2 : WG_NSLOT / 4;   // positions per image group
    int best_tr = 1, best_tc = 1, best_ng = 1;
    double best_eff = -1.0;
    const int ngroups = (a.N + 7) / 8;
    for (int tr = 1; tr <= maxpos; ++tr)
        for (int tc = 1; tr * tc <= maxpos; ++tc) {
            if (tr > a.Ho && tr > 1) continue;
            if (tc > a.Wo && tc > 1) continue;
            const int xs1 = ((tr - 1) * st + 3) * ((tc - 1) * st + 3);
            int ngc = WG_NSLOT / (tr * tc);
            if (ngc > ngroups) ngc = ngroups;
            while (ngc > 1 && ngc * xs1 > 32 * WG_XTASKS) --ngc;
            if (ngc * xs1 > 32 * WG_XTASKS) continue;
            int nr = (a.Ho + tr - 1) / tr, nc = (a.Wo + tc - 1) / tc;
            double cover = (double)a.Ho * a.Wo / ((double)nr * tr * nc * tc);   // useful part of the tiles
            double fill = (double)(ngc * tr * tc) / WG_NSLOT;                    // used dy slots
            double halo = (double)(tr * tc) / xs1;                              // x reuse
            double eff = cover * fill * (0.75 + 0.25 * halo);
            if (eff > best_eff) { best_eff = eff; best_tr = tr; best_tc = tc; best_ng = ngc; }
        }
    if (best_eff < 0.0) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA bwd_weight: no pixel tile fits in LDS");
    a.TR = best_tr; a.TC = best_tc; a.npos = a.TR * a.TC;
    a.ng = best_ng;
    a.IR = (a.TR - 1) * st + 3; a.IC = (a.TC - 1) * st + 3;
    a.xs_per_g = a.IR * a.IC;
    a.xslots = (a.ng * a.xs_per_g + 7) / 8 * 8;
    a.xplane = a.xslots * 16 + 16;
    a.nks = (a.ng * a.npos + 1) / 2;
    a.tiles_r = (a.Ho + a.TR - 1) / a.TR;
    a.tiles_c = (a.Wo + a.TC - 1) / a.TC;
    a.tiles_n = (ngroups + a.ng - 1) / a.ng;
    a.n_ktiles = a.tiles_n * a.tiles_r * a.tiles_c;
    a.pstride = (int32_t)nslots;
    for (int sl = 0; sl < WG_NSLOT; ++sl) {
        int ig = sl / a.npos, pos = sl % a.npos, py = pos / a.TC, px = pos % a.TC;
        bool ok = ig < a.ng;
        a.dy_tab[sl] = ok ? ((uint32_t)ig << 16) | ((uint32_t)py << 8) | (uint32_t)px : 0xFFFFFFFFu;
        a.xb_tab[sl] = ok ? (int16_t)(ig * a.xs_per_g + py * st * a.IC + px * st) : (int16_t)0;
    }
    for (int xs = 0; xs < 32 * WG_XTASKS; ++xs) {
        int ig = xs / a.xs_per_g, rem = xs % a.xs_per_g;
        a.x_tab[xs] = (ig < a.ng) ? ((uint32_t)ig << 16) | ((uint32_t)(rem / a.IC) << 8) | (uint32_t)(rem % a.IC) : 0xFFFFFFFFu;
    }
    size_t lds = (size_t)WG_T * WG_DY_PLANE + 128 + (size_t)WG_T * a.xplane + 128;
    if (lds > WG_LDS_MAX) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA bwd_weight: tile does not fit in LDS");
    if (lds < (size_t)9 * 32 * WG_T * sizeof(float)) lds = (size_t)9 * 32 * WG_T * sizeof(float);   // the epilogue parks one filter half
    static pc_per_device_once lds_attr;
    if (pc_once_pending(lds_attr, ctx->device)) {
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<12>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        pc_once_done(lds_attr, ctx->device);
    }
    int ft = (a.F + WG_T - 1) / WG_T, ct = (a.C + WG_T - 1) / WG_T;
    if (a.xslots > 32 * WG_XTASKS) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA bwd_weight: x tile too large");
    int ks = ctx->num_cu / (ft * ct);
    if (ks > a.n_ktiles) ks = a.n_ktiles;
    if (ks < 1) ks = 1;
    a.ksplit = ks;
    void *scr = nullptr;
    s = pc_scratch(ctx, sizeof(float) * 4 * (size_t)ks * (size_t)nslots, &scr);
    if (s != PC_OK) return s;
    const dim3 grid((unsigned)ct, (unsigned)ft, (unsigned)ks);
    const uint16_t *xp = (const uint16_t *)x, *dyp = (const uint16_t *)dy;
    if (a.nks <= 4) hipLaunchKernelGGL(pc_mfma_wgrad_kernel<4>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    else if (a.nks <= 8) hipLaunchKernelGGL(pc_mfma_wgrad_kernel<8>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    else if (a.nks <= 12) hipLaunchKernelGGL(pc_mfma_wgrad_kernel<12>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    else hipLaunchKernelGGL(pc_mfma_wgrad_kernel<16>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    pc_note_kernel(ctx, "pc_mfma_wgrad_kernel<%d>", a.nks <= 4 ? 4 : a.nks <= 8 ? 8 : a.nks <= 12 ? 12 : 16);
    s = pc_hip_check(ctx, hipGetLastError(), "MFMA bwd_weight launch");
    if (s != PC_OK) return s;
    return pc_launch_wgrad_reduce(ctx, (const float *)scr, ks, nslots, nslots, pk, dw);
}

// Backward-weight of several layers: the layers the wave-specialised kernel takes run in one launch per
// WS_GROUP_MAX layers, followed by one grouped reduction; each layer has the tiles of its own call and at most
// its splits (fixed order of additions: deterministic, but not the bits of the single call when the split differs).
// The other layers go through pc_mfma_bwd_weight first.
// Every layer has its own region of the context's scratch buffer (partial planes, padded copy of x).
pc_status pc_mfma_bwd_weight_group(pc_ctx *ctx, int n, const pc_conv_desc *d, const pc_packed *const *pk, const void *const *x,
                                   const void *const *dy, float *const *dw)
{
    struct Item { int l; WgradWsArgs a; int ct, ft; size_t lds, part_off, pad_off; bool pad_x; int64_t xb, nslots; };
    std::vector<Item> items;
    std::vector<int> single;
    size_t total = 0;
    for (int l = 0; l < n; ++l) {
        const int64_t nslots = pk[l]->nnzk >= 0 ? pk[l]->nnzk : (int64_t)pk[l]->v.F * pk[l]->v.C;
        if (nslots == 0) continue;
        Item it;
        it.l = l;
        it.nslots = nslots;
        if (ctx->plan_cfg == 10 || !ws_plan(ctx, &d[l], nslots, &it.a, &it.ct, &it.ft, &it.lds, &it.pad_x, &it.xb)) {
            single.push_back(l);
            continue;
        }
        items.push_back(it);
    }
    // A layer's own call splits its pixel tiles until the layer alone fills the chip; here the layers fill it
    // together, so every workgroup gets about the same share of all (tile, pixel tile) units: fewer splits, longer
    // main loops per prologue and epilogue, fewer partial planes.
    int64_t units = 0;
    for (const Item &it : items) units += (int64_t)it.ct * it.ft * it.a.n_ktiles;
    int64_t rounds = units / ((int64_t)PC_GROUP_UNITS * ctx->num_cu);
    if (rounds < 1) rounds = 1;
    if (rounds > 4) rounds = 4;
    int64_t share = units / (rounds * (int64_t)ctx->num_cu);
    if (share < 1) share = 1;
    for (Item &it : items) {
        int64_t ks = (it.a.n_ktiles + share - 1) / share;
        if (ks < 1) ks = 1;
        // split counts the XCD-aware re-reading of the workgroup index can use: a multiple of 8, or a divisor of 8
        // (resnet50_imagenet: 317 us against 339 us with arbitrary counts; within 1 % elsewhere)
        if (ks >= 8) ks = (ks + 7) / 8 * 8;
        else if (ks > 4) ks = 8;
        else if (ks == 3) ks = 4;
        if (ks < it.a.ksplit) it.a.ksplit = (int32_t)ks;
        it.part_off = total;
        if (it.a.ksplit > 1) total += (sizeof(float) * 4 * (size_t)it.a.ksplit * (size_t)it.nslots + 255) / 256 * 256;
        it.pad_off = total;
        if (it.pad_x) total += ((size_t)it.xb + 255) / 256 * 256;
    }
    void *scr = nullptr;
    pc_status s = PC_OK;
    if (total) {
        s = pc_scratch(ctx, total, &scr);      // grows the buffer, if it must, before anything is enqueued
        if (s != PC_OK) return s;
    }
    for (int l : single) {
        s = pc_mfma_bwd_weight(ctx, &d[l], pk[l], x[l], dy[l], dw[l]);
        if (s != PC_OK) return s;
    }
    if (items.empty()) return PC_OK;
    if (total) {
        s = pc_scratch(ctx, total, &scr);      // the base may have moved if one of the calls above needed more
        if (s != PC_OK) return s;
    }
    s = ws_set_lds_attr(ctx);
    if (s != PC_OK) return s;
    unsigned char *base = static_cast<unsigned char *>(scr);
    std::vector<WgradReduceItem> red;
    std::vector<int64_t> red_nslots;
    std::vector<const pc_packed *> red_pk;
    for (size_t i0 = 0; i0 < items.size(); i0 += WS_GROUP_MAX) {
        const int m = (int)(items.size() - i0 < WS_GROUP_MAX ? items.size() - i0 : WS_GROUP_MAX);
        WgradWsGroup g;
        memset(&g, 0, sizeof(g));
        g.n = m;
        size_t lds = 0;
        for (int i = 0; i < m; ++i) {
            const Item &it = items[i0 + i];
            WgradWsLayer &y = g.layer[i];
            y.a = it.a;
            y.x = (const uint16_t *)x[it.l];
            if (it.pad_x) {
                void *xp = base + it.pad_off;
                pc_launch_pad_channels(ctx, (const uint16_t *)x[it.l], xp, (int64_t)it.a.N * it.a.H * it.a.W, it.a.Creal, it.a.C);
                y.x = (const uint16_t *)xp;
            }
            y.dy = (const uint16_t *)dy[it.l];
            y.kinfo = pk[it.l]->v.kinfo;
            y.partial = it.a.ksplit > 1 ? reinterpret_cast<float *>(base + it.part_off) : nullptr;
            y.dw = dw[it.l];
            y.gx = it.ct; y.gy = it.ft;
            const int nwg = it.ct * it.ft * it.a.ksplit;
            g.blk0[i + 1] = g.blk0[i] + (nwg + 7) / 8 * 8;
            if (it.lds > lds) lds = it.lds;
            if (it.a.ksplit > 1) {
                WgradReduceItem r;
                memset(&r, 0, sizeof(r));
                r.partial = y.partial; r.dw = y.dw; r.pstride = it.nslots; r.G = it.a.ksplit;
                red.push_back(r);
                red_nslots.push_back(it.nslots);
                red_pk.push_back(pk[it.l]);
            }
        }
        hipLaunchKernelGGL(pc_mfma_wgrad_ws_group_kernel, dim3((unsigned)g.blk0[m]), dim3(512), lds, ctx->stream, g);
        pc_note_kernel(ctx, "pc_mfma_wgrad_ws_group_kernel");
        s = pc_hip_check(ctx, hipGetLastError(), "MFMA bwd_weight (several layers) launch");
        if (s != PC_OK) return s;
    }
    if (red.empty()) return PC_OK;
    return pc_launch_wgrad_reduce_group(ctx, (int)red.size(), red.data(), red_nslots.data(), red_pk.data());
}

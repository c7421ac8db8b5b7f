// Forward and backward-data of a layer with a handful of channels on one side (the first layer of a network: 3 input
// channels), bf16, stride 1, on the matrix cores. Section 5.2 (forward and backward formulas); the first layer is
// pruned like every other one.
//
// With 3 channels the general kernels pad the reduction (forward) or the output rows (backward-data) to 16 or 32
// channels per tap and still move the wide tensor (64 channels per pixel) at the rate of their tile pipeline. Here the
// arithmetic is shaped to the layer instead, and what remains is one pass over the wide tensor:
//   forward:       one k-step of 16 per tap ROW: 3 neighbouring pixels x 4 channels (+ 4 zeros), read from an LDS copy
//                  of the input rows with 4-channel pixels and a zero border; 3 matrix instructions per 32 pixels and
//                  32 filters. The filters of a row tile are permuted so that a lane's 16 accumulators are 2 x 8
//                  consecutive filters of its pixel: the output goes straight from registers to memory in 16-byte
//                  pieces, lanes l and l + 32 side by side.
//   backward-data: v_mfma_f32_16x16x32_bf16 with the (up to 4) input channels as the 16 rows: 9 taps x F/32
//                  instructions per 16 pixels; the weight operand stays in registers, the error tile (8 x 32 pixels
//                  and its border) is staged in LDS once and read by every tap; persistent workgroups keep the loads
//                  of their next tile in flight while they multiply.
#include "pc_mfma.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct ThinArgs {
    int32_t N, H, W, C, F;       // C: the thin side (<= 4 channels), F: the wide side (a multiple of 32)
    int32_t TH, TW, LW;          // output tile, and pixels per staged row (TW + 2)
    int32_t tiles_y, tiles_x;
    int32_t KS;                  // k-steps of 16 per tap in the operand tiles
    uint32_t thin_bytes, wide_bytes;
    uint32_t mg_LW, mg_tx, mg_ty;
};

constexpr uint32_t THIN_OOB = 0x80000000u;   // past any tensor these kernels accept: loads return zero, stores are dropped

// ------------------------------------------------------------------ forward
// NFT: row tiles of 32 filters. Workgroup: TH output rows x TW (a multiple of 32) columns of one image.
// wz: the forward operand tiles [F/32][9][KS][64 lanes][8] (lane = (filter % 32, half), 8 channels each).
template <int NFT, int ACT>
__global__ void __launch_bounds__(256) pc_thin_fwd_kernel(const uint16_t *__restrict__ x, uint16_t *__restrict__ y,
                                                          const uint16_t *__restrict__ wz, ThinArgs a)
{
    extern __shared__ __align__(16) unsigned char lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int g = lane >> 5, px = lane & 31;
    const uint32_t u = pc_udiv(blockIdx.x, a.mg_tx);
    const int tx = (int)(blockIdx.x - u * a.tiles_x);
    const uint32_t n = pc_udiv(u, a.mg_ty);
    const int ty = (int)(u - n * a.tiles_y);
    const int y0 = ty * a.TH, x0 = tx * a.TW;

    // ---- the weight operand. Row rho of a row tile holds filter fr(rho): a lane's accumulators (rows 8j + 4g + i,
    // j = 0..3, i = 0..3) are then filters 16 (j / 2) + 8 g + 4 (j % 2) + i: accumulators 0..7 and 8..15 are 8
    // consecutive filters each. k-step r (tap row r): k = 4 s + c for tap column s = 0..2, 4 zeros after them.
    const int rho = lane & 31;
    const int jr = rho >> 3, gr = (rho >> 2) & 1, ir = rho & 3;
    const int fr = 16 * (jr >> 1) + 8 * gr + 4 * (jr & 1) + ir;
    bf16x8 A[NFT][3];
#pragma unroll
    for (int t = 0; t < NFT; ++t)
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            // lane half 0: taps (r, 0) and (r, 1); half 1: tap (r, 2) and zeros. Channels 0..3 of a tap are the first
            // 8 bytes of lane (filter, half 0) of the tap's first k-step.
            const uint16_t *b0 = wz + ((size_t)((t * 9 + r * 3 + (g ? 2 : 0)) * a.KS) * 512 + fr * 8);
            const uint16_t *b1 = wz + ((size_t)((t * 9 + r * 3 + 1) * a.KS) * 512 + fr * 8);
            const uint2 p0 = *reinterpret_cast<const uint2 *>(b0);
            uint2 p1 = *reinterpret_cast<const uint2 *>(b1);
            if (g) p1 = make_uint2(0u, 0u);
            const v4u32 w4 = {p0.x, p0.y, p1.x, p1.y};
            __builtin_memcpy(&A[t][r], &w4, 16);
        }

    // ---- stage the input rows: pixel (sy, sx) of the staged tile is input pixel (y0 - 1 + sy, x0 - 1 + sx), 4 channels
    // (8 bytes) each, zeros outside the image and past the last channel
    const __amdgpu_buffer_rsrc_t xsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(x), 0, a.thin_bytes, 0x00020000);
    const int HP = (a.TH + 2) * a.LW;
    for (int hp = threadIdx.x; hp < HP; hp += 256) {
        const int sy = (int)pc_udiv((uint32_t)hp, a.mg_LW), sx = hp - sy * a.LW;
        const int iy = y0 - 1 + sy, ix = x0 - 1 + sx;
        const bool ok = (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
        const uint32_t off = ok ? (uint32_t)((((int)n * a.H + iy) * a.W + ix) * a.C * 2) : THIN_OOB;
        uint32_t v[4];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            v[c] = (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(xsrc, (int)(c < a.C ? off : THIN_OOB), c * 2, 0);
        *reinterpret_cast<uint2 *>(lds + (size_t)hp * 8) = make_uint2(v[0] | (v[1] << 16), v[2] | (v[3] << 16));
    }
    __syncthreads();

    // ---- 32 pixels of a row at a time
    const __amdgpu_buffer_rsrc_t ysrc = __builtin_amdgcn_make_buffer_rsrc(y, 0, a.wide_bytes, 0x00020000);
    const int npx = a.TW >> 5, npt = a.TH * npx;
    for (int pt = wave; pt < npt; pt += 4) {
        const int ry = pt / npx, cx = (pt - ry * npx) * 32;
        bf16x8 B[3];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            // lane half 0: pixels x - 1 and x; half 1: pixel x + 1 and zeros
            const unsigned char *p = lds + (size_t)((ry + r) * a.LW + cx + px + 2 * g) * 8;
            const uint2 q0 = *reinterpret_cast<const uint2 *>(p);
            uint2 q1 = *reinterpret_cast<const uint2 *>(p + 8);
            if (g) q1 = make_uint2(0u, 0u);
            const v4u32 b4 = {q0.x, q0.y, q1.x, q1.y};
            __builtin_memcpy(&B[r], &b4, 16);
        }
        const int oy = y0 + ry, ox = x0 + cx + px;
        const bool ok = oy < a.H && ox < a.W;
        const uint32_t obase = ok ? (uint32_t)((((int)n * a.H + oy) * a.W + ox) * a.F * 2) : THIN_OOB;
#pragma unroll
        for (int t = 0; t < NFT; ++t) {
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.0f;
#pragma unroll
            for (int r = 0; r < 3; ++r) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[t][r], B[r], acc, 0, 0, 0);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                v4u32 pv;
#pragma unroll
                for (int e = 0; e < 4; ++e) pv[e] = pc_pack_bf16x2(acc[8 * h + 2 * e], acc[8 * h + 2 * e + 1]);
                if (ACT == PC_ACT_RELU) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) pv[e] &= ~(((pv[e] & 0x80008000u) >> 15) * 0xFFFFu);   // negative (or -0) -> +0
                }
                // filters 32 t + 16 h + 8 g + (0..7)
                __builtin_amdgcn_raw_buffer_store_b128(pv, ysrc, (int)(ok ? obase + (uint32_t)((32 * t + 16 * h + 8 * g) * 2) : THIN_OOB), 0, 0);
            }
        }
    }
}

// ------------------------------------------------------------------ backward-data
// NFK: blocks of 32 filters (the reduction per tap). Persistent workgroups walk tiles of 8 x 32 input pixels of one
// image: the error tile and its border (10 x 34 pixels) are staged in LDS while the loads of the workgroup's next tile
// are already in flight in registers.
// wz: the backward operand tiles [C/32][9][KS][64 lanes][8] (lane = (channel % 32, half), 8 filters each).
// dx[y][x][c] = sum over taps (r, s) and filters f of W[f][c][r][s] * dy[y + 1 - r][x + 1 - s][f].
template <int NFK>
__global__ void __launch_bounds__(256) pc_thin_bwd_data_kernel(const uint16_t *__restrict__ dy, uint16_t *__restrict__ dx,
                                                               const uint16_t *__restrict__ wz, ThinArgs a, int total)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int TH = 8, TW = 32, LW = TW + 2, HP = (TH + 2) * LW;
    constexpr int PITCH = NFK * 64 + 16;      // bytes per staged pixel
    constexpr int PARTS = NFK * 4;            // 16-byte pieces per pixel
    constexpr int NE = HP * PARTS, NB = (NE + 255) / 256;   // pieces per tile, and per thread
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, p16 = lane & 15;

    // ---- the weight operand: rows = channels (lane % 16; rows past the last channel are zero in the tiles), lane
    // quarter q holds filters 32 h + 8 q + (0..7) of tap t: lane (channel, half q % 2) of k-step 2 h + q / 2
    bf16x8 A[9][NFK];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int h = 0; h < NFK; ++h) {
            const uint16_t *b = wz + ((size_t)(t * a.KS + 2 * h + (q >> 1)) * 512 + (p16 + 32 * (q & 1)) * 8);
            const v4u32 w4 = *reinterpret_cast<const v4u32 *>(b);
            __builtin_memcpy(&A[t][h], &w4, 16);
        }

    // ---- staging: piece i of a thread is 16-byte part (tid % PARTS) of staged pixel tid / PARTS + (256 / PARTS) i;
    // staged pixel (sy, sx) is dy pixel (y0 - 1 + sy, x0 - 1 + sx), zeros outside the image
    const __amdgpu_buffer_rsrc_t dsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(dy), 0, a.wide_bytes, 0x00020000);
    const int part = threadIdx.x % PARTS, hp0 = threadIdx.x / PARTS;
    int sysx[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int hp = hp0 + (256 / PARTS) * i;
        const int sy = hp / LW, sx = hp - sy * LW;
        sysx[i] = hp < HP ? (sy << 8) | sx : -1;
    }
    auto issue = [&](int b, v4u32 (&R)[NB]) {
        const bool live = b < total;
        const uint32_t u = pc_udiv((uint32_t)b, a.mg_tx);
        const int tx = b - (int)u * a.tiles_x;
        const uint32_t n = pc_udiv(u, a.mg_ty);
        const int ty = (int)u - (int)n * a.tiles_y;
        const int y0 = ty * TH - 1, x0 = tx * TW - 1;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int iy = y0 + (sysx[i] >> 8), ix = x0 + (sysx[i] & 255);
            const bool ok = live && sysx[i] >= 0 && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
            const uint32_t off = ok ? (uint32_t)((((int)n * a.H + iy) * a.W + ix) * a.F * 2 + part * 16) : THIN_OOB;
            R[i] = __builtin_amdgcn_raw_buffer_load_b128(dsrc, (int)off, 0, 0);
        }
    };
    auto put = [&](const v4u32 (&R)[NB]) {
#pragma unroll
        for (int i = 0; i < NB; ++i)
            if (hp0 + (256 / PARTS) * i < HP)
                *reinterpret_cast<v4u32 *>(lds + (size_t)(hp0 + (256 / PARTS) * i) * PITCH + part * 16) = R[i];
    };

    const __amdgpu_buffer_rsrc_t xsrc = __builtin_amdgcn_make_buffer_rsrc(dx, 0, a.thin_bytes, 0x00020000);
    const int G = gridDim.x;
    v4u32 R[NB];
    issue(blockIdx.x, R);
    for (int b = blockIdx.x; b < total; b += G) {
        put(R);
        __syncthreads();
        issue(b + G, R);
        const uint32_t u = pc_udiv((uint32_t)b, a.mg_tx);
        const int tx = b - (int)u * a.tiles_x;
        const uint32_t n = pc_udiv(u, a.mg_ty);
        const int ty = (int)u - (int)n * a.tiles_y;
        const int y0 = ty * TH, x0 = tx * TW;
        // ---- four groups of 16 pixels per wavefront: rows 2 wave, 2 wave + 1, both halves of the 32 columns
        f32x4 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
        // staged pixel of output pixel (ry, cx) for tap (r, s): (ry + 2 - r, cx + 2 - s)
        const unsigned char *pb = lds + (size_t)((2 * wave + 2) * LW + p16 + 2) * PITCH + q * 16;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int h = 0; h < NFK; ++h)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bf16x8 bq = *reinterpret_cast<const bf16x8 *>(pb + (((j >> 1) - t / 3) * LW + 16 * (j & 1) - t % 3) * PITCH + h * 64);
                    acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[t][h], bq, acc[j], 0, 0, 0);
                }
        // lane quarter 0 holds channels 0..3 of pixel p16 of every group
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int oy = y0 + 2 * wave + (j >> 1), ox = x0 + 16 * (j & 1) + p16;
            const bool ok = q == 0 && oy < a.H && ox < a.W;
            const uint32_t obase = (uint32_t)((((int)n * a.H + oy) * a.W + ox) * a.C * 2);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint32_t w = pc_pack_bf16x2(acc[j][c], 0.0f) & 0xFFFFu;
                __builtin_amdgcn_raw_buffer_store_b16((unsigned short)w, xsrc, (int)((ok && c < a.C) ? obase + c * 2 : THIN_OOB), 0, 0);
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------ host
static bool thin_plan(const pc_conv_desc *d, int TH, int TW, int pitch, ThinArgs *out, size_t *lds)
{
    ThinArgs a;
    memset(&a, 0, sizeof(a));
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = d->C; a.F = d->F;
    a.TH = TH; a.TW = TW; a.LW = TW + 2;
    a.tiles_y = (d->H + TH - 1) / TH;
    a.tiles_x = (d->W + TW - 1) / TW;
    const int64_t thin = (int64_t)d->N * d->H * d->W * d->C * 2, wide = (int64_t)d->N * d->H * d->W * d->F * 2;
    if (thin >= ((int64_t)1 << 31) || wide >= ((int64_t)1 << 31)) return false;   // 32-bit buffer offsets, 2^31 = out of range
    if ((int64_t)d->N * a.tiles_y * a.tiles_x >= ((int64_t)1 << 31)) return false;
    a.thin_bytes = (uint32_t)thin; a.wide_bytes = (uint32_t)wide;
    a.mg_LW = pc_udiv_magic(a.LW); a.mg_tx = pc_udiv_magic(a.tiles_x); a.mg_ty = pc_udiv_magic(a.tiles_y);
    // the multiply-high divisions are exact while dividend * divisor < 2^32
    const int64_t blocks = (int64_t)d->N * a.tiles_y * a.tiles_x;
    if (blocks * a.tiles_x >= ((int64_t)1 << 32) || (blocks / a.tiles_x + 1) * a.tiles_y >= ((int64_t)1 << 32)) return false;
    *lds = (size_t)(TH + 2) * a.LW * pitch + 16;
    *out = a;
    return true;
}

template <int NFT>
static void thin_fwd_launch(hipStream_t st, unsigned grid, size_t lds, const uint16_t *x, uint16_t *y, const uint16_t *wz,
                            const ThinArgs &a, int act)
{
    if (act == PC_ACT_RELU) hipLaunchKernelGGL((pc_thin_fwd_kernel<NFT, PC_ACT_RELU>), dim3(grid), dim3(256), lds, st, x, y, wz, a);
    else hipLaunchKernelGGL((pc_thin_fwd_kernel<NFT, PC_ACT_NONE>), dim3(grid), dim3(256), lds, st, x, y, wz, a);
}

// Forward pass of a layer with at most 4 input channels. *launched stays false when the layer is outside what the
// kernel takes (the caller then uses the general kernels). act: PC_ACT_NONE or PC_ACT_RELU.
pc_status pc_thin_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y, int act, bool *launched)
{
    *launched = false;
    if (d->stride != 1 || d->C > 4 || (d->F & 31) || d->F > 128 || (act != PC_ACT_NONE && act != PC_ACT_RELU)) return PC_OK;
    int TW = (d->W + 31) / 32 * 32;
    if (TW > 256) TW = 256;
    ThinArgs a;
    size_t lds;
    if (!thin_plan(d, 8, TW, 8, &a, &lds)) return PC_OK;
    a.KS = pk->v.Ck / 16;
    const unsigned grid = (unsigned)((int64_t)d->N * a.tiles_y * a.tiles_x);
    const uint16_t *xs = static_cast<const uint16_t *>(x);
    uint16_t *ys = static_cast<uint16_t *>(y);
    switch (d->F / 32) {
    case 1: thin_fwd_launch<1>(ctx->stream, grid, lds, xs, ys, pk->v.wz_fwd, a, act); break;
    case 2: thin_fwd_launch<2>(ctx->stream, grid, lds, xs, ys, pk->v.wz_fwd, a, act); break;
    case 3: thin_fwd_launch<3>(ctx->stream, grid, lds, xs, ys, pk->v.wz_fwd, a, act); break;
    default: thin_fwd_launch<4>(ctx->stream, grid, lds, xs, ys, pk->v.wz_fwd, a, act); break;
    }
    *launched = true;
    pc_note_kernel(ctx, "pc_thin_fwd_kernel<%d, %d>", d->F / 32, act);
    return pc_hip_check(ctx, hipGetLastError(), "first-layer forward launch");
}

// Backward-data pass of a layer with at most 4 input channels and 32 or 64 filters.
pc_status pc_thin_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx, bool *launched)
{
    *launched = false;
    if (d->stride != 1 || d->C > 4 || (d->F != 32 && d->F != 64)) return PC_OK;
    ThinArgs a;
    size_t lds;
    if (!thin_plan(d, 8, 32, d->F * 2 + 16, &a, &lds)) return PC_OK;
    a.KS = pk->v.Fk / 16;
    const int64_t total = (int64_t)d->N * a.tiles_y * a.tiles_x;
    const unsigned grid = (unsigned)(total < 2 * (int64_t)ctx->num_cu ? total : 2 * (int64_t)ctx->num_cu);
    const uint16_t *ds = static_cast<const uint16_t *>(dy);
    uint16_t *xs = static_cast<uint16_t *>(dx);
    if (d->F == 32) hipLaunchKernelGGL((pc_thin_bwd_data_kernel<1>), dim3(grid), dim3(256), lds, ctx->stream, ds, xs, pk->v.wz_bwd, a, (int)total);
    else hipLaunchKernelGGL((pc_thin_bwd_data_kernel<2>), dim3(grid), dim3(256), lds, ctx->stream, ds, xs, pk->v.wz_bwd, a, (int)total);
    *launched = true;
    pc_note_kernel(ctx, "pc_thin_bwd_data_kernel<%d>", d->F / 32);
    return pc_hip_check(ctx, hipGetLastError(), "first-layer backward-data launch");
}

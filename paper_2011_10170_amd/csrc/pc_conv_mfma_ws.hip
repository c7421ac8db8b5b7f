// Forward / backward-data on the matrix cores, persistent wave-specialised kernel (see pc_conv_mfma.hip for the
// implicit-GEMM formulation, the operand tiles and the MFMA register layout).
#include "pc_mfma.h"

// ------------------------------------------------------------------ wave-specialised kernel
// Eight wavefronts per workgroup, one workgroup per CU, walking tiles of 32*A_T output channels x
// 32*B_T pixels (row tile fastest, so workgroups running side by side share the input tile in L2).
//   wavefronts 4..7 (loaders) stage the input halo tile of the NEXT item (tile, 64-channel chunk) into
//     one of two LDS buffers; their global loads are issued KS_DEPTH items ahead into registers, so an
//     HBM round trip is hidden behind several items of MFMA work and never stalls an MFMA wavefront
//     (a wavefront's outstanding loads retire in order: mixing long bulk loads with the short
//     operand loads in one wavefront makes every operand wait for the bulk);
//   wavefronts 0..3 (MFMA) all own the WHOLE tile and split the reduction: wavefront w takes the k-step
//     of channels 16w..16w+15 of every tap of every chunk. A wavefront tile of 64x128 needs half the
//     operand bytes per MFMA of the 32x64 tile an output split would leave at this workgroup size,
//     which keeps both operand paths (A fragments from L2 through the 64 B/clk vector cache, B
//     fragments from LDS) well under their limits. At the end of a tile the four partial sums are
//     added in a fixed order (wavefront 0..3) through LDS, every wavefront finishing and storing a
//     quarter of the tile.
// Both roles execute the same sequence of workgroup barriers: one after the first staged item and one
// per item.
#define KS_NV 8          // 16-byte elements staged per loader thread and item (256 loader threads), reduction split
#define KS_NV1 12        // the same without the reduction split (512-pixel tiles of 32 channels)
#define KS_DEPTH 3       // items in flight in the loader's registers

// Depth of the A-fragment ring: the largest divisor of the fragments per item that does not exceed cap
constexpr int pc_ring_depth(int nf, int cap)
{
    int best = 1;
    for (int d = 1; d <= cap; ++d)
        if (nf % d == 0) best = d;
    return best;
}

// Two bf16 values in a word: each one that is negative (or -0) becomes +0.
__device__ __forceinline__ uint32_t pc_relu_bf16x2(uint32_t u)
{
    return u & ~(((u & 0x80008000u) >> 15) * 0xFFFFu);
}

// Two bf16 values in a word: each one is kept where the matching value of a is positive, else +0.
__device__ __forceinline__ uint32_t pc_mask_bf16x2(uint32_t u, uint32_t a)
{
    const uint32_t lo = ((a & 0xFFFFu) - 1u) < 0x7FFFu ? 0x0000FFFFu : 0u;   // sign clear and not zero
    const uint32_t hi = ((a >> 16) - 1u) < 0x7FFFu ? 0xFFFF0000u : 0u;
    return u & (lo | hi);
}

// The loader wavefronts of the wave-specialised kernels (wavefronts 4..7 of a workgroup of 8): they stage the input
// halo tile of the NEXT item (tile, chunk of KC channels) into one of two LDS buffers, their global loads KS_DEPTH
// items ahead in registers, and execute one workgroup barrier after the first staged item and one per item.
//   vb, G: index of this workgroup in the tile order and the number of workgroups; ntile_blk tiles of nch chunks each
template <int KC, int NV>
__device__ __forceinline__ void pc_ks_loader_role(const uint16_t *__restrict__ in, const MfmaArgs &g, unsigned char *lds, int vb, int G,
                                                  int ntile_blk, int nch)
{
    constexpr int PITCH = 2 * KC + 16;
    constexpr int PARTS = KC / 8;
    const int I = ntile_blk * nch;
    // ------------------------------------------------------------ loaders
    const int tl = threadIdx.x - 256;
    const int part = tl % PARTS;
    // The input is read with buffer loads: an offset past the end of the tensor returns zeros, which
    // serves every element that is not a real input value (zero padding around the image, images
    // past the batch, channels past the last one, unused loader slots) without a branch. Loads and
    // LDS writes stay unconditional, so the compiler can count the loads in flight and wait for
    // exactly the oldest register set.
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(in), 0, g.in_bytes, 0x00020000);
    constexpr uint32_t OOB = 0x80000000u;   // past any tensor this kernel accepts, and no wrap-around with the chunk offset
    const bool part_in_last = (nch - 1) * KC + part * 8 < g.in_CH;   // this thread's channels exist in the last chunk
    int pk[NV], loff[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int e = tl + 256 * v;
        const uint32_t q = (uint32_t)e / PARTS;
        const uint32_t t2 = pc_udiv(q, g.mg_IW);
        const int ix = (int)(q - t2 * g.IW);
        const uint32_t ti = pc_udiv(t2, g.mg_IH);
        const int iy = (int)(t2 - ti * g.IH);
        pk[v] = e < g.nelem ? (int)((ti << 20) | (iy << 10) | ix) : -1;
        loff[v] = e < g.nelem ? (int)q * PITCH + part * 16 : g.xbuf - 16;
    }
    int lk = 0, lch = 0;              // cursor of the next item to load
    uint32_t voff[NV];             // byte offset of every element's pixel (+ its 16-byte part) in the tensor
    auto tile_offsets = [&](int k) {
        const uint32_t tq = pc_udiv((uint32_t)(vb + k * G), g.mg_fd);
        const uint32_t pt = g.m_fast ? tq : (uint32_t)(vb + k * G) - tq * g.fdiv;
        const uint32_t u = pc_udiv(pt, g.mg_tx);
        const int tx = (int)(pt - u * g.tiles_x);
        const uint32_t tnn = pc_udiv(u, g.mg_ty);
        const int ty = (int)(u - tnn * g.tiles_y);
        const int ltn = (int)tnn * g.TI;
        const int ly0 = ty * g.TH * g.iscale + g.ioff_y;
        const int lx0 = tx * g.TW * g.iscale + g.ioff_x;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int n = ltn + (pk[v] >> 20), y = ly0 + ((pk[v] >> 10) & 1023), x = lx0 + (pk[v] & 1023);
            const bool ok = pk[v] >= 0 && n < g.N && (unsigned)y < (unsigned)g.in_H && (unsigned)x < (unsigned)g.in_W;
            voff[v] = ok ? (uint32_t)((n * g.in_H + y) * g.in_W + x) * (uint32_t)(g.in_CH * 2) + part * 16 : OOB;
        }
    };
    tile_offsets(0);
    auto issue = [&](uint4 (&R)[NV]) {
        const int so = lch * (KC * 2);
        const bool cut = (lch == nch - 1 && !part_in_last) || lk >= ntile_blk;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const v4u32 val = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)(cut ? OOB : voff[v]), so, 0);
            R[v] = make_uint4(val.x, val.y, val.z, val.w);
        }
        if (lk < ntile_blk && ++lch == nch) {
            lch = 0;
            if (++lk < ntile_blk) tile_offsets(lk);
        }
    };
    auto put = [&](const uint4 (&R)[NV], int bufoff) {
#pragma unroll
        for (int v = 0; v < NV; ++v) *reinterpret_cast<uint4 *>(lds + bufoff + loff[v]) = R[v];
    };
    uint4 R0[NV], R1[NV], R2[NV];
    issue(R0); issue(R1);
    put(R0, 0);
    __syncthreads();
    issue(R2); issue(R0);
    // item i: while the MFMA wavefronts work on buffer i&1, write item i+1 (register set (i+1)%3) to the
    // other buffer (past the last item: zeros, never read) and refill that set with item i+4
    auto lstep = [&](int i, uint4 (&R)[NV]) {
        put(R, ((i + 1) & 1) * g.xbuf);
        issue(R);
        __syncthreads();
    };
    int i = 0;
    for (; i + 3 <= I; i += 3) {
        lstep(i, R1);
        lstep(i + 1, R2);
        lstep(i + 2, R0);
    }
    if (i < I) {
        lstep(i, R1);
        if (i + 1 < I) lstep(i + 1, R2);
    }
}

// End of a tile when the MFMA wavefronts split the pixels: every wavefront stores its own 32*B_T pixels, 64 at a time
// through a private LDS area (pixel-major bf16 rows): read back, 8 consecutive lanes hold the 128 contiguous bytes of
// one pixel's 64 channels and the stores are whole 16-byte pieces of full lines instead of scattered 8-byte ones.
template <int A_T, int B_T, int ACT>
__device__ __forceinline__ void pc_ks_store_pixels(const f32x16 (&acc)[A_T][B_T], unsigned char *lds, const MfmaArgs &g, int w, int lane,
                                                   int mt, int tn, int gy0, int gx0, int npix, __amdgpu_buffer_rsrc_t osrc,
                                                   __amdgpu_buffer_rsrc_t msrc)
{
    constexpr uint32_t OOB_OUT = 0x80000000u;
    // Every wavefront stores its own 32*B_T pixels, 64 at a time through a private LDS area (pixel-major
    // bf16 rows): read back, 8 consecutive lanes hold the 128 contiguous bytes of one pixel's 64 channels
    // and the stores are whole 16-byte pieces of full lines instead of scattered 8-byte ones.
    unsigned char *stg = lds + g.red_off + w * (64 * 144);
#pragma unroll
    for (int half = 0; half < B_T / 2; ++half) {
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int j = half * 2 + jj;
                    uint2 pkd;
                    pkd.x = pc_pack_bf16x2(acc[ii][j][q4 * 4 + 0], acc[ii][j][q4 * 4 + 1]);
                    pkd.y = pc_pack_bf16x2(acc[ii][j][q4 * 4 + 2], acc[ii][j][q4 * 4 + 3]);
                    *reinterpret_cast<uint2 *>(stg + (jj * 32 + (lane & 31)) * 144 + (ii * 32 + q4 * 8 + (lane >> 5) * 4) * 2) = pkd;
                }
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int px = it * 8 + (lane >> 3), c16 = lane & 7;
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + px * 144 + c16 * 16);
            const int q = (w * B_T + half * 2) * 32 + px;
            const int ti = (int)pc_udiv((uint32_t)q, g.mg_THTW);
            const int rem = q - ti * g.TH * g.TW;
            const int y = (int)pc_udiv((uint32_t)rem, g.mg_TW), x = rem - y * g.TW;
            const int n = tn + ti, gy = gy0 + y, gx = gx0 + x;
            const int m = mt * (32 * A_T) + c16 * 8;
            const bool ok = q < npix && n < g.N && gy < g.GH && gx < g.GW && m < g.out_CH && c16 < 4 * A_T;
            const int oy = gy * g.oscale + g.ooff_y, ox = gx * g.oscale + g.ooff_x;
            const uint32_t off = ok ? (uint32_t)((n * g.out_H + oy) * g.out_W + ox) * (uint32_t)(g.out_CH * 2) + (uint32_t)(m * 2) : OOB_OUT;
            v4u32 pv = {v.x, v.y, v.z, v.w};
            if (ACT == PC_ACT_RELU) {
#pragma unroll
                for (int e = 0; e < 4; ++e) pv[e] = pc_relu_bf16x2(pv[e]);
            } else if (ACT == PC_ACT_RELU_MASK) {
                const v4u32 mk = __builtin_amdgcn_raw_buffer_load_b128(msrc, (int)off, 0, 0);
#pragma unroll
                for (int e = 0; e < 4; ++e) pv[e] = pc_mask_bf16x2(pv[e], mk[e]);
            }
            __builtin_amdgcn_raw_buffer_store_b128(pv, osrc, (int)off, 0, 0);
        }
    }
}

// ACT: PC_ACT_NONE, or a fused step on the stored values: PC_ACT_RELU (negative outputs become +0) or
// PC_ACT_RELU_MASK (outputs are kept where g.act_mask, a tensor of the output's shape, is positive).
template <int A_T, int B_T, int NTAPS, int KC, int KSP, int ACT = PC_ACT_NONE>
__global__ void __launch_bounds__(512, 1)
pc_mfma_conv_ks_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out, const uint16_t *__restrict__ wz, MfmaArgs g)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int KSC = KC / 16;          // k-steps per chunk
    static_assert(KSP == 4 || KSP == 1, "the MFMA wavefronts split the reduction four ways or not at all");
    constexpr int KSW = KC / (16 * KSP);  // k-steps per chunk, tap and MFMA wavefront
    constexpr int NV = KSP == 4 ? KS_NV : KS_NV1;   // 16-byte elements staged per loader thread and item
    constexpr int S = NTAPS * KSW;        // steps per item and wavefront
    constexpr int NF = S * A_T;           // A fragments per item and wavefront
    // the ring has to cover an L2 round trip in MFMA time: narrow pixel tiles issue fewer MFMAs per fragment
    // and have the registers for a whole item of fragments
    constexpr int PFD = pc_ring_depth(NF, B_T >= 4 ? 10 : 18);
    constexpr int PITCH = 2 * KC + 16;
    constexpr int PARTS = KC / 8;
    constexpr int NT = A_T * B_T;
    constexpr int ROUNDS = NT >= 4 ? NT / 4 : 1;
    constexpr int NOWN = NT >= 4 ? 4 : NT;
    constexpr int DB = B_T >= 4 ? 1 : (B_T == 2 ? 2 : 4);   // B fragments are read this many steps ahead
    constexpr int DBS = DB < S ? DB : S;
    constexpr int RB = DBS + 1;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = wave & 3;
    const int G = gridDim.x;
    int vb = blockIdx.x;
    if ((G & 7) == 0) vb = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);   // neighbours in the tile order share an XCD
    const int ntile_blk = (g.total_tiles - vb + G - 1) / G;
    const int nch = g.nchunks;
    const int I = ntile_blk * nch;

    if (wave >= 4) {
        pc_ks_loader_role<KC, NV>(in, g, lds, vb, G, ntile_blk, nch);
        return;
    }

    // ---------------------------------------------------------------- MFMA wavefronts
    const int npix = g.TI * g.TH * g.TW;
    int base[B_T];
#pragma unroll
    for (int j = 0; j < B_T; ++j) {
        // reduction split: every wavefront covers all pixels and its own k-steps; otherwise its own pixels
        int q = ((KSP == 1 ? w * B_T : 0) + j) * 32 + (lane & 31);
        if (q >= npix) q = npix - 1;
        const int ti = (int)pc_udiv((uint32_t)q, g.mg_THTW);
        const int rem = q - ti * g.TH * g.TW;
        const int y = (int)pc_udiv((uint32_t)rem, g.mg_TW), x = rem - y * g.TW;
        base[j] = ((ti * g.IH + y * g.lstep) * g.IW + x * g.lstep) * PITCH + (lane >> 5) * 16 +
                  (KSP == 4 ? w * (KSW * 32) : 0);
    }
    // the pixel sub-tile this wavefront finishes and stores
    const int jo = w % B_T;
    const int qo = jo * 32 + (lane & 31);
    const int o_ti = (int)pc_udiv((uint32_t)qo, g.mg_THTW);
    const int o_y = (int)pc_udiv((uint32_t)(qo - o_ti * g.TH * g.TW), g.mg_TW);
    const int o_x = qo - o_ti * g.TH * g.TW - o_y * g.TW;

    const __amdgpu_buffer_rsrc_t osrc = __builtin_amdgcn_make_buffer_rsrc(out, 0, g.out_bytes, 0x00020000);
    // the mask tensor has the output's shape: it is read at the offsets the output is stored at (past the end: zeros)
    const __amdgpu_buffer_rsrc_t msrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(ACT == PC_ACT_RELU_MASK ? g.act_mask : out), 0, g.out_bytes, 0x00020000);
    constexpr uint32_t OOB_OUT = 0x80000000u;
    // A fragments: buffer loads with the lane's 16 bytes as the vector offset and everything else in the scalar
    // offset. This kernel only runs the full 3x3 tap list in tap order (weight tap t at list position t), so
    // fragment (row tile ii, tap t, k-step kk) of an item lies at (ii*9 + t) * KS + kk fragments of 1 KiB past
    // the item's first one, and the LDS offset of tap t = 3r + s is tap_o0 + r*tap_dr + s*tap_ds: a handful of
    // scalars instead of per-fragment tables that would not fit the scalar registers.
    const __amdgpu_buffer_rsrc_t wsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(wz), 0, g.wz_bytes, 0x00020000);
    const int a_voff = lane * 16;
    const int ksb = g.KS * 1024;          // bytes between the fragments of two taps
    auto a_frag = [&](int item_base, int ph) -> bf16x8 {   // ph: compile-time fragment index inside the item
        const int st = ph / A_T, ii = ph % A_T;
        const v4u32 r = __builtin_amdgcn_raw_buffer_load_b128(wsrc, a_voff, item_base + (ii * 9 + st / KSW) * ksb + (st % KSW) * 1024, 0);
        bf16x8 o;
        __builtin_memcpy(&o, &r, 16);
        return o;
    };
    auto tap_off = [&](int t) -> int { return g.tap_o0 + (t / 3) * g.tap_dr + (t % 3) * g.tap_ds; };
    int mt = 0, tn = 0, gy0 = 0, gx0 = 0;
    auto tile_of = [&](int k, int &mt_, int &tn_, int &gy0_, int &gx0_) {
        const uint32_t t = (uint32_t)(vb + k * G);
        const uint32_t tq = pc_udiv(t, g.mg_fd), trm = t - tq * g.fdiv;
        const uint32_t pt = g.m_fast ? tq : trm;
        mt_ = (int)(g.m_fast ? trm : tq);
        const uint32_t u = pc_udiv(pt, g.mg_tx);
        const int tx = (int)(pt - u * g.tiles_x);
        const uint32_t tnn = pc_udiv(u, g.mg_ty);
        const int ty = (int)(u - tnn * g.tiles_y);
        tn_ = (int)tnn * g.TI;
        gy0_ = ty * g.TH;
        gx0_ = tx * g.TW;
    };
    auto a_base = [&](int mt_, int ch_) -> int {   // byte offset of the item's first fragment for this wavefront
        return ((mt_ * A_T * 9) * g.KS + ch_ * KSC + (KSP == 4 ? w * KSW : 0)) * 1024;
    };
    tile_of(0, mt, tn, gy0, gx0);
    int k = 0, ch = 0;
    int ab = a_base(mt, 0);

    f32x16 acc[A_T][B_T];
#pragma unroll
    for (int i = 0; i < A_T; ++i)
#pragma unroll
        for (int j = 0; j < B_T; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 aring[PFD];
#pragma unroll
    for (int ph = 0; ph < PFD; ++ph) aring[ph] = a_frag(ab, ph);

    __syncthreads();
    for (int i = 0; i < I; ++i) {
        // the item after this one (for the A prefetch); past the end: this one again, unused
        int nk = k, nchk = ch + 1, nmt = mt, ntn = tn, ngy0 = gy0, ngx0 = gx0;
        if (nchk == nch) {
            nchk = 0;
            nk = k + 1;
            if (nk < ntile_blk) tile_of(nk, nmt, ntn, ngy0, ngx0);
            else nchk = ch;
        }
        const int abn = a_base(nmt, nchk);
        const unsigned char *xb = lds + (i & 1) * g.xbuf;

        bf16x8 bring[RB][B_T];
#pragma unroll
        for (int d = 0; d < DBS; ++d)
#pragma unroll
            for (int j = 0; j < B_T; ++j)
                bring[d % RB][j] = *reinterpret_cast<const bf16x8 *>(xb + base[j] + tap_off(d / KSW) + (d % KSW) * 32);
#pragma unroll
        for (int st = 0; st < S; ++st) {
            if (st + DBS < S) {
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    bring[(st + DBS) % RB][j] =
                        *reinterpret_cast<const bf16x8 *>(xb + base[j] + tap_off((st + DBS) / KSW) + ((st + DBS) % KSW) * 32);
            }
            bf16x8 anow[A_T];
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii) {
                const int ph = st * A_T + ii;
                anow[ii] = aring[ph % PFD];
                const int nph = ph + PFD;
                aring[ph % PFD] = nph < NF ? a_frag(ab, nph < NF ? nph : 0) : a_frag(abn, nph < NF ? 0 : nph - NF);
            }
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    acc[ii][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(anow[ii], bring[st % RB][j], acc[ii][j], 0, 0, 0);
            // One wavefront per SIMD issues everything in program order: the loads of the later steps and their
            // address arithmetic go one or two at a time into the shadow of each MFMA instead of in a bunch
            // between two steps, where they would leave the matrix pipe idle.
#pragma unroll
            for (int m = 0; m < A_T * B_T; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);       // address arithmetic
                if (m < B_T) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);              // one LDS read
                else if (m < B_T + A_T) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // one global load
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        // End of a tile: every wavefront leaves the partial tiles it does not own in LDS before the item's
        // barrier (the reduction area is separate from the input buffers and was last read a barrier ago),
        // then adds the four partial sums of the tiles it owns, in the order of the wavefronts, and stores them.
        float *red = reinterpret_cast<float *>(lds + g.red_off);
        if (KSP == 4 && ch == nch - 1) {
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r)
#pragma unroll
                for (int o = 0; o < NOWN; ++o) {
                    if (o == w) continue;
                    const int tau = r * 4 + o;
                    const int wi = w < o ? w : w - 1;
                    float *dst = red + (((r * NOWN + o) * 3 + wi) * 4) * 256 + lane * 4;
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4)
                        *reinterpret_cast<float4 *>(dst + q4 * 256) =
                            make_float4(acc[tau / B_T][tau % B_T][q4 * 4 + 0], acc[tau / B_T][tau % B_T][q4 * 4 + 1],
                                        acc[tau / B_T][tau % B_T][q4 * 4 + 2], acc[tau / B_T][tau % B_T][q4 * 4 + 3]);
                }
        }
        __syncthreads();

        if (KSP == 1 && ch == nch - 1) pc_ks_store_pixels<A_T, B_T, ACT>(acc, lds, g, w, lane, mt, tn, gy0, gx0, npix, osrc, msrc);
        if (KSP == 4 && ch == nch - 1) {
            const int n = tn + o_ti, gy = gy0 + o_y, gx = gx0 + o_x;
            const bool pix_ok = qo < npix && n < g.N && gy < g.GH && gx < g.GW;
            const int oy = gy * g.oscale + g.ooff_y, ox = gx * g.oscale + g.ooff_x;
            const uint32_t opix_off = pix_ok ? (uint32_t)((n * g.out_H + oy) * g.out_W + ox) * (uint32_t)(g.out_CH * 2) : OOB_OUT;
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
#pragma unroll
                for (int o = 0; o < NOWN; ++o) {
                    if (o != w) continue;
                    const int tau = r * 4 + o;
                    const int ti_ = tau / B_T;
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                        for (int ws = 0; ws < 4; ++ws) {
                            float4 p;
                            if (ws == o)
                                p = make_float4(acc[tau / B_T][tau % B_T][q4 * 4 + 0], acc[tau / B_T][tau % B_T][q4 * 4 + 1],
                                                acc[tau / B_T][tau % B_T][q4 * 4 + 2], acc[tau / B_T][tau % B_T][q4 * 4 + 3]);
                            else
                                p = *reinterpret_cast<const float4 *>(red + (((r * NOWN + o) * 3 + (ws < o ? ws : ws - 1)) * 4 + q4) * 256 + lane * 4);
                            if (ws == 0) s = p;
                            else { s.x += p.x; s.y += p.y; s.z += p.z; s.w += p.w; }
                        }
                        // a store past the end of the buffer is dropped: pixels and channels outside the output need no branch
                        const int m = (mt * A_T + ti_) * 32 + q4 * 8 + (lane >> 5) * 4;
                        uint2 pkd;
                        pkd.x = pc_pack_bf16x2(s.x, s.y);
                        pkd.y = pc_pack_bf16x2(s.z, s.w);
                        v2u32 pv = {pkd.x, pkd.y};
                        const int ooff = (int)((m < g.out_CH ? opix_off : OOB_OUT) + (uint32_t)(m * 2));
                        if (ACT == PC_ACT_RELU) {
                            pv[0] = pc_relu_bf16x2(pv[0]);
                            pv[1] = pc_relu_bf16x2(pv[1]);
                        } else if (ACT == PC_ACT_RELU_MASK) {
                            const v2u32 mk = __builtin_amdgcn_raw_buffer_load_b64(msrc, ooff, 0, 0);
                            pv[0] = pc_mask_bf16x2(pv[0], mk[0]);
                            pv[1] = pc_mask_bf16x2(pv[1], mk[1]);
                        }
                        __builtin_amdgcn_raw_buffer_store_b64(pv, osrc, ooff, 0, 0);
                    }
                }
            }
        }
        if (ch == nch - 1) {
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                for (int j = 0; j < B_T; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[ii][j][r] = 0.0f;
        }
        k = nk; ch = nchk; mt = nmt; tn = ntn; gy0 = ngy0; gx0 = ngx0;
        ab = abn;
    }
}

// ------------------------------------------------------------------ structured-sparse variant
// The same kernel with the pixels split over the MFMA wavefronts (tiles of 64 output channels x 128*B_T/... pixels),
// multiplying with v_smfmac_f32_32x32x32_bf16: the weight operand holds at most 2 nonzeros in every 4 consecutive
// reduction entries of a row and the instruction covers 32 reduction entries in the time the dense one covers 16.
// A hard-pruned layer has a weight density of keep * 4/9 per (filter, tap, channel), so nearly every group of 4
// channels holds at most 2 kept weights; the rest (third and fourth nonzeros of a group) form a second operand of
// the same kind whose instruction is issued only for the (row tile, tap, step) fragments where it is not all zero
// (flag bits written at pack time). Both together are exact for any mask; the number of instructions falls with
// the sparsity. Operand layout (measured): the B operand of one instruction is the B operands of two consecutive
// dense steps (16 entries per lane); lane l of the A operand holds row l % 32 and, of the 16 entries of dense step
// l / 32, two stored values per group of 4 with their 2-bit positions in the low (part 1) or high (part 2) half of
// the index word (selected by the instruction's last operand).
typedef __bf16 bf16x16 __attribute__((ext_vector_type(16)));

// The MFMA wavefronts of the structured-sparse kernel. OVF: the overflow weights (third and fourth nonzeros of a
// group of 4) are multiplied as extra reduction columns of a dense matrix instruction at the end of every item, from
// the lists the pack wrote; else through the second operand part, one more sparse instruction wherever a fragment
// holds any. Both are exact; the lists are the cheaper form (a handful of columns per item) but have a fixed
// capacity, which a pack reports per list.
template <int B_T, int KC, int ACT, bool OVF>
__device__ __forceinline__ void pc_sp_mfma_role(uint16_t *__restrict__ out, const SparseOperand &sp, const MfmaArgs &g, unsigned char *lds,
                                                int vb, int G, int ntile_blk, int nch, int lane, int w)
{
    constexpr int A_T = 2;
    constexpr int SS = KC / 32;           // sparse steps per tap and chunk
    constexpr int S = 9 * SS;             // steps per item
    constexpr int NSET = S * A_T;         // operand sets (part 1, part 2, index word) per item
    // sets in flight (what the registers hold beside accumulators and B operands): the kernel's speed follows this depth
    // (56 x 56, 256 -> 256, batch 32, forward, overflow lists: 116 / 111 / 104 us at 6 / 9 / 12 sets)
    constexpr int PFD = pc_ring_depth(NSET, OVF ? 12 : 6);
    constexpr int PITCH = 2 * KC + 16;
    constexpr int DBS = (B_T >= 4 || OVF) ? 1 : 2;   // B operands are read this many steps ahead
    constexpr int RB = DBS + 1;
    static_assert(!OVF || KC == 64, "the overflow lists are per chunk of 64 reduction entries");
    const uint16_t *__restrict__ wsv = sp.val;
    const uint32_t *__restrict__ wsi = sp.idx;
    const uint16_t *__restrict__ wsf = sp.flag;
    const int I = ntile_blk * nch;
    const int npix = g.TI * g.TH * g.TW;
    int base[B_T];
#pragma unroll
    for (int j = 0; j < B_T; ++j) {
        int q = (w * B_T + j) * 32 + (lane & 31);
        if (q >= npix) q = npix - 1;
        const int ti = (int)pc_udiv((uint32_t)q, g.mg_THTW);
        const int rem = q - ti * g.TH * g.TW;
        const int y = (int)pc_udiv((uint32_t)rem, g.mg_TW), x = rem - y * g.TW;
        base[j] = ((ti * g.IH + y * g.lstep) * g.IW + x * g.lstep) * PITCH + (lane >> 5) * 16;
    }
    const __amdgpu_buffer_rsrc_t osrc = __builtin_amdgcn_make_buffer_rsrc(out, 0, g.out_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t msrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(ACT == PC_ACT_RELU_MASK ? g.act_mask : out), 0, g.out_bytes, 0x00020000);
    // Operand sets are read with buffer loads, the lane's bytes as the vector offset and everything else scalar:
    // set (row tile ii, tap t, step s) of an item lies (ii*9 + t) * KS32 + s sets past the item's first one; a set is
    // 2 KiB of values (part 1, part 2) and 256 bytes of index words.
    const int KS32 = g.KS >> 1;
    const __amdgpu_buffer_rsrc_t vsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(wsv), 0, g.wz_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t isrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(wsi), 0, g.wz_bytes >> 3, 0x00020000);
    const int nlists_all = ((g.out_CH + 127) / 128 * 4) * (KS32 >> 1);
    const __amdgpu_buffer_rsrc_t oasrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(sp.ov_a), 0,
                                                                            OVF ? nlists_all * (PC_OV_STEPS * 1024) : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t ocsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t *>(sp.ov_col), 0,
                                                                            OVF ? nlists_all * (PC_OV_STEPS * 64) : 0, 0x00020000);
    const int v_voff = lane * 16, i_voff = lane * 4;
    const int ksb = KS32 * 2048;          // bytes of values between the sets of two taps
    auto set_off = [&](int p) -> int {    // p: compile-time set index inside the item
        const int st = p / A_T, ii = p % A_T;
        return (ii * 9 + st / SS) * ksb + (st % SS) * 2048;
    };
    // (live = false: the lane's offset is past the buffer, the load returns zeros and moves nothing; the part-2 loads of
    // fragments without a nonzero are switched off this way, so that every load stays unconditional and the compiler
    // can count the loads in flight)
    auto load_vals = [&](int item_base, int p, int part, bool live = true) -> bf16x8 {
        const v4u32 r = __builtin_amdgcn_raw_buffer_load_b128(vsrc, live ? v_voff : (int)0x80000000u, item_base + set_off(p) + part * 1024, 0);
        bf16x8 o;
        __builtin_memcpy(&o, &r, 16);
        return o;
    };
    auto load_idx = [&](int item_base, int p) -> uint32_t {
        return __builtin_amdgcn_raw_buffer_load_b32(isrc, i_voff, (item_base + set_off(p)) >> 3, 0);
    };
    // flag bits of the part-2 operands of an item: bit 16*s + t of word ii (KC = 64), bit t (KC = 32)
    auto load_flags = [&](int mt_, int ch_, uint32_t &f0, uint32_t &f1) {
        if (OVF) {                                   // the step counts of the item's two overflow lists instead
            const int l0 = (mt_ * A_T) * (KS32 >> 1) + ch_;
            f0 = __builtin_amdgcn_readfirstlane(sp.ov_cnt[l0]);
            f1 = __builtin_amdgcn_readfirstlane(sp.ov_cnt[l0 + (KS32 >> 1)]);
            return;
        }
        const int r0 = (mt_ * A_T) * KS32 + ch_ * SS, r1 = r0 + KS32;
        uint32_t a, b;
        if (SS == 2) {
            a = reinterpret_cast<const uint32_t *>(wsf)[r0 >> 1];
            b = reinterpret_cast<const uint32_t *>(wsf)[r1 >> 1];
        } else {
            a = wsf[r0];
            b = wsf[r1];
        }
        f0 = __builtin_amdgcn_readfirstlane(a);
        f1 = __builtin_amdgcn_readfirstlane(b);
    };
    auto flag_of = [&](uint32_t f0, uint32_t f1, int p) -> bool {
        if (OVF) return false;
        const int st = p / A_T, ii = p % A_T;
        return (((ii ? f1 : f0) >> (16 * (st % SS) + st / SS)) & 1u) != 0u;
    };
    auto tap_off = [&](int t) -> int { return g.tap_o0 + (t / 3) * g.tap_dr + (t % 3) * g.tap_ds; };
    int mt = 0, tn = 0, gy0 = 0, gx0 = 0;
    auto tile_of = [&](int k, int &mt_, int &tn_, int &gy0_, int &gx0_) {
        const uint32_t t = (uint32_t)(vb + k * G);
        const uint32_t tq = pc_udiv(t, g.mg_fd), trm = t - tq * g.fdiv;
        const uint32_t pt = g.m_fast ? tq : trm;
        mt_ = (int)(g.m_fast ? trm : tq);
        const uint32_t u = pc_udiv(pt, g.mg_tx);
        const int tx = (int)(pt - u * g.tiles_x);
        const uint32_t tnn = pc_udiv(u, g.mg_ty);
        const int ty = (int)(u - tnn * g.tiles_y);
        tn_ = (int)tnn * g.TI;
        gy0_ = ty * g.TH;
        gx0_ = tx * g.TW;
    };
    auto a_base = [&](int mt_, int ch_) -> int { return ((mt_ * A_T * 9) * KS32 + ch_ * SS) * 2048; };
    tile_of(0, mt, tn, gy0, gx0);
    int k = 0, ch = 0;
    int ab = a_base(mt, 0);
    uint32_t fl0, fl1;
    load_flags(mt, 0, fl0, fl1);

    f32x16 acc[A_T][B_T];
#pragma unroll
    for (int i = 0; i < A_T; ++i)
#pragma unroll
        for (int j = 0; j < B_T; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    bf16x8 r1[PFD], r2[PFD];
    uint32_t rx[PFD];
#pragma unroll
    for (int p = 0; p < PFD; ++p) {
        r1[p] = load_vals(ab, p, 0);
        rx[p] = load_idx(ab, p);
        if (!OVF) r2[p] = load_vals(ab, p, 1, flag_of(fl0, fl1, p));
    }

    // Overflow lists (OVF): the first step's A operand and columns of an item's two lists are requested during the item
    // before, decoded and gathered from the staged tile during the first steps of the item, and multiplied there.
    bf16x8 oa0[A_T];
    v4u32 oc0[A_T][2];
    auto load_ovf = [&](int mt_, int ch_) {
#pragma unroll
        for (int ii = 0; ii < A_T; ++ii) {
            const int l = (mt_ * A_T + ii) * (KS32 >> 1) + ch_;
            const v4u32 t = __builtin_amdgcn_raw_buffer_load_b128(oasrc, v_voff, l * (PC_OV_STEPS * 1024), 0);
            __builtin_memcpy(&oa0[ii], &t, 16);
            oc0[ii][0] = __builtin_amdgcn_raw_buffer_load_b128(ocsrc, (lane >> 5) * 32, l * (PC_OV_STEPS * 64), 0);
            oc0[ii][1] = __builtin_amdgcn_raw_buffer_load_b128(ocsrc, (lane >> 5) * 32 + 16, l * (PC_OV_STEPS * 64), 0);
        }
    };
    if (OVF) load_ovf(mt, 0);
    auto col_off = [&](uint32_t c) -> int {
        return g.tap_o0 + __mul24((int)(c >> 12), g.tap_dr) + __mul24((int)((c >> 8) & 15u), g.tap_ds) + (int)(c & 255u) * 2;
    };
    auto as_b = [&](const uint32_t (&h)[8]) -> bf16x8 {
        const uint32_t wd[4] = {h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
        bf16x8 o;
        __builtin_memcpy(&o, wd, 16);
        return o;
    };

    __syncthreads();
    for (int i = 0; i < I; ++i) {
        int nk = k, nchk = ch + 1, nmt = mt, ntn = tn, ngy0 = gy0, ngx0 = gx0;
        if (nchk == nch) {
            nchk = 0;
            nk = k + 1;
            if (nk < ntile_blk) tile_of(nk, nmt, ntn, ngy0, ngx0);
            else nchk = ch;
        }
        const int abn = a_base(nmt, nchk);
        uint32_t nfl0, nfl1;
        load_flags(nmt, nchk, nfl0, nfl1);
        const unsigned char *xb = lds + (i & 1) * g.xbuf;

        auto read_b = [&](int st, int j) -> bf16x16 {   // the B operands of dense steps 2s and 2s+1 of the tap
            const unsigned char *pb = xb + base[j] + tap_off(st / SS) + (st % SS) * 64;
            const bf16x8 lo = *reinterpret_cast<const bf16x8 *>(pb), hi = *reinterpret_cast<const bf16x8 *>(pb + 32);
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
        };
        int ooff[A_T][8];
        bf16x8 obg[A_T][B_T];
        bf16x16 bring[RB][B_T];
#pragma unroll
        for (int d = 0; d < DBS; ++d)
#pragma unroll
            for (int j = 0; j < B_T; ++j) bring[d % RB][j] = read_b(d, j);
#pragma unroll
        for (int st = 0; st < S; ++st) {
            if (st + DBS < S) {
#pragma unroll
                for (int j = 0; j < B_T; ++j) bring[(st + DBS) % RB][j] = read_b(st + DBS, j);
            }
            bf16x8 a1[A_T], a2[A_T];
            uint32_t ax[A_T];
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii) {
                const int p = st * A_T + ii, np = p + PFD;
                a1[ii] = r1[p % PFD];
                if (!OVF) a2[ii] = r2[p % PFD];
                ax[ii] = rx[p % PFD];
                // refill the slot with the set PFD ahead: of this item, or of the next one
                r1[p % PFD] = np < NSET ? load_vals(ab, np < NSET ? np : 0, 0) : load_vals(abn, np < NSET ? 0 : np - NSET, 0);
                rx[p % PFD] = np < NSET ? load_idx(ab, np < NSET ? np : 0) : load_idx(abn, np < NSET ? 0 : np - NSET);
                if (!OVF)
                    r2[p % PFD] = np < NSET ? load_vals(ab, np < NSET ? np : 0, 1, flag_of(fl0, fl1, np < NSET ? np : 0))
                                            : load_vals(abn, np < NSET ? 0 : np - NSET, 1, flag_of(nfl0, nfl1, np < NSET ? 0 : np - NSET));
            }
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    acc[ii][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a1[ii], bring[st % RB][j], acc[ii][j], (int)ax[ii], 0, 0);
#pragma unroll
            for (int m = 0; m < A_T * B_T; ++m) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one matrix instruction
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);       // address arithmetic
                if (m < B_T) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);              // the two LDS reads of a B operand
                else if (m < B_T + A_T) __builtin_amdgcn_sched_group_barrier(0x020, OVF ? 2 : 3, 0);   // the value parts and the index word of a set
            }
            if (OVF) {
                // the first overflow step of the item's two lists, spread over the first steps of the item
                if (st == 0) {
#pragma unroll
                    for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                        for (int e = 0; e < 8; ++e) ooff[ii][e] = col_off(e < 4 ? oc0[ii][0][e] : oc0[ii][1][e - 4]);
                }
                if (st >= 1 && st <= A_T * B_T) {            // one (row tile, pixel sub-tile) gather per step
                    const int ii = (st - 1) / B_T, j = (st - 1) % B_T;
                    const unsigned char *pb = xb + base[j] - (lane >> 5) * 16;
                    uint32_t h[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) h[e] = *reinterpret_cast<const uint16_t *>(pb + ooff[ii][e]);
                    obg[ii][j] = as_b(h);
                }
                if (st == A_T * B_T + 2) {
#pragma unroll
                    for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                        for (int j = 0; j < B_T; ++j)
                            acc[ii][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(oa0[ii], obg[ii][j], acc[ii][j], 0, 0, 0);
                }
                if (st == A_T * B_T + 4) load_ovf(nmt, nchk);  // the next item's (past the end: this one's again, unused)
            }
            __builtin_amdgcn_sched_barrier(0);
            // the second parts: only where the pack found a nonzero (uniform branches on scalar bits)
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii) {
                if (flag_of(fl0, fl1, st * A_T + ii)) {
#pragma unroll
                    for (int j = 0; j < B_T; ++j)
                        acc[ii][j] = __builtin_amdgcn_smfmac_f32_32x32x32_bf16(a2[ii], bring[st % RB][j], acc[ii][j], (int)ax[ii], 0, 1);
                }
            }
        }
        if (OVF) {
            // Further steps of a list (more than 16 overflow weights: the exception): every column of a step is one
            // overflow weight; its B operand is gathered element by element from the staged tile (lane l: pixel l % 32,
            // columns 8 * (l / 32) .. + 7), its A operand has the weight in the row it belongs to and zeros elsewhere.
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii) {
                const int nst = (int)(ii ? fl1 : fl0);
                const int l = (mt * A_T + ii) * (KS32 >> 1) + ch;
                for (int s = 1; s < nst; ++s) {
                    const v4u32 t = __builtin_amdgcn_raw_buffer_load_b128(oasrc, v_voff, (l * PC_OV_STEPS + s) * 1024, 0);
                    bf16x8 oa;
                    __builtin_memcpy(&oa, &t, 16);
                    const v4u32 c0 = __builtin_amdgcn_raw_buffer_load_b128(ocsrc, (lane >> 5) * 32, (l * PC_OV_STEPS + s) * 64, 0);
                    const v4u32 c1 = __builtin_amdgcn_raw_buffer_load_b128(ocsrc, (lane >> 5) * 32 + 16, (l * PC_OV_STEPS + s) * 64, 0);
                    int off[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) off[e] = col_off(e < 4 ? c0[e] : c1[e - 4]);
                    bf16x8 bg[B_T];
#pragma unroll
                    for (int j = 0; j < B_T; ++j) {
                        const unsigned char *pb = xb + base[j] - (lane >> 5) * 16;
                        uint32_t h[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) h[e] = *reinterpret_cast<const uint16_t *>(pb + off[e]);
                        bg[j] = as_b(h);
                    }
#pragma unroll
                    for (int j = 0; j < B_T; ++j)
                        acc[ii][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(oa, bg[j], acc[ii][j], 0, 0, 0);
                }
            }
        }
        __syncthreads();
        if (ch == nch - 1) {
            pc_ks_store_pixels<A_T, B_T, ACT>(acc, lds, g, w, lane, mt, tn, gy0, gx0, npix, osrc, msrc);
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii)
#pragma unroll
                for (int j = 0; j < B_T; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[ii][j][r] = 0.0f;
        }
        k = nk; ch = nchk; mt = nmt; tn = ntn; gy0 = ngy0; gx0 = ngx0;
        ab = abn;
        fl0 = nfl0; fl1 = nfl1;
    }
}

template <int B_T, int KC, int ACT = PC_ACT_NONE>
__global__ void __launch_bounds__(512, 1)
pc_mfma_conv_sp_kernel(const uint16_t *__restrict__ in, uint16_t *__restrict__ out, SparseOperand sp, MfmaArgs g)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int NV = KS_NV1;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int w = wave & 3;
    const int G = gridDim.x;
    int vb = blockIdx.x;
    if ((G & 7) == 0) vb = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);
    const int ntile_blk = (g.total_tiles - vb + G - 1) / G;
    const int nch = g.nchunks;

    if (wave >= 4) {
        pc_ks_loader_role<KC, NV>(in, g, lds, vb, G, ntile_blk, nch);
        return;
    }
    // Does every overflow list of the layer fit? Every MFMA wavefront reads all the counters (a few hundred) and
    // reaches the same answer, so the four need not talk to each other before they pick their loop.
    bool fits = KC == 64 && sp.ov_cnt != nullptr;
    if (fits) {
        const int nlists = ((g.out_CH + 127) / 128 * 4) * (g.KS >> 2);
        bool bad = false;
        for (int l = lane; l < nlists; l += 64) bad |= sp.ov_cnt[l] == PC_OV_BAD;
        fits = __ballot(bad) == 0ull;
    }
    if (fits) {
        if constexpr (KC == 64) pc_sp_mfma_role<B_T, KC, ACT, true>(out, sp, g, lds, vb, G, ntile_blk, nch, lane, w);
    } else {
        pc_sp_mfma_role<B_T, KC, ACT, false>(out, sp, g, lds, vb, G, ntile_blk, nch, lane, w);
    }
}

// ---- wave-specialised kernel: plan and launch (9-tap launches whose channel count is a multiple of 8)
#define KS_LDS_MAX (160 * 1024)

template <int A_T, int B_T, int KC, int KSP, int ACT>
static hipError_t launch_ks_act(int device, hipStream_t st, int grid, size_t lds, const uint16_t *in, uint16_t *out,
                                const uint16_t *wz, const MfmaArgs &g)
{
    static pc_per_device_once attr;
    if (pc_once_pending(attr, device)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pc_mfma_conv_ks_kernel<A_T, B_T, 9, KC, KSP, ACT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, KS_LDS_MAX);
        if (e != hipSuccess) return e;
        pc_once_done(attr, device);
    }
    hipLaunchKernelGGL((pc_mfma_conv_ks_kernel<A_T, B_T, 9, KC, KSP, ACT>), dim3((unsigned)grid), dim3(512), lds, st, in, out, wz, g);
    return hipGetLastError();
}

template <int A_T, int B_T, int KC, int KSP>
static hipError_t launch_ks(int device, hipStream_t st, int grid, size_t lds, const uint16_t *in, uint16_t *out,
                            const uint16_t *wz, const MfmaArgs &g, int act)
{
    if (act == PC_ACT_RELU) return launch_ks_act<A_T, B_T, KC, KSP, PC_ACT_RELU>(device, st, grid, lds, in, out, wz, g);
    if (act == PC_ACT_RELU_MASK) return launch_ks_act<A_T, B_T, KC, KSP, PC_ACT_RELU_MASK>(device, st, grid, lds, in, out, wz, g);
    return launch_ks_act<A_T, B_T, KC, KSP, PC_ACT_NONE>(device, st, grid, lds, in, out, wz, g);
}

template <int B_T, int KC, int ACT>
static hipError_t launch_sp_act(int device, hipStream_t st, int grid, size_t lds, const uint16_t *in, uint16_t *out,
                                const SparseOperand &sp, const MfmaArgs &g)
{
    static pc_per_device_once attr;
    if (pc_once_pending(attr, device)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pc_mfma_conv_sp_kernel<B_T, KC, ACT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, KS_LDS_MAX);
        if (e != hipSuccess) return e;
        pc_once_done(attr, device);
    }
    hipLaunchKernelGGL((pc_mfma_conv_sp_kernel<B_T, KC, ACT>), dim3((unsigned)grid), dim3(512), lds, st, in, out, sp, g);
    return hipGetLastError();
}

template <int B_T, int KC>
static hipError_t launch_sp(int device, hipStream_t st, int grid, size_t lds, const uint16_t *in, uint16_t *out,
                            const SparseOperand &sp, const MfmaArgs &g, int act)
{
    if (act == PC_ACT_RELU) return launch_sp_act<B_T, KC, PC_ACT_RELU>(device, st, grid, lds, in, out, sp, g);
    if (act == PC_ACT_RELU_MASK) return launch_sp_act<B_T, KC, PC_ACT_RELU_MASK>(device, st, grid, lds, in, out, sp, g);
    return launch_sp_act<B_T, KC, PC_ACT_NONE>(device, st, grid, lds, in, out, sp, g);
}

// Fills the tile plan; false when the staged tile does not fit. ksp = 4: the MFMA wavefronts split the
// reduction of a tile of 32*bt pixels (64-channel chunks); ksp = 1: they split a tile of 128*bt pixels
// (32-channel chunks, no reduction across wavefronts).
static bool plan_ks(const MfmaArgs &g, int ext, int at, int bt, int ksp, int kc, MfmaArgs *out, size_t *lds_bytes, double *est, int num_cu)
{
    const int pitch = 2 * kc + 16, parts = kc / 8, nv = ksp == 4 ? KS_NV : KS_NV1;
    MfmaArgs t = g;
    pc_plan_mfma_tiles(&t, (ksp == 4 ? 32 : 128) * bt, ext);
    const int nt = at * bt, nown = nt >= 4 ? 4 : nt;
    const int red_bytes = ksp == 4 ? (nt >= 4 ? nt / 4 : 1) * nown * 12288 : 4 * 64 * 144;   // reduction area / store staging
    // staged pixels: within the loader's registers (nv 16-byte elements per thread) and within LDS
    int cap = 256 * nv / parts;
    if (cap > (KS_LDS_MAX - red_bytes - 32) / (2 * pitch)) cap = (KS_LDS_MAX - red_bytes - 32) / (2 * pitch);
    while (t.TI * t.IH * t.IW > cap) {
        if (t.TI > 1) --t.TI;
        else if (t.TH > 1) {
            t.TH = (t.TH + 1) / 2;
            t.IH = (t.TH - 1) * t.lstep + ext;
            t.tiles_y = (t.GH + t.TH - 1) / t.TH;
        } else return false;
    }
    const int HP = t.TI * t.IH * t.IW;
    t.nelem = HP * parts;
    t.xbuf = HP * pitch + 16;   // one spare 16-byte slot for the loader threads without an element
    t.red_off = 2 * t.xbuf;
    *lds_bytes = (size_t)t.red_off + (size_t)red_bytes;
    if (*lds_bytes > KS_LDS_MAX) return false;
    t.m_tiles = (g.out_CH + 32 * at - 1) / (32 * at);
    const int64_t p_tiles = (int64_t)((t.N + t.TI - 1) / t.TI) * t.tiles_y * t.tiles_x;
    const int64_t total = p_tiles * t.m_tiles;
    if (total > (1 << 30)) return false;
    t.total_tiles = (int)total;
    // Tiles that follow each other run side by side, mostly on one XCD, and share what their common index
    // reads through that XCD's L2: the input tile when the row tile runs fastest, the weights of a row
    // tile when the pixel tile does. The bigger of the two operands is the one to share.
    const int64_t w_bytes = (int64_t)g.out_CH * g.in_CH * 18, x_bytes = (int64_t)g.N * g.in_H * g.in_W * g.in_CH * 2;
    t.m_fast = x_bytes >= w_bytes;
    t.fdiv = t.m_fast ? t.m_tiles : (int)p_tiles;
    int64_t dmax = t.fdiv > t.tiles_x ? t.fdiv : t.tiles_x;
    if (t.tiles_y > dmax) dmax = t.tiles_y;
    if (total * dmax >= ((int64_t)1 << 32)) return false;   // the multiply-high divisions of the tile index stay exact
    const int64_t in_bytes = (int64_t)g.N * g.in_H * g.in_W * g.in_CH * 2;
    if (in_bytes >= ((int64_t)1 << 31)) return false;   // 32-bit buffer offsets, with 2^31 as the out-of-range marker
    t.in_bytes = (uint32_t)in_bytes;
    const int64_t out_bytes = (int64_t)g.N * g.out_H * g.out_W * g.out_CH * 2;
    if (out_bytes >= ((int64_t)1 << 31) || (g.out_CH & (ksp == 4 ? 3 : 7))) return false;   // 8- or 16-byte buffer stores
    t.out_bytes = (uint32_t)out_bytes;
    auto magic = [](int d) { return pc_udiv_magic(d); };
    t.mg_IW = magic(t.IW); t.mg_IH = magic(t.IH); t.mg_TW = magic(t.TW); t.mg_THTW = magic(t.TH * t.TW);
    t.mg_fd = magic(t.fdiv); t.mg_tx = magic(t.tiles_x); t.mg_ty = magic(t.tiles_y);
    t.nchunks = (g.in_CH + kc - 1) / kc;
    t.cps = t.nchunks;
    // cycles of one workgroup: tiles per workgroup x (MFMAs of a tile at 32 cycles each per wavefront + the tile's
    // fixed cost: the reduction across wavefronts, or just the store)
    const int64_t rounds = (total + num_cu - 1) / num_cu;
    // (an item also costs a barrier and the refill of the fragment pipelines: about 450 cycles; inside an item the
    // MFMAs issue at about 70 % of their peak rate in both splits, which weighs the fixed costs against them)
    const double mfma_eff = 0.7;
    if (ksp == 4) *est = (double)rounds * ((double)t.nchunks * (288.0 * at * bt * kc / 64 / mfma_eff + 450.0) + 2500.0);
    else *est = (double)rounds * ((double)t.nchunks * (18.0 * kc * at * bt / mfma_eff + 450.0) + 1200.0);
    // A workgroup with a single 512-pixel tile overlaps nothing: it loads its whole input, multiplies, then stores.
    // Two 256-pixel tiles hide the second load and the first store (measured with cold caches on 32x32 maps,
    // 64 -> 64 channels, batch 128: 23.5 us against 29.8 us), which the cycle count above does not see.
    // With more tiles the smaller tile still gains in the step (shorter loader and store bursts): 1-1.5 % of the
    // ImageNet-sized workloads' steps, measured with this factor at 1.2 and at 1.5.
    if (ksp == 1 && bt == 4) *est *= rounds == 1 ? 1.6 : 1.2;
    *out = t;
    return true;
}

// PC_OK: launched. PC_ERR_UNSUPPORTED without a message: not applicable, the caller uses the other kernel.
pc_status pc_run_mfma_conv_ws(pc_ctx *ctx, int pcfg, const MfmaArgs &g0, int ext, const int *tr, const int *tc,
                              const uint16_t *in, uint16_t *out, const uint16_t *wz, const SparseOperand &sp, bool *launched, int act)
{
    *launched = false;
    // The structured-sparse kernel (override code 22; automatic from 64 reduction channels up): 64 x 256 tiles,
    // 64-channel chunks, pixels split over the MFMA wavefronts.
    if (sp.val && g0.lstep == 1 && (pcfg == 22 || (pcfg < 0 && g0.in_CH >= 64))) {
        MfmaArgs t;
        size_t lds;
        double est;
        bool ok = plan_ks(g0, ext, 2, 2, 1, 64, &t, &lds, &est, ctx->num_cu);
        for (int q = 0; q < 9 && ok; ++q)
            if (t.tap_w[q] != q || tr[q] != (tr[0] ? 2 - q / 3 : q / 3) || tc[q] != (tc[0] ? 2 - q % 3 : q % 3)) ok = false;
        if (ok) {
            const int pitch = 2 * 64 + 16;
            t.tap_dr = (tr[0] ? -1 : 1) * t.IW * pitch;
            t.tap_ds = (tc[0] ? -1 : 1) * pitch;
            t.tap_o0 = (tr[0] * t.IW + tc[0]) * pitch;
            t.wz_bytes = (uint32_t)((size_t)((t.out_CH + 127) / 128 * 4) * 9 * t.KS * 1024);
            const int grid = t.total_tiles < ctx->num_cu ? t.total_tiles : ctx->num_cu;
            const hipError_t e = launch_sp<2, 64>(ctx->device, ctx->stream, grid, lds, in, out, sp, t, act);
            *launched = true;
            pc_note_kernel(ctx, "pc_mfma_conv_sp_kernel<2, 64, %d>", act);
            return pc_hip_check(ctx, e, "MFMA conv (structured-sparse) launch");
        }
        if (pcfg == 22) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: the structured-sparse kernel does not fit this launch");
    }
    if (pcfg == 22) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: the pack holds no structured-sparse operand");
    // candidates: (pixel-tile factor, reduction split); override codes 7, 8, 9 and 13 force one of them
    enum { NCAND = 12 };
    static const int kAt[NCAND] = {2, 2, 2, 2, 2, 1, 2, 2, 2, 1, 2, 2}, kBt[NCAND] = {4, 2, 1, 4, 1, 1, 2, 4, 2, 4, 2, 2},
                     kKsp[NCAND] = {4, 4, 4, 1, 4, 4, 1, 1, 1, 1, 1, 4}, kKc[NCAND] = {64, 64, 64, 32, 128, 128, 32, 16, 16, 32, 64, 128},
                     kCode[NCAND] = {7, 8, 9, 13, 14, 15, 16, 17, 18, 19, 20, 21};
    MfmaArgs best;
    size_t best_lds = 0;
    double best_est = 0.0;
    int best_k = -1;
    for (int k = 0; k < NCAND; ++k) {
        if (pcfg >= 7 && pcfg != kCode[k]) continue;
        // 16-channel chunks are for the few input channels of a first layer and for stride-2 forward passes (the staged tile
        // has four times the pixels of the output tile: with wider chunks it no longer fits and the output tile shrinks:
        // 56 x 56, 128 -> 128, batch 64: 47.6 -> 40.5 us), 32-row tiles for a first layer's few output channels
        if (pcfg < 0 && ((kKc[k] == 16 && g0.in_CH > 16 && g0.lstep != 2) || (kKc[k] != 16 && g0.in_CH <= 16) || (kAt[k] == 1 && kKsp[k] == 1) != (g0.out_CH <= 32))) continue;
        MfmaArgs t;
        size_t lds;
        double est;
        if (!plan_ks(g0, ext, kAt[k], kBt[k], kKsp[k], kKc[k], &t, &lds, &est, ctx->num_cu)) continue;
        if (best_k < 0 || est < best_est) { best = t; best_lds = lds; best_est = est; best_k = k; }
    }
    if (best_k < 0) return PC_OK;
    // The end-of-tile reduction costs about as much as 64 channels of MFMA work: up to 128 reduction channels
    // the cooperative kernel's output split is faster, unless every workgroup has a single tile.
    if (pcfg < 0 && kKsp[best_k] == 4 && (g0.in_CH <= 64 || (g0.in_CH <= 128 && best.total_tiles > ctx->num_cu))) return PC_OK;
    MfmaArgs g = best;
    const int pitch = 2 * kKc[best_k] + 16;
    // the tap list is the full 3x3 in tap order, forward (offset (r, s)) or rotated (offset (2-r, 2-s))
    for (int t = 0; t < 9; ++t)
        if (g.tap_w[t] != t || tr[t] != (tr[0] ? 2 - t / 3 : t / 3) || tc[t] != (tc[0] ? 2 - t % 3 : t % 3)) return PC_OK;
    g.tap_dr = (tr[0] ? -1 : 1) * g.IW * pitch;
    g.tap_ds = (tc[0] ? -1 : 1) * pitch;
    g.tap_o0 = (tr[0] * g.IW + tc[0]) * pitch;
    g.wz_bytes = (uint32_t)((size_t)((g.out_CH + 127) / 128 * 4) * 9 * g.KS * 1024);
    const int grid = g.total_tiles < ctx->num_cu ? g.total_tiles : ctx->num_cu;
    hipError_t e;
    switch (best_k) {
    case 0: e = launch_ks<2, 4, 64, 4>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 1: e = launch_ks<2, 2, 64, 4>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 2: e = launch_ks<2, 1, 64, 4>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 3: e = launch_ks<2, 4, 32, 1>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 4: e = launch_ks<2, 1, 128, 4>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 5: e = launch_ks<1, 1, 128, 4>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 6: e = launch_ks<2, 2, 32, 1>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 7: e = launch_ks<2, 4, 16, 1>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 8: e = launch_ks<2, 2, 16, 1>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 9: e = launch_ks<1, 4, 32, 1>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    case 10: e = launch_ks<2, 2, 64, 1>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    default: e = launch_ks<2, 2, 128, 4>(ctx->device, ctx->stream, grid, best_lds, in, out, wz, g, act); break;
    }
    *launched = true;
    pc_note_kernel(ctx, "pc_mfma_conv_ks_kernel<%d, %d, 9, %d, %d, %d>", kAt[best_k], kBt[best_k], kKc[best_k], kKsp[best_k], act);
    return pc_hip_check(ctx, e, "MFMA conv (wave-specialised) launch");
}

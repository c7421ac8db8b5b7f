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
typedef uint32_t v4u32 __attribute__((ext_vector_type(4)));
typedef uint32_t v2u32 __attribute__((ext_vector_type(2)));

#define MF_LDS_MAX 65536

#ifdef EXP_TIMING
__device__ long long pc_wgrad_dbg[32];
extern "C" void pc_debug_read(long long *out) { (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(pc_wgrad_dbg), sizeof(long long) * 32); }
#define TSTAMP(i) do { if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0) pc_wgrad_dbg[i] = wall_clock64(); } while (0)
#else
#define TSTAMP(i)
#endif
bool pc_mfma_supports(int F, int C) { return (int64_t)F * C < (1 << 23); }   // kinfo packs the slot in 23 bits

struct MfmaArgs {
    int32_t N, in_H, in_W, in_CH;
    int32_t out_H, out_W, out_CH;
    int32_t GH, GW, oscale, ooff_y, ooff_x;
    int32_t iscale, ioff_y, ioff_x, lstep;
    int32_t TI, TH, TW, IH, IW;
    int32_t tiles_y, tiles_x;
    int32_t KS;              // k-steps of 16 in the packed operand (padded reduction length / 16)
    int32_t nchunks, cps;    // chunks of KC channels in total, and per split (blockIdx.z)
    int32_t tap_w[9];        // weight tap index of every list entry
    int32_t tap_off[9];      // LDS byte offset of every list entry
    // used by the wave-specialised kernel only
    int32_t m_tiles, total_tiles;   // row tiles of the output channels; all tiles
    int32_t m_fast, fdiv;           // tile index = slow * fdiv + fast; m_fast: the row tile is the fast index (fdiv = m_tiles), else the pixel tile
    int32_t xbuf, red_off, nelem;   // bytes per staged input buffer, LDS offset of the reduction area, 16-byte elements per buffer
    uint32_t in_bytes, out_bytes, wz_bytes;   // sizes of the input, output and operand-tile buffers (bounds of the buffer accesses)
    int32_t tap_o0, tap_dr, tap_ds; // LDS byte offset of tap 3r+s = tap_o0 + r*tap_dr + s*tap_ds
    // divisions by these run as a multiply-high with floor(2^32 / d) + 1 (exact while dividend * d < 2^32)
    uint32_t mg_IW, mg_IH, mg_TW, mg_THTW, mg_fd, mg_tx, mg_ty;
};

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
template <int A_T, int B_T, int WAVES_M, int WAVES_N, int NTAPS, int KC>
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
        return *reinterpret_cast<const bf16x8 *>(wzl + (int64_t)((i * 9 + g.tap_w[t]) * g.KS + chc * KSC + ks) * 512);
    };
    bf16x8 aring[PF][A_T];
#pragma unroll
    for (int d = 0; d < PF; ++d)
#pragma unroll
        for (int i = 0; i < A_T; ++i) aring[d][i] = a_load(ch0, d, i);

#ifdef EXP_TIMING_CONV
#define CSTAMP(i) TSTAMP(i)
#else
#define CSTAMP(i)
#endif
    CSTAMP(0);
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
    int csi = 2;
    CSTAMP(1);
    for (int ch = ch0; ch < ch1; ++ch) {
        __syncthreads();
        CSTAMP(csi); csi++;
        for (int e = threadIdx.x; e < HP * PARTS; e += 256) {
            const int q = e / PARTS, part = e - q * PARTS;
            const int c = ch * KC + part * 8;
            const int64_t po = pixoff[q];
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (po >= 0 && c < g.in_CH) {
                if ((g.in_CH & 7) == 0) {
                    v = *reinterpret_cast<const uint4 *>(in + po + c);
                } else {   // channel count not a multiple of 8: rows are not 16-byte aligned, load by element
                    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (c + i < g.in_CH) w[i >> 1] |= (uint32_t)in[po + c + i] << ((i & 1) * 16);
                    v = make_uint4(w[0], w[1], w[2], w[3]);
                }
            }
            *reinterpret_cast<uint4 *>(lds + q * PITCH + part * 16) = v;
        }
        CSTAMP(csi); csi++;
        __syncthreads();
        CSTAMP(csi); csi++;
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
                bring[d % RB][j] = *reinterpret_cast<const bf16x8 *>(lds + base[j] + g.tap_off[t1] + k1 * 32);
        }
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            if (st + DB < NS) {
                const int t1 = (st + DB) / KSC, k1 = (st + DB) % KSC;
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    bring[(st + DB) % RB][j] = *reinterpret_cast<const bf16x8 *>(lds + base[j] + g.tap_off[t1] + k1 * 32);
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
#pragma unroll
            for (int i = 0; i < A_T; ++i)
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(anow[i], bring[st % RB][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    CSTAMP(30);
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
    CSTAMP(31);
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
#ifdef EXP_TIMING_KS
#define KSTAMP(i) do { if (blockIdx.x == 0 && (threadIdx.x & 255) == 0) pc_wgrad_dbg[i] = wall_clock64(); } while (0)
#else
#define KSTAMP(i)
#endif
#define KS_NV 8          // 16-byte elements staged per loader thread and item (256 loader threads), reduction split
#define KS_NV1 12        // the same without the reduction split (512-pixel tiles of 32 channels)
#define KS_DEPTH 3       // items in flight in the loader's registers

// q / d with mg = floor(2^32 / d) + 1 from the host (exact while q * d < 2^32); mg == 0 stands for d == 1
__device__ __forceinline__ uint32_t pc_udiv(uint32_t q, uint32_t mg) { return mg ? __umulhi(q, mg) : q; }

// Depth of the A-fragment ring: the largest divisor of the fragments per item that does not exceed cap
constexpr int pc_ring_depth(int nf, int cap)
{
    int best = 1;
    for (int d = 1; d <= cap; ++d)
        if (nf % d == 0) best = d;
    return best;
}

template <int A_T, int B_T, int NTAPS, int KC, int KSP>
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
        // ------------------------------------------------------------ loaders
        KSTAMP(16);
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
        KSTAMP(17);
        issue(R0); issue(R1);
        KSTAMP(18);
        put(R0, 0);
        KSTAMP(19);
        __syncthreads();
        KSTAMP(20);
        issue(R2); issue(R0);
        // item i: while the MFMA wavefronts work on buffer i&1, write item i+1 (register set (i+1)%3) to the
        // other buffer (past the last item: zeros, never read) and refill that set with item i+4
        auto lstep = [&](int i, uint4 (&R)[NV]) {
#ifndef EXP_KS_NO_LOADER
            put(R, ((i + 1) & 1) * g.xbuf);
#endif
            if (i < 4) KSTAMP(21 + 2 * i);
#ifndef EXP_KS_NO_LOADER
            issue(R);
#endif
            __syncthreads();
            if (i < 4) KSTAMP(22 + 2 * i);
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
        return;
    }

    // ---------------------------------------------------------------- MFMA wavefronts
    KSTAMP(0);
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

    KSTAMP(1);
    __syncthreads();
    KSTAMP(2);
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
#ifndef EXP_KS_NO_B
            if (st + DBS < S) {
#pragma unroll
                for (int j = 0; j < B_T; ++j)
                    bring[(st + DBS) % RB][j] =
                        *reinterpret_cast<const bf16x8 *>(xb + base[j] + tap_off((st + DBS) / KSW) + ((st + DBS) % KSW) * 32);
            }
#else
            if (st + DBS < S) {
#pragma unroll
                for (int j = 0; j < B_T; ++j) bring[(st + DBS) % RB][j] = bring[st % RB][j];
            }
#endif
            bf16x8 anow[A_T];
#pragma unroll
            for (int ii = 0; ii < A_T; ++ii) {
                const int ph = st * A_T + ii;
                anow[ii] = aring[ph % PFD];
                const int nph = ph + PFD;
#ifndef EXP_KS_NO_A
                aring[ph % PFD] = nph < NF ? a_frag(ab, nph < NF ? nph : 0) : a_frag(abn, nph < NF ? 0 : nph - NF);
#endif
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
        if (i < 4) KSTAMP(3 + 2 * i);
        __syncthreads();
        if (i < 4) KSTAMP(4 + 2 * i);

        if (KSP == 1 && ch == nch - 1) {
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
                    const bool ok = q < npix && n < g.N && gy < g.GH && gx < g.GW && m < g.out_CH;
                    const int oy = gy * g.oscale + g.ooff_y, ox = gx * g.oscale + g.ooff_x;
                    const uint32_t off = ok ? (uint32_t)((n * g.out_H + oy) * g.out_W + ox) * (uint32_t)(g.out_CH * 2) + (uint32_t)(m * 2) : OOB_OUT;
                    const v4u32 pv = {v.x, v.y, v.z, v.w};
                    __builtin_amdgcn_raw_buffer_store_b128(pv, osrc, (int)off, 0, 0);
                }
            }
        }
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
                        const v2u32 pv = {pkd.x, pkd.y};
                        __builtin_amdgcn_raw_buffer_store_b64(pv, osrc, (int)((m < g.out_CH ? opix_off : OOB_OUT) + (uint32_t)(m * 2)), 0, 0);
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
            if (k == 0) KSTAMP(12);
        }
        if (i == I - 1) KSTAMP(13);
        k = nk; ch = nchk; mt = nmt; tn = ntn; gy0 = ngy0; gx0 = ngx0;
        ab = abn;
    }
}

// ------------------------------------------------------------------ operand tiles
// wz_fwd[mt][tap][ks][lane][8]: mt = filter/32, ks = channel/16; element i of lane l is
// w[f = 32*mt + l%32][c = 16*ks + 8*(l/32) + i][tap], zero when pruned or padded.
// wz_bwd has the roles of filter and channel exchanged (rows = channels, k = filters).
__global__ void __launch_bounds__(256)
pc_pack_tiles_kernel(const float *__restrict__ W, LibArg la, PackView v, int64_t total_fwd)
{
    // one launch fills both operands: the first total_fwd threads wz_fwd, the others wz_bwd
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int bwd = idx >= total_fwd;
    if (bwd) idx -= total_fwd;
    const int Mp = bwd ? v.Cp : v.Fp;          // padded row count (multiple of 128)
    const int KS = (bwd ? v.Fk : v.Ck) / 16;   // padded reduction length / 16
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
    const int64_t total_fwd = (int64_t)(v.Fp / 32) * 9 * (v.Ck / 16) * 64, total_bwd = (int64_t)(v.Cp / 32) * 9 * (v.Fk / 16) * 64;
    hipLaunchKernelGGL(pc_pack_tiles_kernel, dim3((unsigned)((total_fwd + total_bwd + 255) / 256)), dim3(256), 0, ctx->stream,
                       W, la, v, total_fwd);
    return pc_hip_check(ctx, hipGetLastError(), "pack tiles launch");
}

// ------------------------------------------------------------------ planning and launch
struct MfmaCfg { int a, b, wm, wn, kc; };
static const MfmaCfg kCfgs[] = {
    {2, 4, 1, 4, 32}, {2, 4, 2, 2, 32}, {2, 2, 2, 2, 32}, {2, 2, 2, 2, 64}, {1, 2, 2, 2, 64}, {1, 1, 2, 2, 64},
    {1, 2, 2, 2, 16},
};
// automatic choice tries these in order and keeps the first that yields enough workgroups (else the last)
static const int kAutoOrder[] = {4, 5};
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

template <int A_T, int B_T, int WM, int WN, int KC>
static void launch_cfg(hipStream_t st, dim3 grid, size_t lds, int ntaps, const uint16_t *in, uint16_t *out,
                       const uint16_t *wz, float *partial, const MfmaArgs &g)
{
    switch (ntaps) {
    case 9: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 9, KC>), grid, dim3(256), lds, st, in, out, wz, partial, g); break;
    case 4: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 4, KC>), grid, dim3(256), lds, st, in, out, wz, partial, g); break;
    case 2: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 2, KC>), grid, dim3(256), lds, st, in, out, wz, partial, g); break;
    default: hipLaunchKernelGGL((pc_mfma_conv_kernel<A_T, B_T, WM, WN, 1, KC>), grid, dim3(256), lds, st, in, out, wz, partial, g); break;
    }
}


// ---- wave-specialised kernel: plan and launch (9-tap launches whose channel count is a multiple of 8)
#define KS_LDS_MAX (160 * 1024)

template <int A_T, int B_T, int KC, int KSP>
static hipError_t launch_ks(hipStream_t st, int grid, size_t lds, const uint16_t *in, uint16_t *out, const uint16_t *wz,
                            const MfmaArgs &g)
{
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&pc_mfma_conv_ks_kernel<A_T, B_T, 9, KC, KSP>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, KS_LDS_MAX);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    hipLaunchKernelGGL((pc_mfma_conv_ks_kernel<A_T, B_T, 9, KC, KSP>), dim3((unsigned)grid), dim3(512), lds, st, in, out, wz, g);
    return hipGetLastError();
}

// Fills the tile plan; false when the staged tile does not fit. ksp = 4: the MFMA wavefronts split the
// reduction of a tile of 32*bt pixels (64-channel chunks); ksp = 1: they split a tile of 128*bt pixels
// (32-channel chunks, no reduction across wavefronts).
static bool plan_ks(const MfmaArgs &g, int ext, int at, int bt, int ksp, int kc, MfmaArgs *out, size_t *lds_bytes, double *est, int num_cu)
{
    const int pitch = 2 * kc + 16, parts = kc / 8, nv = ksp == 4 ? KS_NV : KS_NV1;
    MfmaArgs t = g;
    plan_mfma_tiles(&t, (ksp == 4 ? 32 : 128) * bt, ext);
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
    auto magic = [](int d) { return d == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) / (uint64_t)d) + 1); };
    t.mg_IW = magic(t.IW); t.mg_IH = magic(t.IH); t.mg_TW = magic(t.TW); t.mg_THTW = magic(t.TH * t.TW);
    t.mg_fd = magic(t.fdiv); t.mg_tx = magic(t.tiles_x); t.mg_ty = magic(t.tiles_y);
    t.nchunks = (g.in_CH + kc - 1) / kc;
    t.cps = t.nchunks;
    // cycles of one workgroup: tiles per workgroup x (MFMAs of a tile at 32 cycles each per wavefront + the tile's
    // fixed cost: the reduction across wavefronts, or just the store)
    const int64_t rounds = (total + num_cu - 1) / num_cu;
    // (an item also costs a barrier and the refill of the fragment pipelines: about 450 cycles)
    if (ksp == 4) *est = (double)rounds * ((double)t.nchunks * (288.0 * at * bt * kc / 64 + 450.0) + 2500.0);
    else *est = (double)rounds * ((double)t.nchunks * (1152.0 * bt + 450.0) + 1200.0);
    *out = t;
    return true;
}

// PC_OK: launched. PC_ERR_UNSUPPORTED without a message: not applicable, the caller uses the other kernel.
static pc_status run_mfma_conv_ks(pc_ctx *ctx, int pcfg, const MfmaArgs &g0, int ext, const int *tr, const int *tc, const uint16_t *in,
                                  uint16_t *out, const uint16_t *wz, bool *launched)
{
    *launched = false;
    // candidates: (pixel-tile factor, reduction split); override codes 7, 8, 9 and 13 force one of them
    enum { NCAND = 6 };
    static const int kAt[NCAND] = {2, 2, 2, 2, 2, 1}, kBt[NCAND] = {4, 2, 1, 4, 1, 1}, kKsp[NCAND] = {4, 4, 4, 1, 4, 4},
                     kKc[NCAND] = {64, 64, 64, 32, 128, 128}, kCode[NCAND] = {7, 8, 9, 13, 14, 15};
    MfmaArgs best;
    size_t best_lds = 0;
    double best_est = 0.0;
    int best_k = -1;
    for (int k = 0; k < NCAND; ++k) {
        if (pcfg >= 7 && pcfg != kCode[k]) continue;
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
    case 0: e = launch_ks<2, 4, 64, 4>(ctx->stream, grid, best_lds, in, out, wz, g); break;
    case 1: e = launch_ks<2, 2, 64, 4>(ctx->stream, grid, best_lds, in, out, wz, g); break;
    case 2: e = launch_ks<2, 1, 64, 4>(ctx->stream, grid, best_lds, in, out, wz, g); break;
    case 3: e = launch_ks<2, 4, 32, 1>(ctx->stream, grid, best_lds, in, out, wz, g); break;
    case 4: e = launch_ks<2, 1, 128, 4>(ctx->stream, grid, best_lds, in, out, wz, g); break;
    default: e = launch_ks<1, 1, 128, 4>(ctx->stream, grid, best_lds, in, out, wz, g); break;
    }
    *launched = true;
    return pc_hip_check(ctx, e, "MFMA conv (wave-specialised) launch");
}

// g holds everything but the tile plan; ext = reach of the tap offsets (3 or 2); tap rows/cols in tr/tc.
static pc_status run_mfma_conv(pc_ctx *ctx, MfmaArgs g, int ext, int ntaps, const int *tr, const int *tc,
                               const uint16_t *in, uint16_t *out, const uint16_t *wz)
{
    int plan_cfg = (ctx->plan_cfg >= 10 && ctx->plan_cfg < 13) ? -1 : ctx->plan_cfg;   // 10 and 11 select a backward-weight kernel
    if (ntaps == 9 && (g.in_CH & 7) == 0 && g.in_CH >= 32 && (plan_cfg < 0 || plan_cfg >= 7) && ctx->plan_split == 0) {
        bool launched = false;
        pc_status s = run_mfma_conv_ks(ctx, plan_cfg, g, ext, tr, tc, in, out, wz, &launched);
        if (launched || s != PC_OK) return s;
    }
    if (plan_cfg >= 7) {   // forced wave-specialised kernel: launches it cannot take (tap subsets) use the automatic choice
        if (ntaps == 9) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA conv: the wave-specialised kernel does not fit this launch");
        plan_cfg = -1;
    }
    int pick = -1, pick_split = 1;
    MfmaArgs best = g;
    const int64_t want = 2 * (int64_t)ctx->num_cu;
    const int n_try = plan_cfg >= 0 ? 1 : (int)(sizeof(kAutoOrder) / sizeof(kAutoOrder[0]));
    for (int k = 0; k < n_try; ++k) {
        int ci = plan_cfg >= 0 ? plan_cfg : kAutoOrder[k];
        if (plan_cfg < 0 && g.in_CH <= 16) ci = 6;   // a handful of input channels: one 16-channel k-step per tap
        const MfmaCfg &c = kCfgs[ci];
        int BM = 32 * c.a * c.wm, BN = 32 * c.b * c.wn;
        MfmaArgs t = g;
        plan_mfma_tiles(&t, BN, ext);
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
        int64_t blocks = (int64_t)((t.N + t.TI - 1) / t.TI) * t.tiles_y * t.tiles_x * ((g.out_CH + BM - 1) / BM);
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
    for (int t = 0; t < ntaps; ++t) g.tap_off[t] = (tr[t] * g.IW + tc[t]) * (2 * c.kc + 16);
    int BM = 32 * c.a * c.wm;
    dim3 grid((unsigned)(((g.N + g.TI - 1) / g.TI) * g.tiles_y * g.tiles_x), (unsigned)((g.out_CH + BM - 1) / BM),
              (unsigned)pick_split);
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
    case 0: launch_cfg<2, 4, 1, 4, 32>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    case 1: launch_cfg<2, 4, 2, 2, 32>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    case 2: launch_cfg<2, 2, 2, 2, 32>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    case 3: launch_cfg<2, 2, 2, 2, 64>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    case 4: launch_cfg<1, 2, 2, 2, 64>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    case 5: launch_cfg<1, 1, 2, 2, 64>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    default: launch_cfg<1, 2, 2, 2, 16>(ctx->stream, grid, lds, ntaps, in, out, wz, partial, g); break;
    }
    pc_status s = pc_hip_check(ctx, hipGetLastError(), "MFMA conv launch");
    if (s != PC_OK || pick_split == 1) return s;
    int64_t n4 = n_out / 4;
    hipLaunchKernelGGL(pc_mfma_splitk_reduce_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, ctx->stream,
                       (const float4 *)partial, n4, pick_split, (uint2 *)out);
    return pc_hip_check(ctx, hipGetLastError(), "split-K reduce launch");
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
    int32_t nnzk;
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

    TSTAMP(0);
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
    TSTAMP(1);

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
    TSTAMP(2);
    if (kt < a.n_ktiles) issue(kt);
    TSTAMP(3);
    int tsi = 4;
    for (; kt < a.n_ktiles; kt += a.ksplit) {
        __syncthreads();
        TSTAMP(tsi); tsi++;
#ifndef EXP_NO_XPOSE
        pc_transpose8x8_store(rd, dyT + (tcg * 8) * WG_DY_PLANE + tcg * 16 + (d_slot << 4), WG_DY_PLANE);
#pragma unroll
        for (int k = 0; k < WG_XTASKS; ++k)
            if (has_x[k]) pc_transpose8x8_store(rx[k], xT + (tcg * 8) * a.xplane + tcg * 16 + (x_slot[k] << 4), a.xplane);
#else
        if (rd[0].x == 0x12345u && rx[0][0].x == 77u && rx[1][1].y == 5u && rx[2][2].z == 6u) dyT[threadIdx.x] = 1;
#endif
        __syncthreads();
        TSTAMP(tsi); tsi++;
        if (kt + a.ksplit < a.n_ktiles) issue(kt + a.ksplit);
        TSTAMP(tsi); tsi++;

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
    TSTAMP(20);
    // Epilogue, one filter half (32 filters) at a time: the waves park their tiles of that half in LDS as
    // out[tap][filter][channel] (float32, 72 KiB), then every thread walks 8 kernels (f, c) of the half and,
    // for the kept ones, gathers the 4 kept taps and writes them as one 16-byte entry in compact slot order.
    float *pout = partial + (int64_t)blockIdx.z * a.nnzk * 4;
    float *ot = reinterpret_cast<float *>(lds);
#pragma unroll
    for (int fh = 0; fh < 2; ++fh) {
        __syncthreads();
        const int h = fh == first_half ? 0 : 1;   // this wave's unit range holding filter half fh
        TSTAMP(22 + fh * 3);
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
        TSTAMP(23 + fh * 3);
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
    TSTAMP(21);
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
#ifdef EXP_TIMING_WS
#define WSTAMP(i) do { if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && (threadIdx.x & 255) == 0) pc_wgrad_dbg[i] = wall_clock64(); } while (0)
#else
#define WSTAMP(i)
#endif
#define WS_NSLOT 16
#define WS_NKS (WS_NSLOT / 2)
#define WS_XSLOTS 48
#define WS_DY_PLANE (WS_NSLOT * 16 + 16)
#define WS_LDS_MAX (160 * 1024 - 256)   // dynamic part; the kernel has a few bytes of static LDS too

struct WgradWsArgs {
    int32_t N, H, W, C, F, Ho, Wo, stride;   // C: channels of the x tensor the kernel reads (padded to a multiple of 8)
    int32_t Creal;                           // channels of the layer (row length of the kinfo table)
    int32_t TR, TC, npos, ng, IR, IC, xs_per_g, xslots, xplane;
    int32_t tiles_r, tiles_c, n_ktiles, ksplit, nnzk;
    int32_t buf_bytes;                     // one LDS buffer: dyT planes, then xT planes
    uint32_t x_bytes, dy_bytes;            // tensor sizes (bounds of the buffer loads)
    uint32_t mg_tc, mg_tr;                 // multiply-high constants of the divisions by tiles_c and tiles_r
    int16_t xb_tab[WS_NSLOT];              // x slot read by dy slot s for tap (0,0)
    uint32_t dy_tab[WS_NSLOT];             // dy slot -> (image group << 16) | (row << 8) | column; 0xFFFFFFFF = unused
    uint32_t x_tab[WS_XSLOTS];             // x slot  -> (image group << 16) | (row << 8) | column inside the x region
};

__global__ void __launch_bounds__(512, 1)
pc_mfma_wgrad_ws_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dy, WgradWsArgs a, PackView v,
                        float *__restrict__ partial, float *__restrict__ dw)
{
    extern __shared__ __align__(16) unsigned char lds[];
    constexpr int XT_OFF = WG_T * WS_DY_PLANE + 128;   // xT planes inside a buffer
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // Workgroups go to the XCDs round-robin by their linear index. The index is re-read so that the workgroups of
    // one XCD share as few pixel splits as possible: each XCD's L2 then fetches its own slice of x and dy once,
    // instead of every XCD fetching all of both.
    int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z;
    {
        const int T = gridDim.x * gridDim.y, ks = a.ksplit;
        const int lin = bx + gridDim.x * (by + gridDim.y * bz);
        const int xcd = lin & 7, r = lin >> 3;
        int tile = -1;
        if ((ks & 7) == 0) {                           // an XCD owns ks/8 splits, all tiles of each
            tile = r % T;
            bz = (r / T) * 8 + xcd;
        } else if (ks < 8 && (8 % ks) == 0 && (T % (8 / ks)) == 0) {   // 8/ks XCDs share a split
            bz = xcd % ks;
            tile = r * (8 / ks) + xcd / ks;
        }
        if (tile >= 0) { bx = tile % (int)gridDim.x; by = tile / (int)gridDim.x; }
    }
    const int c0 = bx * WG_T, f0 = by * WG_T;
    const int nt = (a.n_ktiles - bz + a.ksplit - 1) / a.ksplit;   // pixel tiles of this workgroup
    WSTAMP(0);

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
                kinf[fh][k] = (f < a.F && c < a.Creal) ? v.kinfo[(int64_t)f * a.Creal + c] : 0xFFFFFFFFu;
            }
    };
    float *pout = a.ksplit > 1 ? partial + (int64_t)bz * a.nnzk * 4 : dw;
    const float *ot = reinterpret_cast<const float *>(lds);
    // gathers the 4 kept taps of every kept kernel of filter half fh from the parked tile
    auto gather = [&](int fh) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int p = threadIdx.x + 512 * k;
            const uint32_t info = kinf[fh][k];
            if (info != 0xFFFFFFFFu) {
                uint32_t m = info & 0x1FFu;
                const float *ob = ot + (p >> 6) * WG_T + (p & 63);
                float o[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int t = __builtin_ctz(m);
                    m &= m - 1u;
                    o[j] = ob[t * (32 * WG_T)];
                }
                *reinterpret_cast<float4 *>(pout + (int64_t)(info >> 9) * 4) = make_float4(o[0], o[1], o[2], o[3]);
            }
        }
    };

    if (wave >= 4) {
        // ------------------------------------------------------------ loaders
        WSTAMP(16);
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
        const uint32_t tab0 = dy0 ? a.dy_tab[slot0] : (slot0 < a.xslots ? a.x_tab[slot0] : 0xFFFFFFFFu);
        const uint32_t tab1 = slot1 < a.xslots ? a.x_tab[slot1] : 0xFFFFFFFFu;
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
        WSTAMP(17);
        issue(A0, B0); issue(A1, B1);
        load_kinfo();
        WSTAMP(18);
        put(A0, B0, 0);
        WSTAMP(19);
        __syncthreads();
        WSTAMP(20);
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
            put(A1, B1, a.buf_bytes); if (i == 0) WSTAMP(21); issue(A1, B1); if (i == 0) WSTAMP(22); sync(); if (i == 0) WSTAMP(23);
            put(A0, B0, 0);           if (i == 0) WSTAMP(24); issue(A0, B0); sync(); if (i == 0) WSTAMP(25);
        }
        if (i < nt) { put(A1, B1, a.buf_bytes); issue(A1, B1); sync(); }
#pragma unroll
        for (int fh = 0; fh < 2; ++fh) {
            __syncthreads();
            __syncthreads();
            gather(fh);
        }
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
        for (int kk = 0; kk < WS_NKS; ++kk) xb[kk] = a.xb_tab[2 * kk + g];
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

        WSTAMP(1);
        __syncthreads();
        WSTAMP(2);
        for (int i = 0; i < nt; ++i) {
            const unsigned char *bufp = lds + (i & 1) * a.buf_bytes;
            const unsigned char *ar0 = bufp + o_a0, *ar1 = bufp + o_a1, *bc = bufp + o_b;
            bf16x8 aq[2][2], bq[2][5];
            aq[0][0] = *reinterpret_cast<const bf16x8 *>(ar0);
            aq[0][1] = *reinterpret_cast<const bf16x8 *>(ar1);
#pragma unroll
            for (int b = 0; b < 5; ++b) bq[0][b] = *reinterpret_cast<const bf16x8 *>(bc + ((xb[0] + toff[b]) << 4));
#pragma unroll
            for (int kk = 0; kk < WS_NKS; ++kk) {
                const int cur = kk & 1, nxt = cur ^ 1;
                if (kk + 1 < WS_NKS) {
                    aq[nxt][0] = *reinterpret_cast<const bf16x8 *>(ar0 + (kk + 1) * 32);
                    aq[nxt][1] = *reinterpret_cast<const bf16x8 *>(ar1 + (kk + 1) * 32);
                    const unsigned char *bk = bc + (xb[kk + 1 < WS_NKS ? kk + 1 : 0] << 4);
#pragma unroll
                    for (int b = 0; b < 5; ++b) bq[nxt][b] = *reinterpret_cast<const bf16x8 *>(bk + (toff[b] << 4));
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
            if (i < 4) WSTAMP(3 + 2 * i);
            __syncthreads();
            if (i < 4) WSTAMP(4 + 2 * i);
        }
        // epilogue, one filter half at a time: park the half's tiles as out[tap][filter][channel] (72 KiB)
        float *otw = reinterpret_cast<float *>(lds);
#pragma unroll
        for (int fh = 0; fh < 2; ++fh) {
            __syncthreads();
            const int h = fh == first_half ? 0 : 1;
#pragma unroll
            for (int b = 0; b < 5; ++b) {
                if (h == 0 || b < 4) {
                    const int tap = tg ? 8 - b : b;
                    float *tp = otw + (tap * 32) * WG_T + cl;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const int fr = 8 * (i >> 2) + 4 * g + (i & 3);
                        tp[fr * WG_T] = h == 0 ? acc[b][i] : acc[5 + (b < 4 ? b : 0)][i];
                    }
                }
            }
            __syncthreads();
            gather(fh);
        }
    }

}

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

// Wave-specialised backward-weight: plan and launch. *launched stays false when the layer is outside what
// that kernel takes (the caller then uses the cooperative kernel).
static pc_status pc_mfma_bwd_weight_ws(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, const void *dy,
                                       float *dw, int64_t nnzk, bool *launched)
{
    *launched = false;
    WgradWsArgs a;
    memset(&a, 0, sizeof(a));
    const int st = d->stride;
    a.N = d->N; a.H = d->H; a.W = d->W; a.C = (d->C + 7) / 8 * 8; a.Creal = d->C; a.F = d->F; a.stride = st;
    a.Ho = (d->H - 1) / st + 1; a.Wo = (d->W - 1) / st + 1;
    // 16-byte buffer loads of 8 channels. An input whose channel count is no multiple of 8 (the first layer's 3)
    // is first copied to rows padded to 8 channels; an output-gradient with such a filter count is left to the
    // cooperative kernel, which reads by element.
    if (a.F & 7) return PC_OK;
    const bool pad_x = a.C != a.Creal;
    const int64_t xb = (int64_t)a.N * a.H * a.W * a.C * 2, db = (int64_t)a.N * a.Ho * a.Wo * a.F * 2;
    if (xb >= ((int64_t)1 << 31) || db >= ((int64_t)1 << 31)) return PC_OK;
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
    if (best_eff < 0.0) return PC_OK;
    a.TR = best_tr; a.TC = best_tc; a.npos = a.TR * a.TC; a.ng = best_ng;
    a.IR = (a.TR - 1) * st + 3; a.IC = (a.TC - 1) * st + 3;
    a.xs_per_g = a.IR * a.IC;
    a.xslots = (a.ng * a.xs_per_g + 7) / 8 * 8;
    if (a.xslots > WS_XSLOTS) return PC_OK;
    a.xplane = a.xslots * 16 + 16;
    a.tiles_r = (a.Ho + a.TR - 1) / a.TR;
    a.tiles_c = (a.Wo + a.TC - 1) / a.TC;
    const int tiles_n = (ngroups + a.ng - 1) / a.ng;
    const int64_t nkt = (int64_t)tiles_n * a.tiles_r * a.tiles_c;
    if (nkt * (a.tiles_r > a.tiles_c ? a.tiles_r : a.tiles_c) >= ((int64_t)1 << 31)) return PC_OK;
    a.n_ktiles = (int)nkt;
    a.nnzk = (int32_t)nnzk;
    auto magic = [](int dd) { return dd == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) / (uint64_t)dd) + 1); };
    a.mg_tc = magic(a.tiles_c); a.mg_tr = magic(a.tiles_r);
    for (int sl = 0; sl < WS_NSLOT; ++sl) {
        const int ig = sl / a.npos, pos = sl % a.npos, py = pos / a.TC, px = pos % a.TC;
        const bool ok = ig < a.ng;
        a.dy_tab[sl] = ok ? ((uint32_t)ig << 16) | ((uint32_t)py << 8) | (uint32_t)px : 0xFFFFFFFFu;
        a.xb_tab[sl] = ok ? (int16_t)(ig * a.xs_per_g + py * st * a.IC + px * st) : (int16_t)0;
    }
    for (int xs = 0; xs < WS_XSLOTS; ++xs) {
        const int ig = xs / a.xs_per_g, rem = xs % a.xs_per_g;
        a.x_tab[xs] = (ig < a.ng) ? ((uint32_t)ig << 16) | ((uint32_t)(rem / a.IC) << 8) | (uint32_t)(rem % a.IC) : 0xFFFFFFFFu;
    }
    a.buf_bytes = (WG_T * WS_DY_PLANE + 128 + WG_T * a.xplane + 128 + 255) / 256 * 256;
    size_t lds = 2 * (size_t)a.buf_bytes;
    if (lds < (size_t)9 * 32 * WG_T * sizeof(float)) lds = (size_t)9 * 32 * WG_T * sizeof(float);   // the epilogue parks one filter half
    if (lds > WS_LDS_MAX) return PC_OK;
    int ks = ctx->num_cu / (ft * ct);
    if (ks > a.n_ktiles) ks = a.n_ktiles;
    if (ks < 1) ks = 1;
    a.ksplit = ks;
    void *scr = nullptr;
    const size_t part_bytes = ks > 1 ? (sizeof(float) * 4 * (size_t)ks * (size_t)nnzk + 255) / 256 * 256 : 0;
    if (part_bytes || pad_x) {
        pc_status s = pc_scratch(ctx, part_bytes + (pad_x ? (size_t)xb : 0), &scr);
        if (s != PC_OK) return s;
    }
    if (pad_x) {
        uint4 *xp = reinterpret_cast<uint4 *>(static_cast<unsigned char *>(scr) + part_bytes);
        const int64_t npix = (int64_t)a.N * a.H * a.W, n16 = npix * (a.C / 8);
        hipLaunchKernelGGL(pc_pad_channels_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, ctx->stream,
                           (const uint16_t *)x, xp, npix, a.Creal, a.C);
        x = xp;
    }
    static bool attr_done = false;
    if (!attr_done) {
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_ws_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, WS_LDS_MAX));
        attr_done = true;
    }
    hipLaunchKernelGGL(pc_mfma_wgrad_ws_kernel, dim3((unsigned)ct, (unsigned)ft, (unsigned)ks), dim3(512), lds, ctx->stream,
                       (const uint16_t *)x, (const uint16_t *)dy, a, pk->v, (float *)scr, dw);
    *launched = true;
    pc_status s = pc_hip_check(ctx, hipGetLastError(), "MFMA bwd_weight (wave-specialised) launch");
    if (s != PC_OK || ks == 1) return s;
    return pc_launch_wgrad_reduce(ctx, (const float *)scr, ks, pk, dw);
}

pc_status pc_mfma_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, const void *dy,
                             float *dw)
{
    int64_t nnzk = 0;
    pc_status s = pc_packed_info(ctx, pk, &nnzk, nullptr);
    if (s != PC_OK) return s;
    if (nnzk == 0) return PC_OK;
    if (ctx->plan_cfg != 10) {   // 10 forces the cooperative kernel
        bool launched = false;
        s = pc_mfma_bwd_weight_ws(ctx, d, pk, x, dy, dw, nnzk, &launched);
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
    a.nnzk = (int32_t)nnzk;
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
    static bool lds_attr_set = false;
    if (!lds_attr_set) {
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<12>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        PC_HIP(ctx, hipFuncSetAttribute((const void *)pc_mfma_wgrad_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, WG_LDS_MAX));
        lds_attr_set = true;
    }
    int ft = (a.F + WG_T - 1) / WG_T, ct = (a.C + WG_T - 1) / WG_T;
    if (a.xslots > 32 * WG_XTASKS) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA bwd_weight: x tile too large");
    int ks = ctx->num_cu / (ft * ct);
    if (ks > a.n_ktiles) ks = a.n_ktiles;
    if (ks < 1) ks = 1;
    a.ksplit = ks;
    void *scr = nullptr;
    s = pc_scratch(ctx, sizeof(float) * 4 * (size_t)ks * (size_t)nnzk, &scr);
    if (s != PC_OK) return s;
    const dim3 grid((unsigned)ct, (unsigned)ft, (unsigned)ks);
    const uint16_t *xp = (const uint16_t *)x, *dyp = (const uint16_t *)dy;
    if (a.nks <= 4) hipLaunchKernelGGL(pc_mfma_wgrad_kernel<4>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    else if (a.nks <= 8) hipLaunchKernelGGL(pc_mfma_wgrad_kernel<8>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    else if (a.nks <= 12) hipLaunchKernelGGL(pc_mfma_wgrad_kernel<12>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    else hipLaunchKernelGGL(pc_mfma_wgrad_kernel<16>, grid, dim3(256), lds, ctx->stream, xp, dyp, a, pk->v, (float *)scr);
    s = pc_hip_check(ctx, hipGetLastError(), "MFMA bwd_weight launch");
    if (s != PC_OK) return s;
    return pc_launch_wgrad_reduce(ctx, (const float *)scr, ks, pk, dw);
}

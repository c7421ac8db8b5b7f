// Shared declarations of the matrix-core (MFMA) kernels: operand vector types, the launch description of the
// forward/backward-data kernels, and the helpers both of those kernels' planners use.
#ifndef PC_MFMA_H
#define PC_MFMA_H
#include "pc_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t v4u32 __attribute__((ext_vector_type(4)));
typedef uint32_t v2u32 __attribute__((ext_vector_type(2)));

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
    // stride-2 backward-data as one launch: the four input-pixel parity classes (1, 2, 2 and 4 taps) are four
    // ranges of blockIdx.x, each with its own output offset, extent and tap list (cls_tiles = 0: not used)
    int32_t cls_tiles;               // pixel tiles per class
    int32_t cls_GH[4], cls_GW[4], cls_ooy[4], cls_oox[4], cls_ntaps[4];
    int32_t cls_tap_w[4][4], cls_tap_off[4][4];   // entries past the class's tap count repeat a valid one
    // used by the wave-specialised kernel only
    int32_t m_tiles, total_tiles;   // row tiles of the output channels; all tiles
    int32_t m_fast, fdiv;           // tile index = slow * fdiv + fast; m_fast: the row tile is the fast index (fdiv = m_tiles), else the pixel tile
    int32_t xbuf, red_off, nelem;   // bytes per staged input buffer, LDS offset of the reduction area, 16-byte elements per buffer
    uint32_t in_bytes, out_bytes, wz_bytes;   // sizes of the input, output and operand-tile buffers (bounds of the buffer accesses)
    int32_t tap_o0, tap_dr, tap_ds; // LDS byte offset of tap 3r+s = tap_o0 + r*tap_dr + s*tap_ds
    // divisions by these run as a multiply-high with floor(2^32 / d) + 1 (exact while dividend * d < 2^32)
    uint32_t mg_IW, mg_IH, mg_TW, mg_THTW, mg_fd, mg_tx, mg_ty;
    // wave-specialised kernel with a fused activation step: a tensor of the output's shape whose positive elements
    // let the output through (the ReLU derivative of the backward pass); unused otherwise
    const uint16_t *act_mask;
};

// Fused step at the end of a conv launch (Section 5.2: a = sigma(z) forward, the error times sigma'(z) backward).
enum { PC_ACT_NONE = 0, PC_ACT_RELU = 1, PC_ACT_RELU_MASK = 2 };

// q / d with mg = floor(2^32 / d) + 1 from the host (exact while q * d < 2^32); mg == 0 stands for d == 1
__device__ __forceinline__ uint32_t pc_udiv(uint32_t q, uint32_t mg) { return mg ? __umulhi(q, mg) : q; }
inline uint32_t pc_udiv_magic(int d) { return d == 1 ? 0u : (uint32_t)((((uint64_t)1 << 32) / (uint64_t)d) + 1); }

// Pixel tile of about BN output pixels (TI images x TH x TW) and its staged input extent; ext = reach of the taps.
void pc_plan_mfma_tiles(MfmaArgs *g, int BN, int ext);

// The weight operand in the form the structured-sparse matrix instruction takes (PackView::ws_*_val, _idx, _flag of
// the pass's orientation); val == nullptr: the pack has none.
struct SparseOperand {
    const uint16_t *val;
    const uint32_t *idx;
    const uint16_t *flag;
    // the overflow weights as lists of extra reduction columns (PackView::ov_*_cnt, _a, _col)
    const uint32_t *ov_cnt;
    const uint16_t *ov_a;
    const uint32_t *ov_col;
};

// Wave-specialised forward/backward-data kernel for full 3x3 tap lists. pcfg: -1 = take it when the plan says it
// wins, >= 7 = the forced variant. *launched stays false when the launch is left to the cooperative kernel.
pc_status pc_run_mfma_conv_ws(pc_ctx *ctx, int pcfg, const MfmaArgs &g0, int ext, const int *tr, const int *tc,
                              const uint16_t *in, uint16_t *out, const uint16_t *wz, const SparseOperand &sp, bool *launched,
                              int act = PC_ACT_NONE);

// Copies between a tensor with C < 8 channels per pixel and one with 8-channel (16-byte) pixel rows.
void pc_launch_pad_channels(pc_ctx *ctx, const uint16_t *x, void *xp, int64_t npix, int C, int Cp);
void pc_launch_unpad_channels(pc_ctx *ctx, const void *yp, uint16_t *y, int64_t npix, int C);
#endif

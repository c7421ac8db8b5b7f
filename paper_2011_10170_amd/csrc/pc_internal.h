// Internal declarations shared by the translation units of libpatconv (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include "pc.h"

#define PC_MAX_P 126
#define PC_OV_STEPS 4          // steps of 16 overflow columns per (row tile, 64-entry chunk) list
#define PC_OV_SUB 32           // overflow weights a 32 x 32 block's list holds
#define PC_OV_BAD 0xFFFFFFFFu

struct pc_ctx {
    int device;
    hipStream_t stream;
    pc_variant forced;
    int plan_cfg;          // MFMA conv tile configuration override, -1 = automatic
    int plan_split;        // MFMA conv split-K override, 0 = automatic
    int num_cu;
    char err[256];
    // scratch owned by the context (grown on demand, never shrunk)
    void *scratch;
    size_t scratch_bytes;
    void **retired;        // superseded scratch buffers (a growing host array), kept until pc_destroy: enqueued or captured work may still use them
    int n_retired, cap_retired;
    bool fixed_scratch;    // set for the duration of an entry point that must not allocate: pc_scratch then hands out the
                           // device's fixed buffer, or fails when the request exceeds it
    char last_kernel[160]; // symbol of the kernel that did the work of the last conv call (pc_last_kernel)
    int64_t *nnz_pinned;   // pinned host word for reading back a pack's kernel count
};

// Device-side view of a packed layer. All pointers point into one slab.
struct PackView {
    int32_t F, C, P;
    // filter-major table: rows = filters, kernels ordered (pattern id, channel)
    int32_t *fm_rowptr;   // [F+1]   slot range of filter f
    int32_t *fm_grp;      // [F][P+1] first slot of pattern group p in filter f; [P] = row end
    int32_t *fm_rowtot;   // [F]     kept kernels of filter f (pack-time intermediate)
    uint16_t *fm_c;       // [cap]   input channel of the slot
    uint8_t *fm_pid;      // [cap]   pattern id of the slot
    uint16_t *slot_f;     // [cap]   filter of the slot
    float4 *fm_val;       // [cap]   the 4 kept weights, ascending tap index
    int32_t *slot_of;     // [F][C]  slot of kernel (f,c), -1 when pruned
    uint32_t *kinfo;      // [F][C]  (slot << 9) | 9-bit pattern mask, 0xFFFFFFFF when pruned; nullptr when F*C >= 2^23 (the slot would not fit 23 bits)
    // channel-major table for backward-data: rows = channels, kernels ordered (pattern id, filter)
    int32_t *cm_rowptr;   // [C+1]
    int32_t *cm_grp;      // [C][P+1]
    int32_t *cm_rowtot;   // [C]     kept kernels of channel c (pack-time intermediate)
    uint16_t *cm_f;       // [cap]
    int32_t *cm_slot;     // [cap]   filter-major slot of the entry
    float4 *cm_val;       // [cap]
    // MFMA operand tiles (bf16 bit patterns, zero at every pruned position), fragment order
    uint16_t *wz_fwd;     // A operand of the forward pass
    uint16_t *wz_bwd;     // A operand of the backward-data pass
    // The same operands for the structured-sparse matrix instruction (at most 2 nonzeros in every 4 consecutive
    // reduction entries of a row): row tile rt of 32 rows, tap, step ss of 32 reduction entries.
    //   ws_*_val [rt][tap][ss][2][64 lanes][8]: part 0 holds the first two nonzeros of every group of 4, part 1 the
    //            third and fourth (zero almost everywhere: the two parts together are exact for any mask);
    //   ws_*_idx [rt][tap][ss][64 lanes]: the 2-bit positions of the 8 stored values of a lane, part 0 in the low
    //            half of the word, part 1 in the high half;
    //   ws_*_flag [rt][ss]: bit t set when part 1 of tap t has a nonzero (the instruction for it is skipped otherwise)
    uint16_t *ws_fwd_val, *ws_bwd_val;
    uint32_t *ws_fwd_idx, *ws_bwd_idx;
    uint16_t *ws_fwd_flag, *ws_bwd_flag;
    // The part-1 operand leaves out the third and fourth nonzeros of a group ("overflow" weights, well under 1 % of
    // the kept weights at the keep ratios of the workloads). Besides part 2 they are kept as lists, one per row tile
    // of 32 rows and chunk of 64 reduction entries, ready to be multiplied as extra reduction columns of a dense
    // matrix instruction: up to PC_OV_STEPS steps of 16 columns, each column one (tap, reduction entry) pair.
    //   ov_*_cnt [rt][chunk]: steps of the list, PC_OV_BAD when the list does not fit (the kernel then uses part 2)
    //   ov_*_a   [rt][chunk][step][64 lanes][8]: the A operand of a step (one nonzero per column)
    //   ov_*_col [rt][chunk][step][16]: (tap row << 12) | (tap column << 8) | entry inside the chunk
    //   ov_*_sub_cnt / _sub_ent: the lists of the 32 x 32 blocks as the tile builder leaves them (sorted), merged by
    //            pc_pack_ovf_merge_kernel; entry = (tap << 11 | row << 6 | entry inside the block or chunk, bf16 weight)
    uint32_t *ov_fwd_cnt, *ov_bwd_cnt;
    uint16_t *ov_fwd_a, *ov_bwd_a;
    uint32_t *ov_fwd_col, *ov_bwd_col;
    uint32_t *ov_fwd_sub_cnt, *ov_bwd_sub_cnt;
    uint2 *ov_fwd_sub_ent, *ov_bwd_sub_ent;
    int32_t Fp, Cp;       // F and C rounded up to 128 (row extent of the operand tiles)
    int32_t Fk, Ck;       // F and C rounded up to 64, the largest channel chunk a kernel walks (reduction extent of the operand tiles)
};

struct pc_packed {
    int device;
    pc_dtype dtype;
    int variant;                 // PC_VARIANT_VALU or PC_VARIANT_MFMA
    uint16_t lib[PC_MAX_P];
    uint8_t taps[PC_MAX_P][4];   // kept taps of every pattern, ascending
    void *slab;
    size_t slab_bytes;
    PackView v;
    PackView *v_dev;             // copy of v at the start of the slab, for kernels that serve several packs at once
    hipEvent_t packed_evt;       // recorded after the last pack on this handle
    bool evt_recorded;           // false when that pack was enqueued under stream capture (no event then)
    int64_t nnzk;                // -1 until read back
};

// Pattern pool passed to kernels by value.
struct LibArg {
    int32_t P;
    uint16_t mask[PC_MAX_P];
    uint8_t taps[PC_MAX_P][4];
};

// A kernel's dynamic-LDS limit is a function attribute of a device: it is raised on first use per device.
#define PC_MAX_DEVICES 64
struct pc_per_device_once { bool done[PC_MAX_DEVICES]; };
inline bool pc_once_pending(const pc_per_device_once &o, int device) { return device < 0 || device >= PC_MAX_DEVICES || !o.done[device]; }
inline void pc_once_done(pc_per_device_once &o, int device) { if (device >= 0 && device < PC_MAX_DEVICES) o.done[device] = true; }

pc_status pc_fail(pc_ctx *ctx, pc_status s, const char *fmt, ...);
pc_status pc_hip_check(pc_ctx *ctx, hipError_t e, const char *what);
pc_status pc_scratch(pc_ctx *ctx, size_t bytes, void **out);
// Records the symbol of the kernel a conv call launched (printf-style), for pc_last_kernel.
void pc_note_kernel(pc_ctx *ctx, const char *fmt, ...);
void pc_fill_lib(LibArg *la, const uint16_t *lib, int P);

#define PC_HIP(ctx, call)                                              \
    do {                                                               \
        pc_status _s = pc_hip_check((ctx), (call), #call);             \
        if (_s != PC_OK) return _s;                                    \
    } while (0)

// ---- launches implemented in the other translation units ----
pc_status pc_launch_select(pc_ctx *ctx, const float *W, const float *G, int F, int C, const LibArg &la,
                           pc_keep_mode km, int64_t n_keep, pc_score_mode sm, uint8_t *pid, uint8_t *keep);
pc_status pc_launch_pack(pc_ctx *ctx, pc_packed *pk, const float *W, const uint8_t *pid, const uint8_t *keep);
// Several layers per launch (at most PC_BATCH_MAX per kernel; longer lists are cut into groups).
#define PC_BATCH_MAX 32
// Index l of the range [first[l], first[l + 1]) that holds workgroup b, 0 <= l < n (uniform over the workgroup).
__device__ __forceinline__ int pc_batch_find(const int32_t *first, int n, int b)
{
    int l = 0;
    while (l + 1 < n && b >= first[l + 1]) ++l;
    return l;
}
pc_status pc_launch_select_batch(pc_ctx *ctx, int n, const float *const *W, const float *const *G, const int32_t *F,
                                 const int32_t *C, const LibArg &la, pc_keep_mode km, const int64_t *n_keep, pc_score_mode sm,
                                 uint8_t *const *pid, uint8_t *const *keep);
// One layer of a grouped split reduction (partial planes of G splits -> dw in compact order).
#define PC_REDUCE_GROUP_MAX 20
struct WgradReduceItem {
    const float *partial;
    float *dw;
    const int32_t *nnzk_dev;     // the pack's kept-kernel count on the device
    int64_t pstride, exact;      // plane stride in slots; the count when the host knows it, else -1
    int32_t G, tps;
};
pc_status pc_launch_wgrad_reduce_group(pc_ctx *ctx, int n, WgradReduceItem *items, const int64_t *nslots, const pc_packed *const *pk);
pc_status pc_launch_update_values_batch(pc_ctx *ctx, int n, pc_packed *const *pk, const float *const *W);
pc_status pc_launch_pack_batch(pc_ctx *ctx, int n, pc_packed *const *pk, const float *const *W, const uint8_t *const *pid,
                               const uint8_t *const *keep, const LibArg &la);
pc_status pc_launch_update_values(pc_ctx *ctx, pc_packed *pk, const float *W);
pc_status pc_launch_scatter(pc_ctx *ctx, const pc_packed *pk, const float *compact, float *dense, int from_pack);

pc_status pc_valu_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y);
pc_status pc_valu_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx);
pc_status pc_valu_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x,
                             const void *dy, float *dw);

pc_status pc_launch_wgrad_reduce(pc_ctx *ctx, const float *partial, int G, int64_t pstride, int64_t nslots,
                                 const pc_packed *pk, float *dw);

bool pc_mfma_supports(int F, int C);
// act (PC_ACT_* of pc_mfma.h, 0 = none), act_mask, fused: a ReLU step fused into the launch when the kernel that takes
// it can; *fused tells whether it was (fused == nullptr: never).
pc_status pc_mfma_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y, int act = 0,
                      bool *fused = nullptr);
pc_status pc_mfma_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx, int act = 0,
                           const void *act_mask = nullptr, bool *fused = nullptr);
// First-layer kernels (stride 1, at most 4 input channels); *launched stays false when the layer is outside what they take.
pc_status pc_thin_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y, int act, bool *launched);
pc_status pc_thin_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, void *dx, bool *launched);
// In-place ReLU of n elements; and in-place "keep where the matching element of a is positive, else +0".
pc_status pc_launch_relu(pc_ctx *ctx, void *z, int64_t n, pc_dtype dtype);
pc_status pc_launch_relu_mask(pc_ctx *ctx, void *dz, const void *a, int64_t n, pc_dtype dtype);
pc_status pc_mfma_bwd_weight_group(pc_ctx *ctx, int n, const pc_conv_desc *d, const pc_packed *const *pk, const void *const *x,
                                   const void *const *dy, float *const *dw);
pc_status pc_mfma_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x,
                             const void *dy, float *dw);

// ---- small device helpers ----
#ifdef __HIPCC__
__device__ __forceinline__ float pc_bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t pc_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);   // round to nearest, ties to even (finite inputs)
    return (uint16_t)(u >> 16);
}
// two floats -> two bf16 (round to nearest even, v_cvt_pk_bf16_f32), the first in the low half
__device__ __forceinline__ uint32_t pc_pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    const f2 v = {lo, hi};
    const bf2 b = __builtin_convertvector(v, bf2);
    return *reinterpret_cast<const uint32_t *>(&b);
}
template <typename T> __device__ __forceinline__ float pc_load(const T *p);
template <> __device__ __forceinline__ float pc_load<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float pc_load<uint16_t>(const uint16_t *p) { return pc_bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void pc_store(T *p, float v);
template <> __device__ __forceinline__ void pc_store<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void pc_store<uint16_t>(uint16_t *p, float v) { *p = pc_f32_to_bf16(v); }
#endif

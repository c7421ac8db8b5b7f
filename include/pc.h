/*
 * libpatconv -- pattern-sparse 3x3 convolution for training on AMD MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of ClickTrain (arXiv 2011.10170): every kept 3x3
 * kernel retains exactly 4 of its 9 taps, chosen from a small pattern pool, and connectivity
 * pruning removes whole kernels (Section 2, "Fine-grained pattern-based pruning").
 *
 * Conventions for every entry point
 *   - Pointers named *_dev are caller-owned DEVICE memory on the context's GPU (for example a
 *     torch tensor's data_ptr()). The library never frees them and does not keep them after
 *     the stream-ordered work of the call has run. Pointers named *_host are HOST memory and
 *     are copied before the call returns. The calls that serve several layers at once take HOST arrays with one
 *     entry per layer; those named *_dev_host hold device pointers (the array on the host, each entry a device
 *     tensor as in the single-layer call).
 *   - pc_ctx and pc_packed are library-owned handles, released by pc_destroy / pc_packed_free
 *     (both accept NULL).
 *   - Work is enqueued on the context's HIP stream and is asynchronous to the host unless
 *     stated. One context per host thread; calls on one context must not overlap.
 *   - Arguments are validated on the host before anything is launched. Errors are return
 *     codes only; pc_last_error() gives a message for the last failure on that context.
 *   - Kernel tap index t = 3*r + s (kernel row r, column s, spatial offset (r-1, s-1)).
 *     A pattern is a 9-bit mask with bit t set when tap t is kept; exactly 4 bits are set.
 *   - Weights W and their gradient G are float32 [F][C][3][3] (= [F][C][9]).
 *     Activations are NHWC: x, dx [N][H][W][C]; y, dy [N][Ho][Wo][F]; Ho = (H-1)/stride + 1,
 *     Wo likewise (3x3 window, zero padding 1, stride 1 or 2). Their element type is
 *     desc.dtype: float32, or bfloat16 with float32 accumulation.
 *   - Non-finite inputs give unspecified results.
 */
#ifndef PATCONV_PC_H
#define PATCONV_PC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pc_ctx pc_ctx;
typedef struct pc_packed pc_packed;

typedef enum {
    PC_OK = 0,
    PC_ERR_INVALID_ARG = 1,   /* null pointer, negative count, handle/descriptor mismatch */
    PC_ERR_BAD_LIBRARY = 2,   /* P outside 1..126, a mask >= 512, popcount != 4, duplicate masks */
    PC_ERR_BAD_SHAPE = 3,     /* N,H,W,C,F < 1, C or F > 65535, stride not 1 or 2 */
    PC_ERR_UNSUPPORTED = 4,   /* valid request this build has no kernel for */
    PC_ERR_NOMEM = 5,         /* device or host allocation failed */
    PC_ERR_DEVICE = 6         /* a HIP call failed (no GPU, launch failure, ...) */
} pc_status;

typedef enum { PC_F32 = 0, PC_BF16 = 1 } pc_dtype;

/* Which kernels connectivity pruning keeps (Section 4.3 asks for a user-set number of
 * unimportant kernels per layer; Section 5.2 asks that every filter keeps the same number):
 * PER_FILTER keeps the n_keep best kernels of every filter, PER_LAYER the n_keep best of the layer. */
typedef enum { PC_KEEP_PER_FILTER = 0, PC_KEEP_PER_LAYER = 1 } pc_keep_mode;

/* Score that ranks kernels: RETAINED = Eq. 1 evaluated at the chosen pattern (importance that
 * survives the hard prune); KERNEL = Eq. 2 (all 9 taps). */
typedef enum { PC_SCORE_RETAINED = 0, PC_SCORE_KERNEL = 1 } pc_score_mode;

/* Kernel family used by the three conv passes of a packed layer. */
typedef enum {
    PC_VARIANT_AUTO = 0,  /* chosen at pack time from dtype and shape */
    PC_VARIANT_VALU = 1,  /* pattern-grouped gather on the vector ALUs: only kept taps are multiplied */
    PC_VARIANT_MFMA = 2,  /* bf16 only: matrix-core contraction over tap-major zero-filled weight tiles */
    /* bf16 only, never chosen by AUTO: as MFMA, but the forward / backward-data passes of stride-1 layers with at
     * least 64 reduction channels multiply with the structured-sparse matrix instruction (2 nonzeros in 4 reduction
     * entries, twice the reduction length per instruction); the weights that exceed that form go through a second
     * instruction, issued only where needed, so results are exact for any mask and the instruction count falls
     * with the keep ratio. Measured faster than MFMA below a keep ratio of about 0.12 only (the operand delivery,
     * not the matrix pipe, bounds these kernels). The pack holds both operand forms. */
    PC_VARIANT_MFMA_SPARSE = 3
} pc_variant;

typedef struct {
    int32_t N, H, W, C, F;
    int32_t stride;        /* 1 or 2 */
    pc_dtype dtype;        /* element type of x, y, dy, dx */
} pc_conv_desc;

/* ---- context ---------------------------------------------------------------------------- */

/* Creates a context on HIP device `device`. hip_stream is a hipStream_t the caller owns
 * (NULL = the default stream); all later work of this context is enqueued there.
 * Fails with PC_ERR_DEVICE when the device cannot be used.
 * A context owns one device scratch buffer (partial sums of split reductions, channel-padded copies of a
 * first layer's tensors). It grows when a call needs more than any call before: that call allocates a larger
 * buffer with hipMalloc (at least half as large again) and keeps every older one until pc_destroy, however many
 * there are, so work that is already enqueued, or captured in a HIP graph, keeps a valid address (PC_ERR_NOMEM, with
 * the current buffer unchanged, when the device or the host cannot provide the memory). No allocation may happen
 * during a stream capture: run every layer shape once before capturing. Calls on one context must not overlap (one
 * stream, one scratch buffer). */
pc_status pc_create(pc_ctx **out, int device, void *hip_stream);
void pc_destroy(pc_ctx *ctx);
const char *pc_status_str(pc_status s);
const char *pc_last_error(const pc_ctx *ctx);

/* Symbol of the kernel that did the work of the last pc_conv_fwd / pc_conv_bwd_data / pc_conv_bwd_weight (or _relu,
 * _batch) call on this context, with its template arguments as a profiler prints them, e.g.
 * "pc_mfma_conv_ks_kernel<2, 2, 9, 64, 1, 0>" (helper kernels of the same call, such as the reduction of partial
 * sums, are not named). Lets a measurement attribute a call's duration to a line of a kernel trace. Empty before the
 * first such call; the string lives in the context and is overwritten by the next call. */
const char *pc_last_kernel(const pc_ctx *ctx);

/* Forces the kernel family for later pc_pack / pc_conv_* calls on this context (default AUTO).
 * PC_VARIANT_MFMA or PC_VARIANT_MFMA_SPARSE on a layer it cannot serve makes pc_pack return PC_ERR_UNSUPPORTED. A handle
 * that is re-packed keeps the operand forms it was created with. */
pc_status pc_set_variant(pc_ctx *ctx, pc_variant v);

/* Tuning aid for tests and sweeps: forces a kernel of the matrix-core family instead of the automatic
 * choice (tile_cfg = -1) for later calls on this context.
 *   0..6   forward/backward-data: a tile shape of the cooperative kernel
 *   7..9   forward/backward-data: the persistent wave-specialised kernel, reduction split over its MFMA
 *          wavefronts, tiles of 64 output channels x 128, 64, 32 pixels
 *   13, 16 the same kernel with the pixels split over the wavefronts (64 x 512 and 64 x 256 tiles,
 *          32-channel chunks)
 *   14, 15 as 9 with 128-channel chunks, and with tiles of 32 output channels x 32 pixels
 *   17, 18 as 13, 16 with 16-channel chunks (first layers); 19 as 13 with tiles of 32 output channels;
 *          20 as 16 with 64-channel chunks; 21 as 8 with 128-channel chunks
 *   10, 11 backward-weight: the cooperative / the wave-specialised kernel (the other passes stay automatic)
 *   22     forward/backward-data: the structured-sparse kernel (packs made under PC_VARIANT_MFMA_SPARSE only)
 *   23     the first-layer kernels (stride 1, at most 4 input channels): the automatic choice takes them wherever
 *          they apply; any other code here keeps such a layer on the general kernels
 * The wave-specialised forward/backward-data kernel takes 9-tap launches only: a stride-2 backward-data pass
 * (one launch of the cooperative kernel over the four parity classes of input pixels) takes 0..6 and uses the
 * automatic choice otherwise. split_k > 0 forces that many splits of the reduction in the
 * cooperative forward/backward-data kernel (0 = automatic). A configuration that does not fit a layer makes
 * the conv call return PC_ERR_UNSUPPORTED. Results do not depend on the choice beyond float32 summation
 * order. Returns PC_ERR_INVALID_ARG for values outside these ranges. */
pc_status pc_set_plan_override(pc_ctx *ctx, int32_t tile_cfg, int32_t split_k);

/* Host-only argument checks (usable without a GPU). */
pc_status pc_check_library(const uint16_t *lib_host, int32_t P);
pc_status pc_check_conv_desc(const pc_conv_desc *desc);

/* ---- pattern and kernel selection (Section 4.1, Eq. 1 and Eq. 2) ------------------------- */

/* For every kernel (f,c): tap importance s_t = (g_t*w_t)^2 (G_dev == NULL: s_t = w_t^2, the
 * magnitude criterion); pattern importance I_p = sum of s_t over the 4 taps of pattern p;
 * pid[f][c] = the pool index with the largest I_p (lowest index on ties), written for every
 * kernel. keep[f][c] = 1 for the n_keep kernels with the largest ranking score of their filter
 * (PER_FILTER, 0 <= n_keep <= C) or of the layer (PER_LAYER, 0 <= n_keep <= F*C), equal scores
 * ordered by lower index; else 0.
 * Arithmetic is float32 in a fixed order without fused multiply-add, so results are
 * reproducible bit for bit: s_t = (g*w)*(g*w); I_p = ((s_a+s_b)+s_c)+s_d for taps a<b<c<d;
 * Eq. 2 adds s_0..s_8 left to right.
 *   W_dev, G_dev : float32 [F][C][9] device (G_dev may be NULL)
 *   lib_host     : uint16 [P] host, the pattern pool
 *   pid_dev, keep_dev : uint8 [F][C] device, outputs */
pc_status pc_pattern_select(pc_ctx *ctx, const float *W_dev, const float *G_dev,
                            int32_t F, int32_t C, const uint16_t *lib_host, int32_t P,
                            pc_keep_mode keep_mode, int64_t n_keep, pc_score_mode score_mode,
                            uint8_t *pid_dev, uint8_t *keep_dev);

/* ---- packing (Section 5.1: fixed index arrays generated once, values gathered from the
 *      dense weight tensor; the hard prune W (.) M of Section 6) -------------------------- */

/* Builds the compact layout of one layer from its dense weights and the selection result:
 * a filter-major table of the kept kernels (per filter ordered by pattern id, then channel,
 * with per-pattern group offsets), a channel-major table for the backward-data pass, the
 * 4 kept weights of every kept kernel (rounded to bf16, nearest-even, when compute_dtype is
 * PC_BF16), and for the MFMA variant tap-major zero-filled bf16 weight tiles.
 * Compact slot order (used by dw_compact and pc_scatter_dense): filters ascending; inside a
 * filter by pattern id, then by channel; the 4 entries of a slot are the kept taps in
 * ascending tap index.
 * *out == NULL: a new handle is allocated (device memory sized for F*C kernels).
 * *out != NULL: that handle is re-packed in place; it must have the same F, C and dtype.
 * pid/keep values are trusted to be < P and 0/1. F*C must stay below 2^31 (32-bit slots: PC_ERR_UNSUPPORTED).
 * A pack is bound to its device, not to the context that made it: any context of that device may pass it to
 * the conv calls, on its own stream (for example pc_conv_bwd_weight on a second context and stream beside
 * pc_conv_bwd_data on the first). The caller orders the streams: the pack or value update must have run before
 * another stream's call reads it, and every reader must have finished before the handle is re-packed or freed. */
pc_status pc_pack(pc_ctx *ctx, const float *W_dev, const uint8_t *pid_dev, const uint8_t *keep_dev,
                  int32_t F, int32_t C, const uint16_t *lib_host, int32_t P,
                  pc_dtype compute_dtype, pc_packed **out);

/* pc_pattern_select for several layers at once (the per-batch selection of Section 4.3 runs over every layer of the
 * network): the same results as n_layers single calls, from one launch per 32 layers where every row has at most
 * 8192 kernels and keep_mode is PC_KEEP_PER_FILTER (other layers are served one by one inside the call).
 * One pool, keep mode and score mode for all layers.
 *   W_dev_host, G_dev_host, pid_dev_host, keep_dev_host : HOST arrays [n_layers] of device pointers with the
 *       meaning they have in pc_pattern_select (G_dev_host may be NULL, and so may any of its entries)
 *   F_host, C_host, n_keep_host : HOST arrays [n_layers]
 * The arrays are read before the call returns. */
pc_status pc_pattern_select_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W_dev_host,
                                  const float *const *G_dev_host, const int32_t *F_host, const int32_t *C_host,
                                  const uint16_t *lib_host, int32_t P, pc_keep_mode keep_mode,
                                  const int64_t *n_keep_host, pc_score_mode score_mode,
                                  uint8_t *const *pid_dev_host, uint8_t *const *keep_dev_host);

/* Re-packs several existing handles (each made by pc_pack for its layer's F, C and dtype; all distinct) with one
 * pool: the same tables and tiles as n_layers pc_pack calls, from two or three launches per 32 layers. Every
 * handle keeps the kernel family it has.
 *   W_dev_host, pid_dev_host, keep_dev_host : HOST arrays [n_layers] of device pointers as in pc_pack
 *   packs_host : HOST array [n_layers] of handles */
pc_status pc_pack_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W_dev_host,
                        const uint8_t *const *pid_dev_host, const uint8_t *const *keep_dev_host,
                        const uint16_t *lib_host, int32_t P, pc_packed *const *packs_host);

/* Re-gathers the kept weights from a dense tensor with unchanged tables (the per-iteration
 * dense-to-sparse conversion of Section 5.1). */
pc_status pc_update_values(pc_ctx *ctx, pc_packed *pk, const float *W_dev);

/* pc_update_values for several handles (all distinct) at once: one launch per 32 matrix-core packs that were made
 * with the same pool; other packs are updated one by one inside the call.
 *   packs_host : HOST array [n_layers] of handles; W_dev_host : HOST array [n_layers] of device pointers */
pc_status pc_update_values_batch(pc_ctx *ctx, int32_t n_layers, pc_packed *const *packs_host,
                                 const float *const *W_dev_host);

/* nnz_kernels = number of kept kernels; variant = family in use. The count is read back from the device the
 * first time it is asked for after a pack: that call waits for the pack to finish (for a pack that was
 * enqueued while its stream was being captured into a HIP graph it waits for the whole stream of ctx, and it
 * must not be made during the capture). No other call needs the count on the host: a step of
 * pc_pattern_select, pc_pack and the three passes enqueues without any read-back and can be captured. */
pc_status pc_packed_info(pc_ctx *ctx, const pc_packed *pk, int64_t *nnz_kernels, int32_t *variant);
void pc_packed_free(pc_packed *pk);

/* Expands a compact [nnz_kernels][4] float32 array to dense [F][C][9] float32 with zeros at
 * every pruned position. */
pc_status pc_scatter_dense(pc_ctx *ctx, const pc_packed *pk, const float *compact_dev, float *dense_dev);

/* Writes the hard-pruned weights W (.) M as dense [F][C][9] float32 (values as stored in the
 * pack, i.e. bf16-rounded for a bf16 pack). */
pc_status pc_unpack_dense(pc_ctx *ctx, const pc_packed *pk, float *dense_dev);

/* ---- the three passes (Section 5.2, forward and backward phase) -------------------------- */

/* y[n,oy,ox,f] = sum over kept (c,t) of filter f of x[n, oy*stride+r-1, ox*stride+s-1, c] * w[f,c,t]
 * (zero padding, no bias). */
pc_status pc_conv_fwd(pc_ctx *ctx, const pc_conv_desc *desc, const pc_packed *pk,
                      const void *x_dev, void *y_dev);

/* dx = dy (*) rot180(W): dx[n,iy,ix,c] = sum over kept (f,t) of channel c with
 * (iy+1-r) and (ix+1-s) divisible by stride and in range of
 * dy[n,(iy+1-r)/stride,(ix+1-s)/stride,f] * w[f,c,t]. The activation derivative is not applied. */
pc_status pc_conv_bwd_data(pc_ctx *ctx, const pc_conv_desc *desc, const pc_packed *pk,
                           const void *dy_dev, void *dx_dev);

/* pc_conv_fwd followed by the activation of Section 5.2 (a = sigma(z), sigma = ReLU) in the same launch where the
 * kernel that serves the layer can, else in a second one: a = relu(conv(x)), bit-identical to pc_conv_fwd
 * followed by pc_act_pool_fwd with pool = 1. No selection bytes are written: the backward pass reads the
 * derivative from a itself (pc_conv_bwd_data_relu of the next layer). */
pc_status pc_conv_fwd_relu(pc_ctx *ctx, const pc_conv_desc *desc, const pc_packed *pk,
                           const void *x_dev, void *a_dev);

/* pc_conv_bwd_data followed by the factor sigma'(z) of Section 5.2 for the layer BEFORE this one, whose ReLU output
 * is this layer's input x: dx = (dy (*) rot180(W)) where x > 0, else +0 (x > 0 exactly where that layer's z > 0).
 * Same launch where the kernel can, else a second one; bit-identical to pc_conv_bwd_data followed by that mask.
 *   x_dev : dtype [N][H][W][C], the tensor this layer's forward pass read */
pc_status pc_conv_bwd_data_relu(pc_ctx *ctx, const pc_conv_desc *desc, const pc_packed *pk,
                                const void *dy_dev, const void *x_dev, void *dx_dev);

/* Weight gradient at kept taps only, float32 [nnz_kernels][4] in compact slot order:
 * dw[f,c,t] = sum_{n,oy,ox} dy[n,oy,ox,f] * x[n, oy*stride+r-1, ox*stride+s-1, c].
 * Deterministic: no floating-point atomics (per-split partial sums in the context's scratch buffer, added in a
 * fixed order). The call never reads the kept-kernel count back: until pc_packed_info has been asked for it
 * after the last pack, the partial sums are laid out for F*C slots (16 bytes x splits x F*C of scratch, touched
 * only at kept slots). dw_compact_dev must hold nnz_kernels x 4 floats. */
pc_status pc_conv_bwd_weight(pc_ctx *ctx, const pc_conv_desc *desc, const pc_packed *pk,
                             const void *x_dev, const void *dy_dev, float *dw_compact_dev);

/* pc_conv_bwd_weight for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc. Same arguments, same kernels and the same result, bit for bit, as
 * pc_conv_bwd_weight with the same pack state; but the partial sums (and the channel-padded copy of a first layer's
 * x) live in a fixed buffer of 32 MiB that the library's code object holds on every GPU it is loaded on until the
 * process ends, and the call makes no hipMalloc / hipFree and grows no context buffer. A layer that needs more
 * (the partial sums take at most 16 MiB; a first layer with C not a multiple of 8 adds N*H*W*16 bytes) is rejected
 * with PC_ERR_UNSUPPORTED before anything is launched. All contexts of a GPU share that one buffer and it keeps the
 * last call's contents (nothing in it needs to start at zero): calls that overlap on one GPU, from different
 * contexts or streams, race; the caller serialises them. */
pc_status pc_conv_bwd_weight_noalloc(pc_ctx *ctx, const pc_conv_desc *desc, const pc_packed *pk,
                                     const void *x_dev, const void *dy_dev, float *dw_compact_dev);

/* pc_conv_bwd_weight for several layers at once. The weight gradients of a network's layers do not depend on each
 * other (dE/dW of a layer needs only its own a_prev and delta, Section 5.2), so once every x and dy exists they can
 * all be computed together: the matrix-core layers in one launch per 20 layers plus one reduction launch (the
 * layers share the chip, so each is split less than in its own call: deterministic, equal to the single call up
 * to the float32 order of additions); layers on the gather kernels one by one. Every layer's partial sums have their own region of the context's scratch buffer.
 *   descs_host : HOST array [n_layers] of descriptors; packs_host : HOST array [n_layers] of handles
 *   x_dev_host, dy_dev_host, dw_compact_dev_host : HOST arrays [n_layers] of device pointers as in
 *       pc_conv_bwd_weight (the dw buffers all distinct) */
pc_status pc_conv_bwd_weight_batch(pc_ctx *ctx, int32_t n_layers, const pc_conv_desc *descs_host,
                                   const pc_packed *const *packs_host, const void *const *x_dev_host,
                                   const void *const *dy_dev_host, float *const *dw_compact_dev_host);

/* ---- training-side steps around the path: pattern pool generation (Section 4.2), adaptive
 *      finalisation (Section 4.3), modified group lasso (Section 4.4, Eq. 3 and Eq. 4) ---------- */

/* Steps 1-4 of the pool generation for every kernel (f,c), from the tap importances s_t of
 * pc_pattern_select: (1) the position with the highest importance; (2) the best of its horizontal, vertical
 * and diagonal neighbours; (3) candidate positions = horizontal and vertical neighbours of those two;
 * (4) the pair of candidates that gives the four-tap pattern with the highest importance
 * ((s_a+s_b)+s_c)+s_d, taps ascending. Every arg max takes the first maximum (positions ascending, pairs in
 * lexicographic order). The kernel's candidate pattern adds 1 to its competitive score:
 *   hist_dev  : uint32 [512] device, indexed by the 9-bit mask; accumulated, the caller zeroes it before the
 *               first call (step 5 repeats the call over the epochs)
 *   masks_dev : uint16 [F][C] device or NULL; the candidate pattern of every kernel
 * Float32 in the fixed order above, integer counting: bit-reproducible. */
pc_status pc_dppg_accumulate(pc_ctx *ctx, const float *W_dev, const float *G_dev, int32_t F, int32_t C,
                             uint32_t *hist_dev, uint16_t *masks_dev);

/* Step 6: the n_patterns candidate patterns with the highest competitive scores, equal scores ordered by the
 * lower mask; patterns never produced are not returned. Waits for the stream of ctx.
 *   lib_host   : uint16 [n_patterns] host, output (the first *n_found entries are written)
 *   score_host : uint32 [n_patterns] host or NULL, their scores */
pc_status pc_dppg_pool(pc_ctx *ctx, const uint32_t *hist_dev, int32_t n_patterns, uint16_t *lib_host,
                       uint32_t *score_host, int32_t *n_found);

/* One batch of the adaptive finalisation: counts_dev[f][c][pid_dev[f][c]] += 1 with pid_dev from
 * pc_pattern_select (the caller skips batches its loss margin rules out).
 *   counts_dev : uint32 [F][C][P] device, accumulated; the caller zeroes it first */
pc_status pc_finalize_count(pc_ctx *ctx, const uint8_t *pid_dev, int32_t F, int32_t C, int32_t P,
                            uint32_t *counts_dev);

/* The final pattern of every kernel: the most frequent of its per-batch best patterns (lowest id on ties).
 *   pid_dev : uint8 [F][C] device, output */
pc_status pc_finalize_pick(pc_ctx *ctx, const uint32_t *counts_dev, int32_t F, int32_t C, int32_t P,
                           uint8_t *pid_dev);

/* Gradient of the modified group-lasso penalty, added to a dense weight gradient. With one group per kernel,
 * Z = the weights outside the kernel's pattern, U = all 9 weights of a kernel with keep = 0 (else 0):
 *   dW[f][c][t] += lambda_p * Z_t / ||Z||_2 + lambda_i * U_t / ||U||_2     (a term whose norm is 0 adds 0)
 *   *penalty_dev = lambda_p * sum ||Z|| + lambda_i * sum ||U|| over the layer (float64, NULL: not computed;
 *                  summed in a fixed order)
 * Float32 per kernel (squares added in ascending tap order, correctly rounded square root and division).
 *   W_dev : float32 [F][C][9]; pid_dev, keep_dev : uint8 [F][C]; dW_dev : float32 [F][C][9], accumulated */
pc_status pc_group_lasso_grad(pc_ctx *ctx, const float *W_dev, const uint8_t *pid_dev, const uint8_t *keep_dev,
                              int32_t F, int32_t C, const uint16_t *lib_host, int32_t P,
                              float lambda_p, float lambda_i, float *dW_dev, double *penalty_dev);

/* The four calls above for the layers of a network at once (one launch per 32 layers; the same results as the single
 * calls layer by layer). Arrays named *_host are HOST arrays [n_layers], of device pointers where the single call
 * takes a device pointer; they are read before the call returns. G_dev_host and masks_dev_host may be NULL, and so
 * may their entries. hist_dev is the one pool all layers count into. penalty_dev receives the penalty of all layers
 * together (NULL: not computed; with a penalty at most 32 layers per call, else PC_ERR_UNSUPPORTED). */
pc_status pc_dppg_accumulate_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W_dev_host,
                                   const float *const *G_dev_host, const int32_t *F_host, const int32_t *C_host,
                                   uint32_t *hist_dev, uint16_t *const *masks_dev_host);
pc_status pc_finalize_count_batch(pc_ctx *ctx, int32_t n_layers, const uint8_t *const *pid_dev_host,
                                  const int32_t *F_host, const int32_t *C_host, int32_t P,
                                  uint32_t *const *counts_dev_host);
pc_status pc_finalize_pick_batch(pc_ctx *ctx, int32_t n_layers, const uint32_t *const *counts_dev_host,
                                 const int32_t *F_host, const int32_t *C_host, int32_t P,
                                 uint8_t *const *pid_dev_host);
pc_status pc_group_lasso_grad_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W_dev_host,
                                    const uint8_t *const *pid_dev_host, const uint8_t *const *keep_dev_host,
                                    const int32_t *F_host, const int32_t *C_host, const uint16_t *lib_host, int32_t P,
                                    float lambda_p, float lambda_i, float *const *dW_dev_host, double *penalty_dev);

/* ---- between two chained layers --------------------------------------------------------- */

/* The step from one layer's output z to the next layer's input a (Section 5.2, "Backward Phase Acceleration":
 * a = sigma(z)), for the networks of Section 6: sigma = ReLU, then a max pooling of pool x pool windows with
 * stride pool (pool = 1: none, 2: the VGG pooling). Exact in both dtypes (comparisons and copies only).
 *   z_dev   : dtype [N][H][W][C] device
 *   a_dev   : dtype [N][H/pool][W/pool][C] device, output (an odd last row / column of z is dropped);
 *             relu(z) = z where z > 0, else +0
 *   sel_dev : uint8, shape of a, output: what pc_act_pool_bwd needs. The window position 2*dr + dc of the
 *             maximum (the first in row-major order among equal maxima), 255 where the maximum is not positive
 * 16-byte accesses when C is a multiple of 8 (bfloat16) / 4 (float32), z_dev and a_dev are 16-byte aligned and
 * sel_dev is 8-byte aligned; one element per thread otherwise. PC_ERR_BAD_SHAPE when H or W < pool. */
pc_status pc_act_pool_fwd(pc_ctx *ctx, const void *z_dev, int32_t N, int32_t H, int32_t W, int32_t C,
                          pc_dtype dtype, int32_t pool, void *a_dev, uint8_t *sel_dev);

/* The backward pass of pc_act_pool_fwd (the error times sigma'(z) of Section 5.2, through the pooling): the
 * error of a pooled element goes to the window position sel names, every other element of dz is 0 (also an odd
 * last row / column). N, H, W, C are those of z.
 *   da_dev : dtype [N][H/pool][W/pool][C] device; sel_dev : as written by the forward call
 *   dz_dev : dtype [N][H][W][C] device, output (every element written) */
pc_status pc_act_pool_bwd(pc_ctx *ctx, const void *da_dev, const uint8_t *sel_dev, int32_t N, int32_t H, int32_t W,
                          int32_t C, pc_dtype dtype, int32_t pool, void *dz_dev);

#ifdef __cplusplus
}
#endif
#endif /* PATCONV_PC_H */

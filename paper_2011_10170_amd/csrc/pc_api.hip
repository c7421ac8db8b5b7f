// Host side of libpatconv: argument validation, handles, dispatch. No kernels here.
#include <stdarg.h>
#include <stdlib.h>

#include <new>

#include "pc_internal.h"
#include "pc_mfma.h"

#include <vector>

// ------------------------------------------------------------------ errors
pc_status pc_fail(pc_ctx *ctx, pc_status s, const char *fmt, ...)
{
    if (ctx) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

pc_status pc_hip_check(pc_ctx *ctx, hipError_t e, const char *what)
{
    if (e == hipSuccess) return PC_OK;
    pc_status s = (e == hipErrorOutOfMemory) ? PC_ERR_NOMEM : PC_ERR_DEVICE;
    return pc_fail(ctx, s, "%s: %s", what, hipGetErrorString(e));
}

extern "C" const char *pc_status_str(pc_status s)
{
    switch (s) {
    case PC_OK: return "ok";
    case PC_ERR_INVALID_ARG: return "invalid argument";
    case PC_ERR_BAD_LIBRARY: return "bad pattern library";
    case PC_ERR_BAD_SHAPE: return "bad shape";
    case PC_ERR_UNSUPPORTED: return "unsupported";
    case PC_ERR_NOMEM: return "out of memory";
    case PC_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

extern "C" const char *pc_last_error(const pc_ctx *ctx) { return ctx ? ctx->err : "no context"; }

void pc_note_kernel(pc_ctx *ctx, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->last_kernel, sizeof(ctx->last_kernel), fmt, ap);
    va_end(ap);
}

extern "C" const char *pc_last_kernel(const pc_ctx *ctx) { return ctx ? ctx->last_kernel : ""; }

// ------------------------------------------------------------------ host-only checks
extern "C" pc_status pc_check_library(const uint16_t *lib, int32_t P)
{
    if (!lib) return PC_ERR_INVALID_ARG;
    if (P < 1 || P > PC_MAX_P) return PC_ERR_BAD_LIBRARY;
    for (int i = 0; i < P; ++i) {
        if (lib[i] >= 512 || __builtin_popcount(lib[i]) != 4) return PC_ERR_BAD_LIBRARY;
        for (int j = 0; j < i; ++j)
            if (lib[j] == lib[i]) return PC_ERR_BAD_LIBRARY;
    }
    return PC_OK;
}

extern "C" pc_status pc_check_conv_desc(const pc_conv_desc *d)
{
    if (!d) return PC_ERR_INVALID_ARG;
    if (d->N < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->F < 1) return PC_ERR_BAD_SHAPE;
    if (d->C > 65535 || d->F > 65535) return PC_ERR_BAD_SHAPE;
    if (d->stride != 1 && d->stride != 2) return PC_ERR_BAD_SHAPE;
    if (d->dtype != PC_F32 && d->dtype != PC_BF16) return PC_ERR_INVALID_ARG;
    // flat element indices are computed in 64 bits; per-image extents must fit 32 bits
    if ((int64_t)d->H * d->W * d->C >= (1ll << 31) || (int64_t)d->H * d->W * d->F >= (1ll << 31))
        return PC_ERR_BAD_SHAPE;
    return PC_OK;
}

void pc_fill_lib(LibArg *la, const uint16_t *lib, int P)
{
    memset(la, 0, sizeof(*la));
    la->P = P;
    for (int i = 0; i < P; ++i) {
        la->mask[i] = lib[i];
        int j = 0;
        for (int t = 0; t < 9; ++t)
            if (lib[i] & (1u << t)) la->taps[i][j++] = (uint8_t)t;
    }
}

// ------------------------------------------------------------------ fixed scratch buffer
// Device memory for the entry point that must not allocate (pc_conv_bwd_weight_noalloc): a file-scope array, so it
// exists on every GPU the library's code is loaded on, from then until the process ends. In host code the array's
// name is only a handle for hipGetSymbolAddress; the address kernels and copies use is looked up once per device,
// with that device current, and kept here.
#define PC_FIXED_SCRATCH_BYTES (32u << 20)
static __device__ __align__(256) unsigned char pc_fixed_scratch_mem[PC_FIXED_SCRATCH_BYTES];
static void *g_fixed_scratch[PC_MAX_DEVICES];

// The calling thread's current device must be `device`.
static hipError_t pc_fixed_scratch_lookup(int device)
{
    if (device < 0 || device >= PC_MAX_DEVICES || g_fixed_scratch[device]) return hipSuccess;
    void *p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(pc_fixed_scratch_mem));
    if (e == hipSuccess) g_fixed_scratch[device] = p;
    return e;
}

// ------------------------------------------------------------------ context
extern "C" pc_status pc_create(pc_ctx **out, int device, void *hip_stream)
{
    if (!out) return PC_ERR_INVALID_ARG;
    *out = nullptr;
    int n = 0;
    if (hipGetDeviceCount(&n) != hipSuccess || device < 0 || device >= n) return PC_ERR_DEVICE;
    if (hipSetDevice(device) != hipSuccess) return PC_ERR_DEVICE;
    if (pc_fixed_scratch_lookup(device) != hipSuccess) return PC_ERR_DEVICE;
    pc_ctx *ctx = new (std::nothrow) pc_ctx();
    if (!ctx) return PC_ERR_NOMEM;
    memset(ctx, 0, sizeof(*ctx));
    ctx->device = device;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->forced = PC_VARIANT_AUTO;
    ctx->plan_cfg = -1;
    ctx->plan_split = 0;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) { delete ctx; return PC_ERR_DEVICE; }
    ctx->num_cu = prop.multiProcessorCount;
    if (hipHostMalloc((void **)&ctx->nnz_pinned, sizeof(int64_t), hipHostMallocDefault) != hipSuccess) {
        delete ctx;
        return PC_ERR_NOMEM;
    }
    *out = ctx;
    return PC_OK;
}

extern "C" void pc_destroy(pc_ctx *ctx)
{
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->scratch) (void)hipFree(ctx->scratch);
    for (int i = 0; i < ctx->n_retired; ++i) (void)hipFree(ctx->retired[i]);
    free(ctx->retired);
    if (ctx->nnz_pinned) (void)hipHostFree(ctx->nnz_pinned);
    delete ctx;
}

extern "C" pc_status pc_set_variant(pc_ctx *ctx, pc_variant v)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (v != PC_VARIANT_AUTO && v != PC_VARIANT_VALU && v != PC_VARIANT_MFMA && v != PC_VARIANT_MFMA_SPARSE)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_set_variant: unknown variant %d", (int)v);
    ctx->forced = v;
    return PC_OK;
}

extern "C" pc_status pc_set_plan_override(pc_ctx *ctx, int32_t tile_cfg, int32_t split_k)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (tile_cfg < -1 || tile_cfg > 23 || tile_cfg == 12 || split_k < 0 || split_k > 64)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_set_plan_override: tile_cfg %d split_k %d out of range", tile_cfg, split_k);
    ctx->plan_cfg = tile_cfg;
    ctx->plan_split = split_k;
    return PC_OK;
}

pc_status pc_scratch(pc_ctx *ctx, size_t bytes, void **out)
{
    if (ctx->fixed_scratch) {
        void *p = ctx->device < PC_MAX_DEVICES ? g_fixed_scratch[ctx->device] : nullptr;
        if (!p) return pc_fail(ctx, PC_ERR_UNSUPPORTED, "no fixed scratch buffer on device %d", ctx->device);
        if (bytes > PC_FIXED_SCRATCH_BYTES)
            return pc_fail(ctx, PC_ERR_UNSUPPORTED, "this layer needs %zu bytes of scratch, the fixed buffer holds %u", bytes,
                           (unsigned)PC_FIXED_SCRATCH_BYTES);
        *out = p;
        return PC_OK;
    }
    if (bytes > ctx->scratch_bytes) {
        // Work that is enqueued, or captured in a HIP graph, keeps the address it was given: the old buffer is never
        // freed before pc_destroy. The list of old buffers grows on the host (the buffer grows by at least half each
        // time, so the list stays short); when it cannot grow, the call fails and the current buffer stays.
        if (ctx->scratch && ctx->n_retired == ctx->cap_retired) {
            const int cap = ctx->cap_retired ? 2 * ctx->cap_retired : 16;
            void **grown = (void **)realloc(ctx->retired, sizeof(void *) * (size_t)cap);
            if (!grown) return pc_fail(ctx, PC_ERR_NOMEM, "scratch: host allocation failed");
            ctx->retired = grown;
            ctx->cap_retired = cap;
        }
        size_t want = bytes + bytes / 2 + (1u << 20);
        void *fresh = nullptr;
        PC_HIP(ctx, hipMalloc(&fresh, want));
        if (ctx->scratch) ctx->retired[ctx->n_retired++] = ctx->scratch;
        ctx->scratch = fresh;
        ctx->scratch_bytes = want;
    }
    *out = ctx->scratch;
    return PC_OK;
}

// ------------------------------------------------------------------ select
extern "C" pc_status pc_pattern_select(pc_ctx *ctx, const float *W, const float *G, int32_t F, int32_t C,
                                       const uint16_t *lib, int32_t P, pc_keep_mode km, int64_t n_keep,
                                       pc_score_mode sm, uint8_t *pid, uint8_t *keep)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!W || !pid || !keep || !lib) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select: null pointer");
    if (F < 1 || C < 1 || F > 65535 || C > 65535)
        return pc_fail(ctx, PC_ERR_BAD_SHAPE, "pc_pattern_select: F=%d C=%d out of range", F, C);
    pc_status s = pc_check_library(lib, P);
    if (s != PC_OK) return pc_fail(ctx, s, "pc_pattern_select: bad library (P=%d)", P);
    if (km != PC_KEEP_PER_FILTER && km != PC_KEEP_PER_LAYER)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select: keep_mode %d", (int)km);
    if (sm != PC_SCORE_RETAINED && sm != PC_SCORE_KERNEL)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select: score_mode %d", (int)sm);
    int64_t lim = (km == PC_KEEP_PER_FILTER) ? (int64_t)C : (int64_t)F * C;
    if (n_keep < 0 || n_keep > lim)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select: n_keep %lld outside 0..%lld",
                       (long long)n_keep, (long long)lim);
    PC_HIP(ctx, hipSetDevice(ctx->device));
    LibArg la;
    pc_fill_lib(&la, lib, P);
    return pc_launch_select(ctx, W, G, F, C, la, km, n_keep, sm, pid, keep);
}

extern "C" pc_status pc_pattern_select_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W, const float *const *G,
                                             const int32_t *F, const int32_t *C, const uint16_t *lib, int32_t P,
                                             pc_keep_mode km, const int64_t *n_keep, pc_score_mode sm, uint8_t *const *pid,
                                             uint8_t *const *keep)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!W || !F || !C || !n_keep || !pid || !keep || !lib)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select_batch: null pointer");
    pc_status s = pc_check_library(lib, P);
    if (s != PC_OK) return pc_fail(ctx, s, "pc_pattern_select_batch: bad library (P=%d)", P);
    if (km != PC_KEEP_PER_FILTER && km != PC_KEEP_PER_LAYER)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select_batch: keep_mode %d", (int)km);
    if (sm != PC_SCORE_RETAINED && sm != PC_SCORE_KERNEL)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select_batch: score_mode %d", (int)sm);
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l] || !pid[l] || !keep[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select_batch: null pointer in layer %d", l);
        if (F[l] < 1 || C[l] < 1 || F[l] > 65535 || C[l] > 65535)
            return pc_fail(ctx, PC_ERR_BAD_SHAPE, "pc_pattern_select_batch: layer %d: F=%d C=%d out of range", l, F[l], C[l]);
        const int64_t lim = (km == PC_KEEP_PER_FILTER) ? (int64_t)C[l] : (int64_t)F[l] * C[l];
        if (n_keep[l] < 0 || n_keep[l] > lim)
            return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pattern_select_batch: layer %d: n_keep %lld outside 0..%lld", l,
                           (long long)n_keep[l], (long long)lim);
    }
    PC_HIP(ctx, hipSetDevice(ctx->device));
    LibArg la;
    pc_fill_lib(&la, lib, P);
    return pc_launch_select_batch(ctx, n_layers, W, G, F, C, la, km, n_keep, sm, pid, keep);
}

// ------------------------------------------------------------------ pack
static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Carves the slab. With base == nullptr only the size is computed.
static size_t carve(PackView *v, PackView **v_dev, char *base, int F, int C, bool mfma, bool sparse)
{
    size_t off = 0;
    size_t cap = (size_t)F * C;
    auto take = [&](size_t bytes) {
        char *p = base ? base + off : nullptr;
        off = align_up(off + bytes, 256);
        return p;
    };
    v->F = F;
    v->C = C;
    v->Fp = (F + 127) / 128 * 128;
    v->Cp = (C + 127) / 128 * 128;
    v->Fk = (F + 63) / 64 * 64;
    v->Ck = (C + 63) / 64 * 64;
    *v_dev = (PackView *)take(sizeof(PackView));
    v->fm_rowptr = (int32_t *)take(sizeof(int32_t) * (F + 1));
    v->fm_grp = (int32_t *)take(sizeof(int32_t) * (size_t)F * (PC_MAX_P + 1));
    v->fm_rowtot = (int32_t *)take(sizeof(int32_t) * F);
    v->fm_c = (uint16_t *)take(sizeof(uint16_t) * cap);
    v->fm_pid = (uint8_t *)take(cap);
    v->slot_f = (uint16_t *)take(sizeof(uint16_t) * cap);
    v->fm_val = (float4 *)take(sizeof(float4) * cap);
    v->slot_of = (int32_t *)take(sizeof(int32_t) * cap);
    v->kinfo = cap < ((size_t)1 << 23) ? (uint32_t *)take(sizeof(uint32_t) * cap) : nullptr;   // only the matrix-core kernels read it
    v->cm_rowptr = (int32_t *)take(sizeof(int32_t) * (C + 1));
    v->cm_grp = (int32_t *)take(sizeof(int32_t) * (size_t)C * (PC_MAX_P + 1));
    v->cm_rowtot = (int32_t *)take(sizeof(int32_t) * C);
    v->cm_f = (uint16_t *)take(sizeof(uint16_t) * cap);
    v->cm_slot = (int32_t *)take(sizeof(int32_t) * cap);
    v->cm_val = (float4 *)take(sizeof(float4) * cap);
    if (mfma) {
        v->wz_fwd = (uint16_t *)take(sizeof(uint16_t) * 9 * (size_t)v->Fp * v->Ck);
        v->wz_bwd = (uint16_t *)take(sizeof(uint16_t) * 9 * (size_t)v->Cp * v->Fk);
    } else {
        v->wz_fwd = v->wz_bwd = nullptr;
    }
    if (mfma && sparse) {
        v->ws_fwd_val = (uint16_t *)take(sizeof(uint16_t) * 9 * (size_t)v->Fp * v->Ck);
        v->ws_bwd_val = (uint16_t *)take(sizeof(uint16_t) * 9 * (size_t)v->Cp * v->Fk);
        v->ws_fwd_idx = (uint32_t *)take(sizeof(uint32_t) * 64 * 9 * (size_t)(v->Fp / 32) * (v->Ck / 32));
        v->ws_bwd_idx = (uint32_t *)take(sizeof(uint32_t) * 64 * 9 * (size_t)(v->Cp / 32) * (v->Fk / 32));
        v->ws_fwd_flag = (uint16_t *)take(sizeof(uint16_t) * (size_t)(v->Fp / 32) * (v->Ck / 32));
        v->ws_bwd_flag = (uint16_t *)take(sizeof(uint16_t) * (size_t)(v->Cp / 32) * (v->Fk / 32));
        const size_t lf = (size_t)(v->Fp / 32) * (v->Ck / 64), lb = (size_t)(v->Cp / 32) * (v->Fk / 64);
        v->ov_fwd_cnt = (uint32_t *)take(sizeof(uint32_t) * lf);
        v->ov_bwd_cnt = (uint32_t *)take(sizeof(uint32_t) * lb);
        v->ov_fwd_a = (uint16_t *)take((size_t)1024 * PC_OV_STEPS * lf);
        v->ov_bwd_a = (uint16_t *)take((size_t)1024 * PC_OV_STEPS * lb);
        v->ov_fwd_col = (uint32_t *)take((size_t)64 * PC_OV_STEPS * lf);
        v->ov_bwd_col = (uint32_t *)take((size_t)64 * PC_OV_STEPS * lb);
        v->ov_fwd_sub_cnt = (uint32_t *)take(sizeof(uint32_t) * 2 * lf);
        v->ov_bwd_sub_cnt = (uint32_t *)take(sizeof(uint32_t) * 2 * lb);
        v->ov_fwd_sub_ent = (uint2 *)take(sizeof(uint2) * PC_OV_SUB * 2 * lf);
        v->ov_bwd_sub_ent = (uint2 *)take(sizeof(uint2) * PC_OV_SUB * 2 * lb);
    } else {
        v->ws_fwd_val = v->ws_bwd_val = nullptr;
        v->ws_fwd_idx = v->ws_bwd_idx = nullptr;
        v->ws_fwd_flag = v->ws_bwd_flag = nullptr;
        v->ov_fwd_cnt = v->ov_bwd_cnt = nullptr;
        v->ov_fwd_a = v->ov_bwd_a = nullptr;
        v->ov_fwd_col = v->ov_bwd_col = nullptr;
        v->ov_fwd_sub_cnt = v->ov_bwd_sub_cnt = nullptr;
        v->ov_fwd_sub_ent = v->ov_bwd_sub_ent = nullptr;
    }
    return off;
}

extern "C" void pc_packed_free(pc_packed *pk)
{
    if (!pk) return;
    (void)hipSetDevice(pk->device);
    if (pk->packed_evt) {
        (void)hipEventSynchronize(pk->packed_evt);
        (void)hipEventDestroy(pk->packed_evt);
    }
    (void)hipDeviceSynchronize();
    if (pk->slab) (void)hipFree(pk->slab);
    delete pk;
}

extern "C" pc_status pc_pack(pc_ctx *ctx, const float *W, const uint8_t *pid, const uint8_t *keep,
                             int32_t F, int32_t C, const uint16_t *lib, int32_t P, pc_dtype dt, pc_packed **out)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!W || !pid || !keep || !lib || !out) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack: null pointer");
    if (F < 1 || C < 1 || F > 65535 || C > 65535)
        return pc_fail(ctx, PC_ERR_BAD_SHAPE, "pc_pack: F=%d C=%d out of range", F, C);
    if (dt != PC_F32 && dt != PC_BF16) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack: dtype %d", (int)dt);
    if ((int64_t)F * C >= ((int64_t)1 << 31))   // slots and row offsets of the tables are 32-bit
        return pc_fail(ctx, PC_ERR_UNSUPPORTED, "pc_pack: F*C = %lld kernels, the tables hold fewer than 2^31", (long long)F * C);
    pc_status s = pc_check_library(lib, P);
    if (s != PC_OK) return pc_fail(ctx, s, "pc_pack: bad library (P=%d)", P);

    int variant;
    bool can_mfma = (dt == PC_BF16) && pc_mfma_supports(F, C);
    const bool want_sparse = ctx->forced == PC_VARIANT_MFMA_SPARSE;
    if (ctx->forced == PC_VARIANT_MFMA || want_sparse) {
        if (!can_mfma)
            return pc_fail(ctx, PC_ERR_UNSUPPORTED, "pc_pack: MFMA variant needs bf16 and supported F=%d C=%d", F, C);
        variant = PC_VARIANT_MFMA;
    } else if (ctx->forced == PC_VARIANT_VALU) {
        variant = PC_VARIANT_VALU;
    } else {
        variant = can_mfma ? PC_VARIANT_MFMA : PC_VARIANT_VALU;
    }
    PC_HIP(ctx, hipSetDevice(ctx->device));

    pc_packed *pk = *out;
    if (pk) {
        if (pk->v.F != F || pk->v.C != C || pk->dtype != dt || pk->device != ctx->device)
            return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack: handle was packed for another layer shape or dtype");
        if (variant == PC_VARIANT_MFMA && !pk->v.wz_fwd) variant = PC_VARIANT_VALU;  // no tiles in this slab
    } else {
        pk = new (std::nothrow) pc_packed();
        if (!pk) return pc_fail(ctx, PC_ERR_NOMEM, "pc_pack: host allocation failed");
        memset(pk, 0, sizeof(*pk));
        pk->device = ctx->device;
        pk->dtype = dt;
        bool tiles = (dt == PC_BF16) && pc_mfma_supports(F, C);
        pk->slab_bytes = carve(&pk->v, &pk->v_dev, nullptr, F, C, tiles, want_sparse);
        hipError_t e = hipMalloc(&pk->slab, pk->slab_bytes);
        if (e != hipSuccess) {
            delete pk;
            return pc_hip_check(ctx, e, "pc_pack: hipMalloc");
        }
        carve(&pk->v, &pk->v_dev, (char *)pk->slab, F, C, tiles, want_sparse);
        e = hipMemcpy(pk->v_dev, &pk->v, sizeof(PackView), hipMemcpyHostToDevice);   // pointers and extents: fixed for the handle's life
        if (e != hipSuccess) {
            (void)hipFree(pk->slab);
            delete pk;
            return pc_hip_check(ctx, e, "pc_pack: hipMemcpy");
        }
        if (hipEventCreateWithFlags(&pk->packed_evt, hipEventDisableTiming) != hipSuccess) {
            (void)hipFree(pk->slab);
            delete pk;
            return pc_fail(ctx, PC_ERR_DEVICE, "pc_pack: event creation failed");
        }
    }
    pk->variant = variant;
    pk->v.P = P;
    pk->nnzk = -1;
    memcpy(pk->lib, lib, sizeof(uint16_t) * P);
    LibArg la;
    pc_fill_lib(&la, lib, P);
    memcpy(pk->taps, la.taps, sizeof(pk->taps));
    s = pc_launch_pack(ctx, pk, W, pid, keep);
    // An event recorded while the stream is being captured into a graph cannot be waited on afterwards, so a
    // captured pack records none; pc_packed_info then waits for the context's stream instead.
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ctx->stream, &cap) != hipSuccess) {
        (void)hipGetLastError();
        cap = hipStreamCaptureStatusNone;
    }
    pk->evt_recorded = false;
    if (s == PC_OK && cap == hipStreamCaptureStatusNone) {
        s = pc_hip_check(ctx, hipEventRecord(pk->packed_evt, ctx->stream), "hipEventRecord");
        pk->evt_recorded = s == PC_OK;
    }
    if (s != PC_OK) {
        if (!*out) pc_packed_free(pk);
        return s;
    }
    *out = pk;
    return PC_OK;
}

extern "C" pc_status pc_pack_batch(pc_ctx *ctx, int32_t n_layers, const float *const *W, const uint8_t *const *pid,
                                   const uint8_t *const *keep, const uint16_t *lib, int32_t P, pc_packed *const *packs)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!W || !pid || !keep || !lib || !packs) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack_batch: null pointer");
    pc_status s = pc_check_library(lib, P);
    if (s != PC_OK) return pc_fail(ctx, s, "pc_pack_batch: bad library (P=%d)", P);
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l] || !pid[l] || !keep[l] || !packs[l])
            return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack_batch: null pointer in layer %d", l);
        if (packs[l]->device != ctx->device) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack_batch: layer %d: other device", l);
        for (int m = 0; m < l; ++m)
            if (packs[m] == packs[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_pack_batch: layers %d and %d share a handle", m, l);
    }
    PC_HIP(ctx, hipSetDevice(ctx->device));
    LibArg la;
    pc_fill_lib(&la, lib, P);
    for (int l = 0; l < n_layers; ++l) {
        pc_packed *pk = packs[l];
        pk->v.P = P;
        pk->nnzk = -1;
        pk->evt_recorded = false;
        memcpy(pk->lib, lib, sizeof(uint16_t) * P);
        memcpy(pk->taps, la.taps, sizeof(pk->taps));
    }
    s = pc_launch_pack_batch(ctx, n_layers, packs, W, pid, keep, la);
    if (s != PC_OK) return s;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(ctx->stream, &cap) != hipSuccess) {
        (void)hipGetLastError();
        cap = hipStreamCaptureStatusNone;
    }
    if (cap == hipStreamCaptureStatusNone)
        for (int l = 0; l < n_layers; ++l) {
            s = pc_hip_check(ctx, hipEventRecord(packs[l]->packed_evt, ctx->stream), "hipEventRecord");
            if (s != PC_OK) return s;
            packs[l]->evt_recorded = true;
        }
    return PC_OK;
}

extern "C" pc_status pc_update_values(pc_ctx *ctx, pc_packed *pk, const float *W)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!pk || !W) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values: null pointer");
    if (pk->device != ctx->device) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values: other device");
    PC_HIP(ctx, hipSetDevice(ctx->device));
    return pc_launch_update_values(ctx, pk, W);
}

extern "C" pc_status pc_update_values_batch(pc_ctx *ctx, int32_t n_layers, pc_packed *const *packs, const float *const *W)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!packs || !W) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values_batch: null pointer");
    for (int l = 0; l < n_layers; ++l) {
        if (!packs[l] || !W[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values_batch: null pointer in layer %d", l);
        if (packs[l]->device != ctx->device) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values_batch: layer %d: other device", l);
        for (int m = 0; m < l; ++m)
            if (packs[m] == packs[l])
                return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_update_values_batch: layers %d and %d share a handle", m, l);
    }
    PC_HIP(ctx, hipSetDevice(ctx->device));
    return pc_launch_update_values_batch(ctx, n_layers, packs, W);
}

extern "C" pc_status pc_packed_info(pc_ctx *ctx, const pc_packed *pk, int64_t *nnz, int32_t *variant)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!pk) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_packed_info: null handle");
    if (nnz) {
        pc_packed *m = const_cast<pc_packed *>(pk);
        if (m->nnzk < 0) {
            PC_HIP(ctx, hipSetDevice(ctx->device));
            if (pk->evt_recorded) PC_HIP(ctx, hipEventSynchronize(pk->packed_evt));
            else PC_HIP(ctx, hipStreamSynchronize(ctx->stream));
            int32_t n = 0;
            PC_HIP(ctx, hipMemcpy(&n, pk->v.fm_rowptr + pk->v.F, sizeof(int32_t), hipMemcpyDeviceToHost));
            m->nnzk = n;
        }
        *nnz = m->nnzk;
    }
    if (variant) *variant = (pk->variant == PC_VARIANT_MFMA && pk->v.ws_fwd_val) ? (int32_t)PC_VARIANT_MFMA_SPARSE : pk->variant;
    return PC_OK;
}

extern "C" pc_status pc_scatter_dense(pc_ctx *ctx, const pc_packed *pk, const float *compact, float *dense)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!pk || !compact || !dense) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_scatter_dense: null pointer");
    PC_HIP(ctx, hipSetDevice(ctx->device));
    return pc_launch_scatter(ctx, pk, compact, dense, 0);
}

extern "C" pc_status pc_unpack_dense(pc_ctx *ctx, const pc_packed *pk, float *dense)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (!pk || !dense) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_unpack_dense: null pointer");
    PC_HIP(ctx, hipSetDevice(ctx->device));
    return pc_launch_scatter(ctx, pk, nullptr, dense, 1);
}

// ------------------------------------------------------------------ conv passes
static pc_status check_conv(pc_ctx *ctx, const char *who, const pc_conv_desc *d, const pc_packed *pk,
                            const void *a, const void *b, const void *c)
{
    if (!d || !pk || !a || !b || !c) return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: null pointer", who);
    pc_status s = pc_check_conv_desc(d);
    if (s != PC_OK)
        return pc_fail(ctx, s, "%s: bad descriptor N=%d H=%d W=%d C=%d F=%d stride=%d dtype=%d", who, d->N, d->H,
                       d->W, d->C, d->F, d->stride, (int)d->dtype);
    if (d->C != pk->v.C || d->F != pk->v.F)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: descriptor C=%d F=%d but the pack holds C=%d F=%d", who, d->C,
                       d->F, pk->v.C, pk->v.F);
    if (d->dtype != pk->dtype)
        return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: descriptor dtype differs from the pack's compute dtype", who);
    if (pk->device != ctx->device) return pc_fail(ctx, PC_ERR_INVALID_ARG, "%s: pack lives on another device", who);
    return pc_hip_check(ctx, hipSetDevice(ctx->device), "hipSetDevice");
}

extern "C" pc_status pc_conv_fwd(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *y)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = check_conv(ctx, "pc_conv_fwd", d, pk, x, y, y);
    if (s != PC_OK) return s;
    return pk->variant == PC_VARIANT_MFMA ? pc_mfma_fwd(ctx, d, pk, x, y) : pc_valu_fwd(ctx, d, pk, x, y);
}

extern "C" pc_status pc_conv_bwd_data(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy,
                                      void *dx)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = check_conv(ctx, "pc_conv_bwd_data", d, pk, dy, dx, dx);
    if (s != PC_OK) return s;
    return pk->variant == PC_VARIANT_MFMA ? pc_mfma_bwd_data(ctx, d, pk, dy, dx) : pc_valu_bwd_data(ctx, d, pk, dy, dx);
}

extern "C" pc_status pc_conv_fwd_relu(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x, void *a)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = check_conv(ctx, "pc_conv_fwd_relu", d, pk, x, a, a);
    if (s != PC_OK) return s;
    bool fused = false;
    s = pk->variant == PC_VARIANT_MFMA ? pc_mfma_fwd(ctx, d, pk, x, a, PC_ACT_RELU, &fused) : pc_valu_fwd(ctx, d, pk, x, a);
    if (s != PC_OK || fused) return s;
    const int64_t n = (int64_t)d->N * ((d->H - 1) / d->stride + 1) * ((d->W - 1) / d->stride + 1) * d->F;
    return pc_launch_relu(ctx, a, n, d->dtype);
}

extern "C" pc_status pc_conv_bwd_data_relu(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *dy, const void *x,
                                           void *dx)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = check_conv(ctx, "pc_conv_bwd_data_relu", d, pk, dy, x, dx);
    if (s != PC_OK) return s;
    bool fused = false;
    s = pk->variant == PC_VARIANT_MFMA ? pc_mfma_bwd_data(ctx, d, pk, dy, dx, PC_ACT_RELU_MASK, x, &fused)
                                       : pc_valu_bwd_data(ctx, d, pk, dy, dx);
    if (s != PC_OK || fused) return s;
    return pc_launch_relu_mask(ctx, dx, x, (int64_t)d->N * d->H * d->W * d->C, d->dtype);
}

extern "C" pc_status pc_conv_bwd_weight(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x,
                                        const void *dy, float *dw)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = check_conv(ctx, "pc_conv_bwd_weight", d, pk, x, dy, dw);
    if (s != PC_OK) return s;
    return pk->variant == PC_VARIANT_MFMA ? pc_mfma_bwd_weight(ctx, d, pk, x, dy, dw)
                                          : pc_valu_bwd_weight(ctx, d, pk, x, dy, dw);
}

extern "C" pc_status pc_conv_bwd_weight_noalloc(pc_ctx *ctx, const pc_conv_desc *d, const pc_packed *pk, const void *x,
                                                const void *dy, float *dw)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    pc_status s = check_conv(ctx, "pc_conv_bwd_weight_noalloc", d, pk, x, dy, dw);
    if (s != PC_OK) return s;
    // the same kernels as pc_conv_bwd_weight; every scratch request of the call is served from the fixed buffer
    ctx->fixed_scratch = true;
    s = pk->variant == PC_VARIANT_MFMA ? pc_mfma_bwd_weight(ctx, d, pk, x, dy, dw) : pc_valu_bwd_weight(ctx, d, pk, x, dy, dw);
    ctx->fixed_scratch = false;
    return s;
}

extern "C" pc_status pc_conv_bwd_weight_batch(pc_ctx *ctx, int32_t n_layers, const pc_conv_desc *descs, const pc_packed *const *packs,
                                              const void *const *x, const void *const *dy, float *const *dw)
{
    if (!ctx) return PC_ERR_INVALID_ARG;
    if (n_layers < 0) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_conv_bwd_weight_batch: n_layers %d", n_layers);
    if (n_layers == 0) return PC_OK;
    if (!descs || !packs || !x || !dy || !dw) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_conv_bwd_weight_batch: null pointer");
    std::vector<pc_conv_desc> md;
    std::vector<const pc_packed *> mp;
    std::vector<const void *> mx, mdy;
    std::vector<float *> mdw;
    for (int l = 0; l < n_layers; ++l) {
        if (!packs[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_conv_bwd_weight_batch: null handle in layer %d", l);
        pc_status s = check_conv(ctx, "pc_conv_bwd_weight_batch", &descs[l], packs[l], x[l], dy[l], dw[l]);
        if (s != PC_OK) return s;
        for (int m = 0; m < l; ++m)
            if (dw[m] == dw[l]) return pc_fail(ctx, PC_ERR_INVALID_ARG, "pc_conv_bwd_weight_batch: layers %d and %d share dw", m, l);
    }
    // the gather kernels one layer at a time, then the matrix-core layers together
    for (int l = 0; l < n_layers; ++l) {
        if (packs[l]->variant == PC_VARIANT_MFMA) {
            md.push_back(descs[l]); mp.push_back(packs[l]); mx.push_back(x[l]); mdy.push_back(dy[l]); mdw.push_back(dw[l]);
        } else {
            pc_status s = pc_valu_bwd_weight(ctx, &descs[l], packs[l], x[l], dy[l], dw[l]);
            if (s != PC_OK) return s;
        }
    }
    if (md.empty()) return PC_OK;
    return pc_mfma_bwd_weight_group(ctx, (int)md.size(), md.data(), mp.data(), mx.data(), mdy.data(), mdw.data());
}

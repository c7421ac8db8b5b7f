"""ctypes binding of libpatconv.so: the same entry points as include/pc.h, argument marshalling only.

Device buffers are passed as anything with a ``data_ptr()`` method (torch tensors on the context's
GPU) or as integer addresses. Nothing here computes: every step runs in the library's kernels.
There is no fallback: if the library is missing, load() raises.
"""
from __future__ import annotations

import ctypes as ct
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpatconv.so")

PC_OK = 0
PC_ERR_INVALID_ARG, PC_ERR_BAD_LIBRARY, PC_ERR_BAD_SHAPE, PC_ERR_UNSUPPORTED, PC_ERR_NOMEM, PC_ERR_DEVICE = range(1, 7)
PC_F32, PC_BF16 = 0, 1
PC_KEEP_PER_FILTER, PC_KEEP_PER_LAYER = 0, 1
PC_SCORE_RETAINED, PC_SCORE_KERNEL = 0, 1
PC_VARIANT_AUTO, PC_VARIANT_VALU, PC_VARIANT_MFMA, PC_VARIANT_MFMA_SPARSE = 0, 1, 2, 3

EXPORTS = [
    "pc_create", "pc_destroy", "pc_status_str", "pc_last_error", "pc_last_kernel", "pc_set_variant", "pc_set_plan_override",
    "pc_check_library", "pc_check_conv_desc", "pc_pattern_select", "pc_pack", "pc_update_values",
    "pc_packed_info", "pc_packed_free", "pc_scatter_dense", "pc_unpack_dense",
    "pc_conv_fwd", "pc_conv_bwd_data", "pc_conv_bwd_weight", "pc_conv_bwd_weight_noalloc",
    "pc_dppg_accumulate", "pc_dppg_pool", "pc_finalize_count", "pc_finalize_pick", "pc_group_lasso_grad",
    "pc_act_pool_fwd", "pc_act_pool_bwd", "pc_pattern_select_batch", "pc_pack_batch", "pc_update_values_batch",
    "pc_dppg_accumulate_batch", "pc_finalize_count_batch", "pc_finalize_pick_batch", "pc_group_lasso_grad_batch", "pc_conv_bwd_weight_batch", "pc_conv_fwd_relu", "pc_conv_bwd_data_relu",
]


class pc_conv_desc(ct.Structure):
    _fields_ = [("N", ct.c_int32), ("H", ct.c_int32), ("W", ct.c_int32), ("C", ct.c_int32), ("F", ct.c_int32),
                ("stride", ct.c_int32), ("dtype", ct.c_int)]


class PcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("libpatconv status %d: %s" % (status, message))
        self.status = status


_lib = None


def load():
    """Loads libpatconv.so. Raises if it has not been built (paper_2011_10170_amd/build.py)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libpatconv.so is not built: run `python -m paper_2011_10170_amd.build` "
                           "(there is no CPU fallback)")
    lib = ct.CDLL(LIB_PATH)
    vp, i32, i64 = ct.c_void_p, ct.c_int32, ct.c_int64
    lib.pc_create.argtypes = [ct.POINTER(vp), ct.c_int, vp]
    lib.pc_destroy.argtypes = [vp]
    lib.pc_destroy.restype = None
    lib.pc_status_str.argtypes = [ct.c_int]
    lib.pc_status_str.restype = ct.c_char_p
    lib.pc_last_error.argtypes = [vp]
    lib.pc_last_error.restype = ct.c_char_p
    lib.pc_last_kernel.argtypes = [vp]
    lib.pc_last_kernel.restype = ct.c_char_p
    lib.pc_set_variant.argtypes = [vp, ct.c_int]
    lib.pc_set_plan_override.argtypes = [vp, i32, i32]
    lib.pc_check_library.argtypes = [vp, i32]
    lib.pc_check_conv_desc.argtypes = [ct.POINTER(pc_conv_desc)]
    lib.pc_pattern_select.argtypes = [vp, vp, vp, i32, i32, vp, i32, ct.c_int, i64, ct.c_int, vp, vp]
    lib.pc_pack.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, ct.c_int, ct.POINTER(vp)]
    lib.pc_update_values.argtypes = [vp, vp, vp]
    lib.pc_packed_info.argtypes = [vp, vp, ct.POINTER(i64), ct.POINTER(i32)]
    lib.pc_packed_free.argtypes = [vp]
    lib.pc_packed_free.restype = None
    lib.pc_scatter_dense.argtypes = [vp, vp, vp, vp]
    lib.pc_unpack_dense.argtypes = [vp, vp, vp]
    lib.pc_conv_fwd.argtypes = [vp, ct.POINTER(pc_conv_desc), vp, vp, vp]
    lib.pc_conv_bwd_data.argtypes = [vp, ct.POINTER(pc_conv_desc), vp, vp, vp]
    lib.pc_conv_bwd_weight.argtypes = [vp, ct.POINTER(pc_conv_desc), vp, vp, vp, vp]
    lib.pc_conv_bwd_weight_noalloc.argtypes = [vp, ct.POINTER(pc_conv_desc), vp, vp, vp, vp]
    lib.pc_dppg_accumulate.argtypes = [vp, vp, vp, i32, i32, vp, vp]
    lib.pc_dppg_pool.argtypes = [vp, vp, i32, vp, vp, ct.POINTER(i32)]
    lib.pc_finalize_count.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.pc_finalize_pick.argtypes = [vp, vp, i32, i32, i32, vp]
    lib.pc_group_lasso_grad.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, ct.c_float, ct.c_float, vp, vp]
    lib.pc_pattern_select_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, ct.c_int, vp, ct.c_int, vp, vp]
    lib.pc_pack_batch.argtypes = [vp, i32, vp, vp, vp, vp, i32, vp]
    lib.pc_update_values_batch.argtypes = [vp, i32, vp, vp]
    lib.pc_conv_bwd_weight_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp]
    lib.pc_conv_fwd_relu.argtypes = [vp, vp, vp, vp, vp]
    lib.pc_conv_bwd_data_relu.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.pc_dppg_accumulate_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
    lib.pc_finalize_count_batch.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    lib.pc_finalize_pick_batch.argtypes = [vp, i32, vp, vp, vp, i32, vp]
    lib.pc_group_lasso_grad_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, i32, ct.c_float, ct.c_float, vp, vp]
    lib.pc_act_pool_fwd.argtypes = [vp, vp, i32, i32, i32, i32, ct.c_int, i32, vp, vp]
    lib.pc_act_pool_bwd.argtypes = [vp, vp, vp, i32, i32, i32, i32, ct.c_int, i32, vp]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name not in ("pc_destroy", "pc_packed_free", "pc_status_str", "pc_last_error", "pc_last_kernel"):
            fn.restype = ct.c_int
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return int(t)


def _lib_arr(masks: Sequence[int]):
    arr = (ct.c_uint16 * len(masks))(*[int(m) for m in masks])
    return arr


def _check(ctx, status: int):
    if status != PC_OK:
        lib = load()
        msg = lib.pc_status_str(status).decode()
        if ctx:
            detail = lib.pc_last_error(ctx).decode()
            if detail:
                msg += " (" + detail + ")"
        raise PcError(status, msg)


def make_desc(N, H, W, C, F, stride, dtype) -> pc_conv_desc:
    return pc_conv_desc(int(N), int(H), int(W), int(C), int(F), int(stride), int(dtype))


def pc_create(device: int = 0, hip_stream: Optional[int] = None) -> int:
    ctx = ct.c_void_p()
    _check(None, load().pc_create(ct.byref(ctx), int(device), hip_stream))
    return ctx.value


def pc_destroy(ctx) -> None:
    load().pc_destroy(ctx)


def pc_last_kernel(ctx) -> str:
    return load().pc_last_kernel(ctx).decode()


def pc_set_variant(ctx, variant: int) -> None:
    _check(ctx, load().pc_set_variant(ctx, int(variant)))


def pc_set_plan_override(ctx, tile_cfg: int = -1, split_k: int = 0) -> None:
    _check(ctx, load().pc_set_plan_override(ctx, int(tile_cfg), int(split_k)))


def pc_check_library(masks: Sequence[int]) -> int:
    return load().pc_check_library(ct.cast(_lib_arr(masks), ct.c_void_p), len(masks))


def pc_check_conv_desc(desc: pc_conv_desc) -> int:
    return load().pc_check_conv_desc(ct.byref(desc))


def pc_pattern_select(ctx, W, G, F, C, masks, keep_mode, n_keep, score_mode, pid, keep) -> None:
    arr = _lib_arr(masks)
    _check(ctx, load().pc_pattern_select(ctx, _ptr(W), _ptr(G), int(F), int(C), ct.cast(arr, ct.c_void_p), len(masks),
                                         int(keep_mode), int(n_keep), int(score_mode), _ptr(pid), _ptr(keep)))


def pc_pack(ctx, W, pid, keep, F, C, masks, compute_dtype, reuse: Optional[int] = None) -> int:
    arr = _lib_arr(masks)
    out = ct.c_void_p(reuse)
    _check(ctx, load().pc_pack(ctx, _ptr(W), _ptr(pid), _ptr(keep), int(F), int(C), ct.cast(arr, ct.c_void_p),
                               len(masks), int(compute_dtype), ct.byref(out)))
    return out.value


def pc_update_values(ctx, pk, W) -> None:
    _check(ctx, load().pc_update_values(ctx, pk, _ptr(W)))


def pc_packed_info(ctx, pk):
    nnz = ct.c_int64()
    var = ct.c_int32()
    _check(ctx, load().pc_packed_info(ctx, pk, ct.byref(nnz), ct.byref(var)))
    return nnz.value, var.value


def pc_packed_free(pk) -> None:
    load().pc_packed_free(pk)


def pc_scatter_dense(ctx, pk, compact, dense) -> None:
    _check(ctx, load().pc_scatter_dense(ctx, pk, _ptr(compact), _ptr(dense)))


def pc_unpack_dense(ctx, pk, dense) -> None:
    _check(ctx, load().pc_unpack_dense(ctx, pk, _ptr(dense)))


def pc_conv_fwd(ctx, desc, pk, x, y) -> None:
    _check(ctx, load().pc_conv_fwd(ctx, ct.byref(desc), pk, _ptr(x), _ptr(y)))


def pc_conv_bwd_data(ctx, desc, pk, dy, dx) -> None:
    _check(ctx, load().pc_conv_bwd_data(ctx, ct.byref(desc), pk, _ptr(dy), _ptr(dx)))


def pc_conv_bwd_weight(ctx, desc, pk, x, dy, dw_compact) -> None:
    _check(ctx, load().pc_conv_bwd_weight(ctx, ct.byref(desc), pk, _ptr(x), _ptr(dy), _ptr(dw_compact)))


def pc_conv_bwd_weight_noalloc(ctx, desc, pk, x, dy, dw_compact) -> None:
    _check(ctx, load().pc_conv_bwd_weight_noalloc(ctx, ct.byref(desc), pk, _ptr(x), _ptr(dy), _ptr(dw_compact)))


def pc_dppg_accumulate(ctx, W, G, F, C, hist, masks=None) -> None:
    _check(ctx, load().pc_dppg_accumulate(ctx, _ptr(W), _ptr(G), int(F), int(C), _ptr(hist), _ptr(masks)))


def pc_dppg_pool(ctx, hist, n_patterns: int):
    """Returns (masks, scores) of the patterns with the highest competitive scores (at most n_patterns)."""
    lib_out = (ct.c_uint16 * n_patterns)()
    score_out = (ct.c_uint32 * n_patterns)()
    n = ct.c_int32()
    _check(ctx, load().pc_dppg_pool(ctx, _ptr(hist), int(n_patterns), ct.cast(lib_out, ct.c_void_p),
                                    ct.cast(score_out, ct.c_void_p), ct.byref(n)))
    return [int(lib_out[i]) for i in range(n.value)], [int(score_out[i]) for i in range(n.value)]


def pc_finalize_count(ctx, pid, F, C, P, counts) -> None:
    _check(ctx, load().pc_finalize_count(ctx, _ptr(pid), int(F), int(C), int(P), _ptr(counts)))


def pc_finalize_pick(ctx, counts, F, C, P, pid) -> None:
    _check(ctx, load().pc_finalize_pick(ctx, _ptr(counts), int(F), int(C), int(P), _ptr(pid)))


def pc_group_lasso_grad(ctx, W, pid, keep, F, C, masks, lambda_p, lambda_i, dW, penalty=None) -> None:
    arr = _lib_arr(masks)
    _check(ctx, load().pc_group_lasso_grad(ctx, _ptr(W), _ptr(pid), _ptr(keep), int(F), int(C), ct.cast(arr, ct.c_void_p),
                                           len(masks), float(lambda_p), float(lambda_i), _ptr(dW), _ptr(penalty)))


def pc_act_pool_fwd(ctx, z, N, H, W, C, dtype, pool, a, sel) -> None:
    _check(ctx, load().pc_act_pool_fwd(ctx, _ptr(z), int(N), int(H), int(W), int(C), int(dtype), int(pool), _ptr(a), _ptr(sel)))


def pc_act_pool_bwd(ctx, da, sel, N, H, W, C, dtype, pool, dz) -> None:
    _check(ctx, load().pc_act_pool_bwd(ctx, _ptr(da), _ptr(sel), int(N), int(H), int(W), int(C), int(dtype), int(pool), _ptr(dz)))


def _ptr_array(items):
    return (ct.c_void_p * len(items))(*[_ptr(t) for t in items])


def pc_pattern_select_batch(ctx, W, G, F, C, masks, keep_mode, n_keep, score_mode, pid, keep) -> None:
    """W, G (or None), pid, keep: lists of device tensors; F, C, n_keep: lists of ints."""
    n = len(W)
    arr = _lib_arr(masks)
    _check(ctx, load().pc_pattern_select_batch(
        ctx, n, _ptr_array(W), _ptr_array(G) if G is not None else None, (ct.c_int32 * n)(*[int(v) for v in F]),
        (ct.c_int32 * n)(*[int(v) for v in C]), ct.cast(arr, ct.c_void_p), len(masks), int(keep_mode),
        (ct.c_int64 * n)(*[int(v) for v in n_keep]), int(score_mode), _ptr_array(pid), _ptr_array(keep)))


def pc_pack_batch(ctx, W, pid, keep, masks, packs) -> None:
    """Re-packs the existing handles `packs` (a list) from lists of device tensors."""
    n = len(W)
    arr = _lib_arr(masks)
    _check(ctx, load().pc_pack_batch(ctx, n, _ptr_array(W), _ptr_array(pid), _ptr_array(keep), ct.cast(arr, ct.c_void_p),
                                     len(masks), (ct.c_void_p * n)(*[int(p) for p in packs])))


def pc_update_values_batch(ctx, packs, W) -> None:
    n = len(packs)
    _check(ctx, load().pc_update_values_batch(ctx, n, (ct.c_void_p * n)(*[int(p) for p in packs]), _ptr_array(W)))


def _i32_array(vals):
    return (ct.c_int32 * len(vals))(*[int(v) for v in vals])


def pc_dppg_accumulate_batch(ctx, W, G, F, C, hist, masks=None) -> None:
    _check(ctx, load().pc_dppg_accumulate_batch(ctx, len(W), _ptr_array(W), _ptr_array(G) if G is not None else None,
                                                _i32_array(F), _i32_array(C), _ptr(hist),
                                                _ptr_array(masks) if masks is not None else None))


def pc_finalize_count_batch(ctx, pid, F, C, P, counts) -> None:
    _check(ctx, load().pc_finalize_count_batch(ctx, len(pid), _ptr_array(pid), _i32_array(F), _i32_array(C), int(P), _ptr_array(counts)))


def pc_finalize_pick_batch(ctx, counts, F, C, P, pid) -> None:
    _check(ctx, load().pc_finalize_pick_batch(ctx, len(pid), _ptr_array(counts), _i32_array(F), _i32_array(C), int(P), _ptr_array(pid)))


def pc_group_lasso_grad_batch(ctx, W, pid, keep, F, C, masks, lambda_p, lambda_i, dW, penalty=None) -> None:
    arr = _lib_arr(masks)
    _check(ctx, load().pc_group_lasso_grad_batch(ctx, len(W), _ptr_array(W), _ptr_array(pid), _ptr_array(keep), _i32_array(F),
                                                 _i32_array(C), ct.cast(arr, ct.c_void_p), len(masks), float(lambda_p),
                                                 float(lambda_i), _ptr_array(dW), _ptr(penalty)))


def pc_conv_bwd_weight_batch(ctx, descs, packs, x, dy, dw) -> None:
    """descs: list of pc_conv_desc; packs: list of handles; x, dy, dw: lists of device tensors."""
    n = len(descs)
    darr = (pc_conv_desc * n)(*descs)
    _check(ctx, load().pc_conv_bwd_weight_batch(ctx, n, ct.cast(darr, ct.c_void_p), (ct.c_void_p * n)(*[int(p) for p in packs]),
                                                _ptr_array(x), _ptr_array(dy), _ptr_array(dw)))


def pc_conv_fwd_relu(ctx, desc, pk, x, a) -> None:
    _check(ctx, load().pc_conv_fwd_relu(ctx, ct.byref(desc), pk, _ptr(x), _ptr(a)))


def pc_conv_bwd_data_relu(ctx, desc, pk, dy, x, dx) -> None:
    _check(ctx, load().pc_conv_bwd_data_relu(ctx, ct.byref(desc), pk, _ptr(dy), _ptr(x), _ptr(dx)))

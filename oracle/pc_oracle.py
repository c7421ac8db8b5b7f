"""ctypes access to the CPU oracle (oracle/pc_oracle.c). Test infrastructure only.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use this
module. It imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pc_oracle.c")
_LIB = os.path.join(_HERE, "libpc_oracle.so")
_lib = None

KEEP_PER_FILTER, KEEP_PER_LAYER = 0, 1
SCORE_RETAINED, SCORE_KERNEL = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc. Contraction is off so float32 operation order is as written."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = ct.CDLL(_LIB)
        _lib.orc_select.restype = ct.c_int
        _lib.orc_compact_order.restype = ct.c_int64
        _lib.orc_num_threads.restype = ct.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ct.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def out_dim(n: int, stride: int) -> int:
    return (n - 1) // stride + 1


def bf16_round(a: np.ndarray) -> np.ndarray:
    a = _f32(a)
    out = np.empty_like(a)
    lib().orc_bf16_round(_p(a), ct.c_int64(a.size), _p(out))
    return out


def select(W: np.ndarray, G: Optional[np.ndarray], lib_masks: np.ndarray, n_keep: int,
           keep_mode: int = KEEP_PER_FILTER, score_mode: int = SCORE_RETAINED) -> Tuple[np.ndarray, np.ndarray]:
    """W, G: [F][C][9] float32. Returns (pid uint8 [F][C], keep uint8 [F][C])."""
    W = _f32(W)
    F, C = W.shape[0], W.shape[1]
    G = None if G is None else _f32(G)
    masks = np.ascontiguousarray(lib_masks, dtype=np.uint16)
    pid = np.empty((F, C), dtype=np.uint8)
    keep = np.empty((F, C), dtype=np.uint8)
    rc = lib().orc_select(_p(W), _p(G), F, C, _p(masks), int(masks.size), int(keep_mode),
                          ct.c_int64(int(n_keep)), int(score_mode), _p(pid), _p(keep))
    if rc != 0:
        raise ValueError("orc_select: bad argument")
    return pid, keep


def mask(pid: np.ndarray, keep: np.ndarray, lib_masks: np.ndarray) -> np.ndarray:
    """0/1 tensor M [F][C][9]."""
    F, C = pid.shape
    masks = np.ascontiguousarray(lib_masks, dtype=np.uint16)
    M = np.empty((F, C, 9), dtype=np.uint8)
    lib().orc_mask(_p(np.ascontiguousarray(pid)), _p(np.ascontiguousarray(keep)), _p(masks), F, C, _p(M))
    return M


def apply_mask(W: np.ndarray, M: np.ndarray) -> np.ndarray:
    W = _f32(W)
    M = np.ascontiguousarray(M, dtype=np.uint8)
    out = np.empty_like(W)
    lib().orc_apply_mask(_p(W), _p(M), ct.c_int64(W.size), _p(out))
    return out


def compact_order(pid: np.ndarray, keep: np.ndarray, P: int) -> Tuple[np.ndarray, np.ndarray]:
    F, C = pid.shape
    pid = np.ascontiguousarray(pid)
    keep = np.ascontiguousarray(keep)
    n = lib().orc_compact_order(_p(pid), _p(keep), F, C, int(P), None, None)
    sf = np.empty(n, dtype=np.int32)
    sc = np.empty(n, dtype=np.int32)
    lib().orc_compact_order(_p(pid), _p(keep), F, C, int(P), _p(sf), _p(sc))
    return sf, sc


def gather_compact(dense: np.ndarray, pid: np.ndarray, lib_masks: np.ndarray,
                   slot_f: np.ndarray, slot_c: np.ndarray) -> np.ndarray:
    dense = _f32(dense)
    C = pid.shape[1]
    masks = np.ascontiguousarray(lib_masks, dtype=np.uint16)
    out = np.empty((slot_f.size, 4), dtype=np.float32)
    lib().orc_gather_compact(_p(dense), _p(np.ascontiguousarray(pid)), _p(masks), _p(slot_f), _p(slot_c),
                             ct.c_int64(slot_f.size), C, _p(out))
    return out


def _dims(x_shape, F):
    N, H, W, C = x_shape
    return int(N), int(H), int(W), int(C), int(F)


def conv_fwd(x: np.ndarray, Wm: np.ndarray, stride: int = 1) -> np.ndarray:
    """x [N][H][W][C], Wm [F][C][9] (already masked) -> y [N][Ho][Wo][F]."""
    x, Wm = _f32(x), _f32(Wm)
    N, H, W, C, F = _dims(x.shape, Wm.shape[0])
    assert Wm.shape[1] == C
    y = np.empty((N, out_dim(H, stride), out_dim(W, stride), F), dtype=np.float32)
    lib().orc_conv_fwd(_p(x), _p(Wm), N, H, W, C, F, int(stride), _p(y))
    return y


def conv_fwd_at(x: np.ndarray, Wm: np.ndarray, stride: int, idx: np.ndarray) -> np.ndarray:
    x, Wm = _f32(x), _f32(Wm)
    N, H, W, C, F = _dims(x.shape, Wm.shape[0])
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float32)
    lib().orc_conv_fwd_at(_p(x), _p(Wm), N, H, W, C, F, int(stride), _p(idx), ct.c_int64(idx.size), _p(out))
    return out


def conv_bwd_data(dy: np.ndarray, Wm: np.ndarray, x_shape, stride: int = 1) -> np.ndarray:
    dy, Wm = _f32(dy), _f32(Wm)
    N, H, W, C, F = _dims(x_shape, Wm.shape[0])
    assert dy.shape == (N, out_dim(H, stride), out_dim(W, stride), F)
    dx = np.empty((N, H, W, C), dtype=np.float32)
    lib().orc_conv_bwd_data(_p(dy), _p(Wm), N, H, W, C, F, int(stride), _p(dx))
    return dx


def conv_bwd_data_at(dy: np.ndarray, Wm: np.ndarray, x_shape, stride: int, idx: np.ndarray) -> np.ndarray:
    dy, Wm = _f32(dy), _f32(Wm)
    N, H, W, C, F = _dims(x_shape, Wm.shape[0])
    idx = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty(idx.size, dtype=np.float32)
    lib().orc_conv_bwd_data_at(_p(dy), _p(Wm), N, H, W, C, F, int(stride), _p(idx), ct.c_int64(idx.size), _p(out))
    return out


def conv_bwd_weight(x: np.ndarray, dy: np.ndarray, M: np.ndarray, stride: int = 1) -> np.ndarray:
    """Dense [F][C][9] gradient, zero wherever M is zero."""
    x, dy = _f32(x), _f32(dy)
    M = np.ascontiguousarray(M, dtype=np.uint8)
    N, H, W, C, F = _dims(x.shape, M.shape[0])
    dW = np.empty((F, C, 9), dtype=np.float32)
    lib().orc_conv_bwd_weight(_p(x), _p(dy), _p(M), N, H, W, C, F, int(stride), _p(dW))
    return dW


def conv_bwd_weight_at(x: np.ndarray, dy: np.ndarray, F: int, stride: int, widx: np.ndarray) -> np.ndarray:
    x, dy = _f32(x), _f32(dy)
    N, H, W, C, F = _dims(x.shape, F)
    widx = np.ascontiguousarray(widx, dtype=np.int64)
    out = np.empty(widx.size, dtype=np.float32)
    lib().orc_conv_bwd_weight_at(_p(x), _p(dy), N, H, W, C, F, int(stride), _p(widx), ct.c_int64(widx.size), _p(out))
    return out

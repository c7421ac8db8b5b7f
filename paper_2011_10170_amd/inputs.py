"""Seeded synthetic inputs and workload shape tables.

This module serves both the CPU oracle and the HIP path with the *same* arrays.
It holds no arithmetic of the method itself: only a counter-based random
generator, bf16 storage conversion of generated activations, the pattern
libraries used by the workloads, and the layer shape lists.

Generator: value i of stream s under seed k is a pure function of (k, s, i)
(splitmix64 finaliser over a mixed counter, then Box-Muller), so any slice of
any tensor can be regenerated independently and in any order.
"""
from __future__ import annotations

import itertools
import zlib
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple

import numpy as np

BASE_SEED = 20201110

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)


def _mix64(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on an array of uint64 (wrapping arithmetic)."""
    with np.errstate(over="ignore"):
        z = (z ^ (z >> _U64(30))) * _M1
        z = (z ^ (z >> _U64(27))) * _M2
        z = z ^ (z >> _U64(31))
    return z


def stream_id(*parts) -> int:
    """Stable 32-bit stream id from a tuple of names/numbers (crc32 of its repr)."""
    return zlib.crc32(repr(tuple(parts)).encode()) & 0xFFFFFFFF


def _key(seed: int, stream: int) -> np.uint64:
    k = np.array([(seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D)
                  & 0xFFFFFFFFFFFFFFFF], dtype=_U64)
    return _mix64(k)[0]


def uniform01(seed: int, stream: int, n: int, offset: int = 0, lane: int = 0) -> np.ndarray:
    """n float64 values in the open interval (0, 1); element i uses counter offset+i."""
    key = _key(seed, stream)
    with np.errstate(over="ignore"):
        ctr = (np.arange(offset, offset + n, dtype=_U64) * _U64(2) + _U64(lane)) * _GOLDEN + key
    h = _mix64(ctr)
    return ((h >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, n: int, offset: int = 0, chunk: int = 1 << 22) -> np.ndarray:
    """n standard-normal float32 values (Box-Muller on two hashed uniforms per element)."""
    out = np.empty(n, dtype=np.float32)
    for lo in range(0, n, chunk):
        m = min(chunk, n - lo)
        u1 = uniform01(seed, stream, m, offset + lo, 0)
        u2 = uniform01(seed, stream, m, offset + lo, 1)
        out[lo:lo + m] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)).astype(np.float32)
    return out


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# Pattern libraries. A pattern is a 9-bit mask; bit t = 3*r + s keeps the tap
# at kernel row r, column s. Every pattern keeps exactly 4 taps.
# --------------------------------------------------------------------------

def mask_of(taps: Sequence[int]) -> int:
    m = 0
    for t in taps:
        m |= 1 << t
    return m


def all_four_tap_masks() -> List[int]:
    """All C(9,4) masks, in lexicographic order of their tap tuples."""
    return [mask_of(c) for c in itertools.combinations(range(9), 4)]


_BLOCKS = [(0, 1, 3, 4), (1, 2, 4, 5), (3, 4, 6, 7), (4, 5, 7, 8)]
_TEES = [(1, 3, 4, 5), (1, 4, 5, 7), (3, 4, 5, 7), (1, 3, 4, 7)]
# The four further masks of the 12-pattern pool, stored as constants (drawn once with this module's generator from
# the masks the paper's pool generation can produce; tests/test_oracle_train.py checks with the oracle's own
# enumeration that each of them can be produced).
_EXTRA12 = [228, 402, 114, 147]


def _draw_without_replacement(pool: Sequence[int], k: int, seed: int, stream: int) -> List[int]:
    u = uniform01(seed, stream, len(pool))
    order = np.argsort(u, kind="stable")
    return [pool[i] for i in order[:k]]


def make_library(P: int, seed: int = BASE_SEED) -> np.ndarray:
    """Pattern library of the benchmark configurations, as uint16 masks.

    P=4: the four 2x2 blocks containing the centre. P=8: those plus the four
    centre+3-edge-neighbour T shapes. P=12: those plus 4 stored masks of the kind
    the pool generation produces. P=16: 16 seeded draws from all 126.
    P=126: every four-of-nine mask. Other P: the first P of a seeded shuffle of all 126.
    """
    if P == 4:
        lib = [mask_of(t) for t in _BLOCKS]
    elif P == 8:
        lib = [mask_of(t) for t in _BLOCKS + _TEES]
    elif P == 12:
        lib = [mask_of(t) for t in _BLOCKS + _TEES] + list(_EXTRA12)
    elif P == 126:
        lib = all_four_tap_masks()
    else:
        lib = _draw_without_replacement(all_four_tap_masks(), P, seed, stream_id("lib", P))
    assert len(lib) == P and len(set(lib)) == P
    return np.array(lib, dtype=np.uint16)


# --------------------------------------------------------------------------
# Workloads
# --------------------------------------------------------------------------

@dataclass(frozen=True)
class Layer:
    N: int
    H: int
    W: int
    C: int
    F: int
    stride: int = 1

    @property
    def Ho(self) -> int:
        return (self.H - 1) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W - 1) // self.stride + 1


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str          # "f32" or "bf16"
    P: int
    keep: float
    layers: Tuple[Layer, ...]
    with_select: bool = False   # the timed step also runs select (+ pack)


def kept_per_filter(keep: float, C: int) -> int:
    """Integer kept-kernel count per filter for a connectivity ratio: round half up, at least 1."""
    return max(1, int(np.floor(keep * C + 0.5)))


def _vgg16(N: int, H0: int) -> Tuple[Layer, ...]:
    chans = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256),
             (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]
    pool_after = {1, 3, 6, 9}   # 2x2 max-pool after these layer indices (0-based)
    out, h = [], H0
    for i, (c, f) in enumerate(chans):
        out.append(Layer(N, h, h, c, f, 1))
        if i in pool_after:
            h //= 2
    return tuple(out)


def _resnet18_cifar(N: int) -> Tuple[Layer, ...]:
    out = [Layer(N, 32, 32, 64, 64, 1)] * 4
    out += [Layer(N, 32, 32, 64, 128, 2)] + [Layer(N, 16, 16, 128, 128, 1)] * 3
    out += [Layer(N, 16, 16, 128, 256, 2)] + [Layer(N, 8, 8, 256, 256, 1)] * 3
    out += [Layer(N, 8, 8, 256, 512, 2)] + [Layer(N, 4, 4, 512, 512, 1)] * 3
    return tuple(out)


def _resnet50_imagenet(N: int) -> Tuple[Layer, ...]:
    out = [Layer(N, 56, 56, 64, 64, 1)] * 3
    out += [Layer(N, 56, 56, 128, 128, 2)] + [Layer(N, 28, 28, 128, 128, 1)] * 3
    out += [Layer(N, 28, 28, 256, 256, 2)] + [Layer(N, 14, 14, 256, 256, 1)] * 5
    out += [Layer(N, 14, 14, 512, 512, 2)] + [Layer(N, 7, 7, 512, 512, 1)] * 2
    return tuple(out)


WORKLOADS: Dict[str, Workload] = {
    "single_f32": Workload("single_f32", "f32", 4, 0.5, (Layer(8, 32, 32, 16, 16, 1),)),
    "vgg16_cifar": Workload("vgg16_cifar", "bf16", 8, 0.3, _vgg16(128, 32)),
    "resnet18_cifar": Workload("resnet18_cifar", "bf16", 8, 0.4, _resnet18_cifar(128), with_select=True),
    "resnet50_imagenet": Workload("resnet50_imagenet", "bf16", 12, 0.25, _resnet50_imagenet(64)),
    "vgg16_imagenet": Workload("vgg16_imagenet", "bf16", 16, 0.2, _vgg16(32, 224), with_select=True),
}
WORKLOAD_ORDER = ["single_f32", "vgg16_cifar", "resnet18_cifar", "resnet50_imagenet", "vgg16_imagenet"]


# --------------------------------------------------------------------------
# Tensors
# --------------------------------------------------------------------------

def gen_weights(F: int, C: int, seed: int, tag) -> np.ndarray:
    """Kaiming-normal (fan-in 9*C) fp32 weights, layout [F][C][3][3] flattened to [F][C][9]."""
    w = normal(seed, stream_id("W", tag, F, C), F * C * 9) * np.float32(np.sqrt(2.0 / (9.0 * C)))
    return w.reshape(F, C, 9)


def gen_weight_grads(F: int, C: int, seed: int, tag) -> np.ndarray:
    """Dense standard-normal stand-in for dE/dW, layout [F][C][9]."""
    return normal(seed, stream_id("G", tag, F, C), F * C * 9).reshape(F, C, 9)


PERIOD = 8388593   # prime; tensors longer than this repeat their first PERIOD values cyclically


def gen_activations(shape: Tuple[int, ...], seed: int, tag, relu: bool, dtype: str):
    """NHWC activations. relu=True gives max(0, N(0,1)) (post-ReLU feature maps),
    relu=False gives N(0,1) (incoming output gradients). Tensors with more than PERIOD
    elements repeat their first PERIOD values cyclically (generation time; the period is
    prime, so it never lines up with a tensor dimension).

    Returns (values_f32, storage): values_f32 holds exactly the numbers the
    kernels see (already rounded to bf16 when dtype == "bf16"); storage is the
    array to upload (float32, or uint16 bf16 bit patterns)."""
    n = int(np.prod(shape))
    a = normal(seed, stream_id("act", tag, tuple(shape), relu), min(n, PERIOD))
    if relu:
        np.maximum(a, np.float32(0), out=a)
    if n > PERIOD:
        a = np.resize(a, n)
    if dtype == "bf16":
        bits = f32_to_bf16_bits(a)
        return bf16_bits_to_f32(bits).reshape(shape), bits.reshape(shape)
    return a.reshape(shape), a.reshape(shape)

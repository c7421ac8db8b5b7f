"""Shared helpers for the GPU parity tests: build one layer's seeded inputs, run the oracle,
run the HIP path through the C ABI, compare."""
from __future__ import annotations

import numpy as np

from paper_2011_10170_amd import inputs as I

CANARY = 64


def rel_l2(a, b) -> float:
    a = np.asarray(a, dtype=np.float64).reshape(-1)
    b = np.asarray(b, dtype=np.float64).reshape(-1)
    den = float(np.linalg.norm(b))
    num = float(np.linalg.norm(a - b))
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


# ---------------------------------------------------------------- per-element bound
# Every output element is a sum of products. With float32 accumulation of exact products (bf16 x bf16 fits float32)
# the error of the sum is a small multiple of 2^-24 times mag = sum of |product| (typically 2^-25 * mag even for a
# fully sequential sum of any length, because the rounding errors add like a random walk; 2^-21 leaves a factor 16),
# and a bf16 result adds one rounding of at most 2^-8 relative (half a unit in the last place of 8 significant bits).
# mag comes from the same oracle routine applied to the absolute values of its inputs.
RTOL = {"bf16": 2.0 ** -8 * (1.0 + 2.0 ** -6), "f32": 2.0 ** -22}
ATOL_MAG = 2.0 ** -21
# relative L2 bounds: the stated ones are 1e-4 (float32) and 2e-2 (bf16 storage); the bf16 one is held at the
# measured level (1.7e-3: the output rounding alone) with a margin
TOL_L2 = {"f32": 1e-4, "bf16": 4e-3}
TOL_L2_DW = 1e-4


def elementwise_excess(got, ref, mag, out_kind: str):
    """(largest |got - ref| / tolerance over the elements, flat index of that element); <= 1 passes."""
    got = np.asarray(got, dtype=np.float64).reshape(-1)
    ref = np.asarray(ref, dtype=np.float64).reshape(-1)
    mag = np.asarray(mag, dtype=np.float64).reshape(-1)
    assert got.shape == ref.shape == mag.shape
    if got.size == 0:
        return 0.0, -1
    tol = RTOL[out_kind] * np.abs(ref) + ATOL_MAG * mag + 1e-37
    ratio = np.abs(got - ref) / tol
    ratio = np.where(np.isfinite(got), ratio, np.inf)
    i = int(np.argmax(ratio))
    return float(ratio[i]), i


def assert_close(got, ref, mag, out_kind: str, l2_tol: float, what: str = ""):
    """Both gates: the relative L2 norm of the difference, and every single element within its own bound."""
    e = rel_l2(got, ref)
    worst, at = elementwise_excess(got, ref, mag, out_kind)
    print("  %s rel_l2 %.3g, worst element at %.3f of its bound (flat index %d)" % (what, e, worst, at), flush=True)
    assert e <= l2_tol, (what, "rel_l2", e)
    assert worst <= 1.0, (what, "element", at, "error / bound", worst)


def stratified_indices(shape, rng, max_samples=150000):
    """Flat indices into an NHWC tensor, one per stratum (image, row, segment of sx pixels, group of sc channels),
    at a random place inside it: every 32-pixel x 32-channel accumulator tile of every kernel tile holds at least
    one sample (sx = sc = 16: four), whatever tile grid the planner chose. Strata grow to 32 when there would be
    more than max_samples of them."""
    N, H, W, CH = shape
    sx = sc = 16
    count = lambda: N * H * ((W + sx - 1) // sx) * ((CH + sc - 1) // sc)
    if count() > max_samples:
        sc = 32
    if count() > max_samples:
        sx = 32
    nx, ncg = (W + sx - 1) // sx, (CH + sc - 1) // sc
    n, y, xs, cg = np.meshgrid(np.arange(N), np.arange(H), np.arange(nx), np.arange(ncg), indexing="ij")
    n, y, xs, cg = (a.reshape(-1).astype(np.int64) for a in (n, y, xs, cg))
    wx = np.minimum(sx, W - xs * sx)
    wc = np.minimum(sc, CH - cg * sc)
    x = xs * sx + (rng.random(n.size) * wx).astype(np.int64)
    c = cg * sc + (rng.random(n.size) * wc).astype(np.int64)
    return ((n * H + y) * W + x) * CH + c


class Case:
    def __init__(self, layer: I.Layer, dtype: str, P: int, n_keep: int, seed: int = I.BASE_SEED, tag="case",
                 lib=None):
        self.layer, self.dtype, self.P, self.n_keep = layer, dtype, P, n_keep
        L = layer
        self.lib = I.make_library(P) if lib is None else np.asarray(lib, dtype=np.uint16)
        self.W = I.gen_weights(L.F, L.C, seed, tag)
        self.G = I.gen_weight_grads(L.F, L.C, seed, tag)
        self.x, self.x_store = I.gen_activations((L.N, L.H, L.W, L.C), seed, (tag, "x"), True, dtype)
        self.dy, self.dy_store = I.gen_activations((L.N, L.Ho, L.Wo, L.F), seed, (tag, "dy"), False, dtype)


def oracle_masks(oracle, case: Case, score_mode=0, keep_mode=0, with_grad=True):
    pid, keep = oracle.select(case.W, case.G if with_grad else None, case.lib, case.n_keep,
                              keep_mode=keep_mode, score_mode=score_mode)
    M = oracle.mask(pid, keep, case.lib)
    Wsrc = oracle.bf16_round(case.W) if case.dtype == "bf16" else case.W
    Wm = oracle.apply_mask(Wsrc, M)
    return pid, keep, M, Wm


# ---------------------------------------------------------------- device side
def _torch():
    import torch
    return torch


def to_dev(arr: np.ndarray):
    torch = _torch()
    if arr.dtype == np.uint16:     # bf16 bit patterns
        return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def from_dev_f32(t) -> np.ndarray:
    torch = _torch()
    if t.dtype == torch.bfloat16:
        bits = t.view(torch.int16).cpu().numpy().view(np.uint16)
        return I.bf16_bits_to_f32(bits)
    return t.cpu().numpy()


class Guarded:
    """Device buffer with sentinel-filled margins to catch writes outside the tensor."""

    def __init__(self, n_elem: int, torch_dtype):
        torch = _torch()
        self.n = n_elem
        self.buf = torch.full((n_elem + 2 * CANARY,), 7.0, dtype=torch_dtype, device="cuda")
        self.body = self.buf[CANARY:CANARY + n_elem]
        if n_elem:
            self.body.fill_(float("nan"))
        self.ptr = self.buf.data_ptr() + CANARY * self.buf.element_size()   # valid even when n_elem == 0

    def margins_intact(self) -> bool:
        torch = _torch()
        m = torch.cat([self.buf[:CANARY], self.buf[CANARY + self.n:]]).float()
        return bool((m == 7.0).all().item())


class GpuLayer:
    """Runs select -> pack -> the three passes of one layer through the C ABI."""

    def __init__(self, B, ctx, case: Case, variant=0, score_mode=0, keep_mode=0, with_grad=True):
        torch = _torch()
        self.B, self.ctx, self.case = B, ctx, case
        L = case.layer
        self.dt = B.PC_BF16 if case.dtype == "bf16" else B.PC_F32
        self.tdt = torch.bfloat16 if case.dtype == "bf16" else torch.float32
        B.pc_set_variant(ctx, variant)
        self.W = to_dev(case.W)
        self.G = to_dev(case.G) if with_grad else None
        self.pid = torch.full((L.F, L.C), 255, dtype=torch.uint8, device="cuda")
        self.keep = torch.full((L.F, L.C), 255, dtype=torch.uint8, device="cuda")
        B.pc_pattern_select(ctx, self.W, self.G, L.F, L.C, case.lib, keep_mode, case.n_keep, score_mode,
                            self.pid, self.keep)
        self.pk = B.pc_pack(ctx, self.W, self.pid, self.keep, L.F, L.C, case.lib, self.dt)
        self.nnzk, self.variant = B.pc_packed_info(ctx, self.pk)
        self.desc = B.make_desc(L.N, L.H, L.W, L.C, L.F, L.stride, self.dt)
        self.x = to_dev(case.x_store)
        self.dy = to_dev(case.dy_store)

    def fwd(self):
        L = self.case.layer
        g = Guarded(L.N * L.Ho * L.Wo * L.F, self.tdt)
        self.B.pc_conv_fwd(self.ctx, self.desc, self.pk, self.x, g.ptr)
        _torch().cuda.synchronize()
        assert g.margins_intact()
        return from_dev_f32(g.body).reshape(L.N, L.Ho, L.Wo, L.F)

    def bwd_data(self):
        L = self.case.layer
        g = Guarded(L.N * L.H * L.W * L.C, self.tdt)
        self.B.pc_conv_bwd_data(self.ctx, self.desc, self.pk, self.dy, g.ptr)
        _torch().cuda.synchronize()
        assert g.margins_intact()
        return from_dev_f32(g.body).reshape(L.N, L.H, L.W, L.C)

    def bwd_weight(self):
        torch = _torch()
        g = Guarded(self.nnzk * 4, torch.float32)
        self.B.pc_conv_bwd_weight(self.ctx, self.desc, self.pk, self.x, self.dy, g.ptr)
        torch.cuda.synchronize()
        assert g.margins_intact()
        return g.body.cpu().numpy().reshape(self.nnzk, 4), g

    def scatter(self, compact_dev):
        torch = _torch()
        L = self.case.layer
        dense = torch.full((L.F, L.C, 9), float("nan"), dtype=torch.float32, device="cuda")
        self.B.pc_scatter_dense(self.ctx, self.pk, compact_dev, dense)
        torch.cuda.synchronize()
        return dense.cpu().numpy()

    def unpack(self):
        torch = _torch()
        L = self.case.layer
        dense = torch.full((L.F, L.C, 9), float("nan"), dtype=torch.float32, device="cuda")
        self.B.pc_unpack_dense(self.ctx, self.pk, dense)
        torch.cuda.synchronize()
        return dense.cpu().numpy()

    def masks(self):
        _torch().cuda.synchronize()
        return self.pid.cpu().numpy(), self.keep.cpu().numpy()

    def close(self):
        self.B.pc_packed_free(self.pk)
        self.pk = None

"""Pins for the oracle's three convolution passes (CPU only).

Independent routes used: PyTorch-CPU conv2d and autograd in float64 (library routine), an
im2col product written here (the matrix view of Section 5.1), closed forms, adjoint identities.
"""
import itertools
import os

import numpy as np
import pytest
import torch

from paper_2011_10170_amd import inputs as I

SHAPES = [
    # N, H, W, C, F, stride
    (2, 6, 6, 3, 4, 1),
    (1, 5, 7, 4, 3, 1),
    (2, 8, 8, 5, 6, 2),
    (1, 7, 5, 3, 2, 2),
    (1, 1, 1, 2, 2, 1),
    (1, 2, 2, 3, 3, 2),
    (3, 9, 4, 8, 5, 1),
]


def _case(oracle, shape, P=8, keep=0.5, seed=7):
    N, H, W, C, F, stride = shape
    Wt = I.gen_weights(F, C, seed, ("t", shape))
    G = I.gen_weight_grads(F, C, seed, ("t", shape))
    lib = I.make_library(P)
    pid, kp = oracle.select(Wt, G, lib, I.kept_per_filter(keep, C))
    M = oracle.mask(pid, kp, lib)
    Wm = oracle.apply_mask(Wt, M)
    x, _ = I.gen_activations((N, H, W, C), seed, ("x", shape), True, "f32")
    Ho, Wo = oracle.out_dim(H, stride), oracle.out_dim(W, stride)
    dy, _ = I.gen_activations((N, Ho, Wo, F), seed, ("dy", shape), False, "f32")
    return x, dy, Wm, M, pid, kp, lib


def _torch_fwd(x, Wm, stride):
    xt = torch.from_numpy(x.astype(np.float64)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(Wm.astype(np.float64)).reshape(Wm.shape[0], Wm.shape[1], 3, 3)
    return xt, wt, torch.nn.functional.conv2d(xt, wt, stride=stride, padding=1)


@pytest.mark.parametrize("shape", SHAPES)
def test_fwd_matches_torch_conv2d(oracle, shape):
    x, dy, Wm, *_ = _case(oracle, shape)
    _, _, yt = _torch_fwd(x, Wm, shape[5])
    y = oracle.conv_fwd(x, Wm, shape[5])
    ref = yt.permute(0, 2, 3, 1).numpy()
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref.astype(np.float32), rtol=0, atol=1e-6)


@pytest.mark.parametrize("shape", SHAPES)
def test_bwd_matches_torch_autograd(oracle, shape):
    x, dy, Wm, M, *_ = _case(oracle, shape)
    stride = shape[5]
    xt, wt, _ = _torch_fwd(x, Wm, stride)
    xt = xt.clone().requires_grad_(True)
    wt = wt.clone().requires_grad_(True)
    yt = torch.nn.functional.conv2d(xt, wt, stride=stride, padding=1)
    yt.backward(torch.from_numpy(dy.astype(np.float64)).permute(0, 3, 1, 2))
    dx_ref = xt.grad.permute(0, 2, 3, 1).numpy()
    dw_ref = wt.grad.reshape(Wm.shape).numpy() * M
    dx = oracle.conv_bwd_data(dy, Wm, x.shape, stride)
    dw = oracle.conv_bwd_weight(x, dy, M, stride)
    np.testing.assert_allclose(dx, dx_ref.astype(np.float32), rtol=0, atol=2e-6)
    np.testing.assert_allclose(dw, dw_ref.astype(np.float32), rtol=1e-6, atol=1e-5)
    assert np.all(dw[M == 0] == 0.0)


def _im2col_product(x, Wm, stride):
    """Section 5.1's matrix view: (F x 9C) filter matrix times (9C x Ho*Wo) patch matrix, per image."""
    N, H, W, C = x.shape
    F = Wm.shape[0]
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    xp = np.zeros((N, H + 2, W + 2, C), dtype=np.float64)
    xp[:, 1:H + 1, 1:W + 1, :] = x
    # filter matrix columns ordered (c, r, s), as a [F][C][3][3] tensor flattens
    A = Wm.astype(np.float64).reshape(F, C * 9)
    out = np.empty((N, Ho, Wo, F))
    for n in range(N):
        B = np.empty((C * 9, Ho * Wo))
        for c in range(C):
            for r in range(3):
                for s in range(3):
                    patch = xp[n, r:r + (Ho - 1) * stride + 1:stride, s:s + (Wo - 1) * stride + 1:stride, c]
                    B[c * 9 + r * 3 + s] = patch.reshape(-1)
        out[n] = (A @ B).T.reshape(Ho, Wo, F)
    return out


@pytest.mark.parametrize("shape", SHAPES[:4])
def test_fwd_matches_im2col_product(oracle, shape):
    x, dy, Wm, *_ = _case(oracle, shape)
    y = oracle.conv_fwd(x, Wm, shape[5])
    np.testing.assert_allclose(y, _im2col_product(x, Wm, shape[5]).astype(np.float32), rtol=0, atol=1e-6)


def test_im2col_shape_of_the_papers_example():
    consts = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()[:2]
                consts[k] = int(v)
    F, C, H = 256, 128, 224
    assert (F, 9 * C) == (consts["im2col_filter_rows"], consts["im2col_filter_cols"])
    assert H * H == consts["im2col_input_cols"]


def test_all_ones_counts_in_range_taps(oracle):
    """x = 1, kept weights = 1: y = number of kept taps that fall inside the image."""
    N, H, W, C, F = 1, 5, 6, 6, 4
    lib = I.make_library(8)
    rng = np.random.default_rng(0)
    pid = rng.integers(0, 8, size=(F, C)).astype(np.uint8)
    keep = np.zeros((F, C), np.uint8)
    for f in range(F):
        keep[f, rng.permutation(C)[:3]] = 1
    M = oracle.mask(pid, keep, lib)
    Wm = M.astype(np.float32)
    y = oracle.conv_fwd(np.ones((N, H, W, C), np.float32), Wm, 1)
    # interior: every kept kernel contributes its 4 taps
    assert np.all(y[0, 1:H - 1, 1:W - 1, :] == 4.0 * 3)
    for oy, ox, f in itertools.product(range(H), range(W), range(F)):
        cnt = 0
        for c in range(C):
            if not keep[f, c]:
                continue
            for t in range(9):
                if (int(lib[pid[f, c]]) >> t) & 1:
                    iy, ix = oy + t // 3 - 1, ox + t % 3 - 1
                    cnt += (0 <= iy < H) and (0 <= ix < W)
        assert y[0, oy, ox, f] == cnt


def test_impulse_shows_flipped_pattern(oracle):
    """A unit impulse at (py,px) in channel c gives y[py-(r-1), px-(s-1), f] = Wm[f,c,r,s]."""
    H = W = 7
    C, F = 3, 2
    lib = I.make_library(4)
    Wt = I.gen_weights(F, C, 3, "imp")
    pid = np.array([[0, 1, 2], [3, 2, 1]], np.uint8)
    keep = np.array([[1, 0, 1], [1, 1, 0]], np.uint8)
    M = oracle.mask(pid, keep, lib)
    Wm = oracle.apply_mask(Wt, M)
    for c in range(C):
        x = np.zeros((1, H, W, C), np.float32)
        x[0, 3, 3, c] = 1.0
        y = oracle.conv_fwd(x, Wm, 1)
        expect = np.zeros((1, H, W, F), np.float32)
        for f in range(F):
            for r in range(3):
                for s in range(3):
                    expect[0, 3 - (r - 1), 3 - (s - 1), f] = Wm[f, c, 3 * r + s]
        assert np.array_equal(y, expect)


def test_single_pattern_is_a_plain_stencil(oracle):
    """P = 1, all kernels kept, C = F = 1: a fixed 4-tap stencil written out by hand."""
    lib = np.array([I.mask_of((1, 3, 4, 5))], np.uint16)     # up, left, centre, right
    Wt = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 9)
    pid, keep = oracle.select(Wt, None, lib, 1)
    Wm = oracle.apply_mask(Wt, oracle.mask(pid, keep, lib))
    x, _ = I.gen_activations((1, 6, 5, 1), 11, "stencil", False, "f32")
    xp = np.pad(x[0, :, :, 0].astype(np.float64), 1)
    expect = 2 * xp[0:6, 1:6] + 4 * xp[1:7, 0:5] + 5 * xp[1:7, 1:6] + 6 * xp[1:7, 2:7]
    y = oracle.conv_fwd(x, Wm, 1)
    np.testing.assert_allclose(y[0, :, :, 0], expect.astype(np.float32), rtol=0, atol=1e-6)


@pytest.mark.parametrize("shape", SHAPES)
def test_adjoint_identities(oracle, shape):
    """<fwd(x;W), dy> = <x, bwd_data(dy;W)> = <W, bwd_weight(x,dy)> on the kept taps."""
    x, dy, Wm, M, *_ = _case(oracle, shape)
    stride = shape[5]
    y = oracle.conv_fwd(x, Wm, stride).astype(np.float64)
    dx = oracle.conv_bwd_data(dy, Wm, x.shape, stride).astype(np.float64)
    dw = oracle.conv_bwd_weight(x, dy, M, stride).astype(np.float64)
    lhs = float((y * dy).sum())
    scale = float(np.abs(y * dy).sum()) + 1e-30
    assert abs(lhs - float((x * dx).sum())) <= 1e-5 * scale
    assert abs(lhs - float((Wm * dw).sum())) <= 1e-5 * scale


@pytest.mark.parametrize("shape", SHAPES[:4])
def test_sampled_variants_agree_with_full(oracle, shape):
    x, dy, Wm, M, *_ = _case(oracle, shape)
    stride = shape[5]
    F = Wm.shape[0]
    y = oracle.conv_fwd(x, Wm, stride)
    dx = oracle.conv_bwd_data(dy, Wm, x.shape, stride)
    dw = oracle.conv_bwd_weight(x, dy, np.ones_like(M), stride)
    idx = np.arange(y.size, dtype=np.int64)
    assert np.array_equal(oracle.conv_fwd_at(x, Wm, stride, idx), y.reshape(-1))
    idx = np.arange(dx.size, dtype=np.int64)
    np.testing.assert_allclose(oracle.conv_bwd_data_at(dy, Wm, x.shape, stride, idx), dx.reshape(-1),
                               rtol=0, atol=1e-6)
    idx = np.arange(dw.size, dtype=np.int64)
    assert np.array_equal(oracle.conv_bwd_weight_at(x, dy, F, stride, idx), dw.reshape(-1))


def test_compact_order_and_gather(oracle):
    F, C, P = 5, 9, 8
    lib = I.make_library(P)
    Wt = I.gen_weights(F, C, 5, "cmp")
    pid, keep = oracle.select(Wt, None, lib, 4)
    sf, sc = oracle.compact_order(pid, keep, P)
    assert sf.size == F * 4
    # filter ascending; within a filter (pattern id, channel) ascending
    keys = [(int(f), int(pid[f, c]), int(c)) for f, c in zip(sf, sc)]
    assert keys == sorted(keys)
    assert sorted(zip(sf.tolist(), sc.tolist())) == sorted(zip(*np.nonzero(keep)))
    comp = oracle.gather_compact(Wt, pid, lib, sf, sc)
    for i, (f, c) in enumerate(zip(sf, sc)):
        taps = [t for t in range(9) if (int(lib[pid[f, c]]) >> t) & 1]
        assert np.array_equal(comp[i], Wt[f, c, taps])


def test_bf16_round_matches_torch(oracle):
    a = I.normal(3, 4, 100000) * np.float32(3.0)
    a[:4] = [0.0, 1.0, 1.00390625, 1.01171875]   # exact, exact, tie -> even (down), tie -> even (up)
    ours = oracle.bf16_round(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, ref)
    assert np.array_equal(I.bf16_bits_to_f32(I.f32_to_bf16_bits(a)), ref)

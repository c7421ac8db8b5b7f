"""CPU oracle for the step between two convolution layers of a chained network (test infrastructure only).

Plain numpy, written from the definitions; it shares no code with the HIP library and imports nothing from it.
Only tests/ may use it.

What it follows (ClickTrain, arXiv 2011.10170): Section 5.2, "Backward Phase Acceleration": the layer output
before the activation is z = a_prev (*) W, the next layer's input is a = sigma(z), and the error that reaches the
previous layer is multiplied elementwise by sigma'(z). The networks of Section 6 (VGG-16 on CIFAR and ImageNet)
use sigma = ReLU and place a 2x2 max pooling of stride 2 between groups of layers, so the step between two
layers is
    forward   a = maxpool_q(relu(z))                    q = 1 (no pooling) or 2
    backward  dz = d a / d z applied to da: the error of a pooled element goes to the window position that
              held the maximum when that maximum is positive, and nowhere otherwise.
Both are exact in any precision (comparisons and copies only), so outputs are compared bit for bit.

Readings where the text is silent: relu(z) = z where z > 0, else +0; a window whose maximum is not positive
passes no error; among equal positive maxima the first position in row-major order of the window (dr, dc) wins
(the subgradient chosen; the forward value does not depend on it); pooling windows do not overlap and an odd
last row / column is dropped (output extent H // 2), its dz is 0. The record kept for the backward pass is one
byte per output element: the window position 2*dr + dc of the maximum, 255 when no error passes.

Pins (tests/test_oracle_chain.py): a hand-worked map with ties and all-negative windows; PyTorch-CPU
`max_pool2d(relu(z))` and its autograd on tie-free inputs of odd and even extents; finite differences of the
forward function; the invariants (at most one nonzero dz per window, sum(dz) = sum of the passed da).
"""
from __future__ import annotations

from typing import Tuple

import numpy as np

NONE = 255


def act_pool_fwd(z: np.ndarray, pool: int) -> Tuple[np.ndarray, np.ndarray]:
    """z [N][H][W][C] -> (a [N][H//pool][W//pool][C] of z's dtype, sel uint8 of a's shape)."""
    assert z.ndim == 4 and pool in (1, 2)
    N, H, W, C = z.shape
    Ho, Wo = H // pool, W // pool
    # window positions in row-major order; np.argmax returns the first maximum
    win = np.stack([z[:, dr:dr + Ho * pool:pool, dc:dc + Wo * pool:pool, :]
                    for dr in range(pool) for dc in range(pool)], axis=0)
    arg = np.argmax(win, axis=0)
    m = np.take_along_axis(win, arg[None], axis=0)[0]
    pos = m > 0
    a = np.where(pos, m, np.zeros((), dtype=z.dtype)).astype(z.dtype)
    sel = np.where(pos, arg, NONE).astype(np.uint8)
    return a, sel


def act_pool_bwd(da: np.ndarray, sel: np.ndarray, H: int, W: int, pool: int) -> np.ndarray:
    """da, sel [N][H//pool][W//pool][C] -> dz [N][H][W][C] of da's dtype."""
    assert da.shape == sel.shape and pool in (1, 2)
    N, Ho, Wo, C = da.shape
    assert Ho == H // pool and Wo == W // pool
    dz = np.zeros((N, H, W, C), dtype=da.dtype)
    for dr in range(pool):
        for dc in range(pool):
            k = dr * pool + dc
            dz[:, dr:dr + Ho * pool:pool, dc:dc + Wo * pool:pool, :] = np.where(sel == k, da, np.zeros((), dtype=da.dtype))
    return dz

"""CPU oracle for the training-side steps next to the convolution path (test infrastructure only).

Plain numpy, written from the method's description; it shares no code with the HIP library and imports
nothing from it. Only tests/ may use it.

What it follows (ClickTrain, arXiv 2011.10170):
  - Section 4.2 "Proposed dynamic pool generation process", steps 1-6: per kernel, the highest-scoring weight
    position, then the best of its 8 neighbours, then the candidate positions (horizontal / vertical neighbours
    of those two, diagonals excluded by the section's "Detailed optimizations"), then the best candidate pattern
    = the two first positions plus the pair of candidate positions with the highest pattern importance
    (Section 4.1, Eq. 1); a global pool counts how often each candidate pattern was produced ("competitive
    score", 1 per occurrence); the final pool is the N patterns with the highest counts.
  - Section 4.3 "Adaptive pattern and kernel finalization": per batch the best pattern of every kernel is
    counted; the final pattern of a kernel is the one counted most often.
  - Section 4.4 "Modified group lasso regularization", Eq. 3 and Eq. 4: Z = W (.) not P (weights outside the
    chosen pattern), U = W (.) not I (all weights of the unimportant kernels); the penalty is
    lambda_P * sum over kernels of ||Z_k||_2 + lambda_I * sum over kernels of ||U_k||_2 with one group per 3x3
    kernel; its gradient is lambda_P * Z_k / ||Z_k|| + lambda_I * U_k / ||U_k|| (0 where the norm is 0).

Discrete outputs (masks, counts, picks) are compared bit-exactly, so the float32 operation order is part of
their definition and is the one of the selection step: importance s_t = (g_t*w_t)*(g_t*w_t) (two rounded
multiplies; s_t = w_t*w_t without gradients), pattern importance ((s_a+s_b)+s_c)+s_d over the pattern's taps in
ascending order, the first maximum wins every arg max (positions in ascending tap index, candidate pairs in
lexicographic order of (lower tap, higher tap), patterns in ascending mask value). The group-lasso gradient is
floating point: computed here in float64.

Readings where the text is silent: ties as above; a pool asked for more patterns than were ever produced
returns only the produced ones; the "competitive score" of a pattern is its number of occurrences.

Pins (tests/test_oracle_train.py): a hand-worked kernel; brute force over all 126 four-tap masks on random
kernels; the count of reachable masks by exhaustive enumeration; histogram totals; finite differences and
PyTorch-CPU autograd of the penalty for the gradient; unit-norm and support invariants. No function is unpinned.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np


def _neighbours(diagonal: bool):
    out = []
    for t in range(9):
        r, s = divmod(t, 3)
        nb = []
        for u in range(9):
            r2, s2 = divmod(u, 3)
            dr, ds = abs(r - r2), abs(s - s2)
            if u == t or dr > 1 or ds > 1:
                continue
            if not diagonal and dr + ds != 1:
                continue
            nb.append(u)
        out.append(nb)
    return out


NB8 = _neighbours(True)     # horizontal, vertical and diagonal neighbours of every position (step 2)
NB4 = _neighbours(False)    # horizontal and vertical neighbours only (step 3)


def tap_scores(W: np.ndarray, G: Optional[np.ndarray]) -> np.ndarray:
    """Importance of every weight, float32 [F][C][9] (Section 4.1: squared first-order Taylor term)."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    if G is None:
        return W * W
    gw = np.ascontiguousarray(G, dtype=np.float32) * W
    return gw * gw


def _ordered_sum(s4: np.ndarray) -> np.ndarray:
    """((s_a + s_b) + s_c) + s_d in float32; s4[..., 0..3] are the importances in ascending tap order."""
    return ((s4[..., 0] + s4[..., 1]) + s4[..., 2]) + s4[..., 3]


def dppg_candidate_masks(W: np.ndarray, G: Optional[np.ndarray]) -> np.ndarray:
    """Steps 1-4 for every kernel: the 9-bit mask (bit t = tap t) of its best candidate pattern, uint16 [F][C]."""
    s = tap_scores(W, G)
    F, C = s.shape[:2]
    s = s.reshape(-1, 9)
    n = s.shape[0]
    rows = np.arange(n)
    t1 = np.argmax(s, axis=1)                                   # step 1 (first maximum)
    nb8 = np.zeros((9, 9), dtype=bool)
    nb4 = np.zeros((9, 9), dtype=bool)
    for t in range(9):
        nb8[t, NB8[t]] = True
        nb4[t, NB4[t]] = True
    s_nb = np.where(nb8[t1], s, np.float32(-np.inf))
    t2 = np.argmax(s_nb, axis=1)                                # step 2
    cand = nb4[t1] | nb4[t2]                                    # step 3
    cand[rows, t1] = False
    cand[rows, t2] = False
    best = np.full(n, -np.inf, dtype=np.float32)
    best_mask = np.zeros(n, dtype=np.uint16)
    for a in range(9):                                          # step 4: every pair of candidate positions
        for b in range(a + 1, 9):
            ok = cand[:, a] & cand[:, b]
            taps = np.sort(np.stack([t1, t2, np.full(n, a), np.full(n, b)], axis=1), axis=1)
            score = _ordered_sum(np.take_along_axis(s, taps, axis=1))
            better = ok & (score > best)
            best = np.where(better, score, best)
            m = ((1 << t1) | (1 << t2) | (1 << a) | (1 << b)).astype(np.uint16)
            best_mask = np.where(better, m, best_mask)
    return best_mask.reshape(F, C)


def dppg_accumulate(hist: np.ndarray, W: np.ndarray, G: Optional[np.ndarray]) -> np.ndarray:
    """Step 4/5: adds one count per kernel to the candidate pool, hist uint32 [512] indexed by mask."""
    masks = dppg_candidate_masks(W, G).reshape(-1)
    out = hist.astype(np.uint32).copy()
    np.add.at(out, masks, 1)
    return out


def dppg_pool(hist: np.ndarray, n_patterns: int) -> Tuple[np.ndarray, np.ndarray]:
    """Step 6: the n_patterns masks with the highest counts (ties: lower mask first) and their counts."""
    order = sorted((m for m in range(512) if hist[m] > 0), key=lambda m: (-int(hist[m]), m))[:n_patterns]
    return np.array(order, dtype=np.uint16), np.array([hist[m] for m in order], dtype=np.uint32)


def finalize_count(counts: np.ndarray, pid: np.ndarray) -> np.ndarray:
    """One batch of Section 4.3: counts[f][c][pid[f][c]] += 1. counts uint32 [F][C][P]."""
    out = counts.astype(np.uint32).copy()
    F, C = pid.shape
    f, c = np.meshgrid(np.arange(F), np.arange(C), indexing="ij")
    out[f, c, pid] += 1
    return out


def finalize_pick(counts: np.ndarray) -> np.ndarray:
    """Most frequent best pattern of every kernel (first maximum), uint8 [F][C]."""
    return np.argmax(counts, axis=2).astype(np.uint8)


def group_lasso_masks(pid: np.ndarray, keep: np.ndarray, lib_masks: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """not P and not I of Eq. 3 as 0/1 tensors [F][C][9]: positions outside the kernel's pattern; unimportant kernels."""
    bits = (np.asarray(lib_masks, dtype=np.int64)[pid.astype(np.int64)][..., None] >> np.arange(9)) & 1
    not_p = (1 - bits).astype(np.float64)
    not_i = np.repeat((keep == 0).astype(np.float64)[..., None], 9, axis=2)
    return not_p, not_i


def group_lasso_penalty(W, pid, keep, lib_masks, lambda_p: float, lambda_i: float) -> float:
    """The two added terms of Eq. 4 for one layer, float64."""
    not_p, not_i = group_lasso_masks(pid, keep, lib_masks)
    W = np.asarray(W, dtype=np.float64)
    z = W * not_p
    u = W * not_i
    return float(lambda_p * np.sqrt((z * z).sum(axis=2)).sum() + lambda_i * np.sqrt((u * u).sum(axis=2)).sum())


def group_lasso_grad(W, pid, keep, lib_masks, lambda_p: float, lambda_i: float) -> np.ndarray:
    """Gradient of the penalty with respect to W, float64 [F][C][9] (0 for a group whose norm is 0)."""
    not_p, not_i = group_lasso_masks(pid, keep, lib_masks)
    W = np.asarray(W, dtype=np.float64)
    out = np.zeros_like(W)
    for mask, lam in ((not_p, lambda_p), (not_i, lambda_i)):
        v = W * mask
        nrm = np.sqrt((v * v).sum(axis=2, keepdims=True))
        safe = np.where(nrm > 0, nrm, 1.0)
        out += lam * np.where(nrm > 0, v / safe, 0.0)
    return out

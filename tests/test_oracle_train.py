"""Pins for oracle/pc_oracle_train.py (pool generation, finalisation counters, modified group lasso).

None of these checks re-uses the oracle's own code path: hand-worked kernels, a brute force over all 126
four-tap masks written with Python sets and loops, exhaustive enumeration of what the construction can reach,
finite differences and PyTorch-CPU autograd of the penalty.
"""
import itertools

import numpy as np
import pytest

from oracle import pc_oracle_train as T
from paper_2011_10170_amd import inputs as I


def _adjacent(t, u, diagonal):
    r, s = divmod(t, 3)
    r2, s2 = divmod(u, 3)
    dr, ds = abs(r - r2), abs(s - s2)
    if t == u or dr > 1 or ds > 1:
        return False
    return diagonal or dr + ds == 1


def test_neighbour_tables():
    # centre: 8 neighbours, 4 without diagonals; corner: 3 and 2; edge: 5 and 3
    assert [len(T.NB8[t]) for t in range(9)] == [3, 5, 3, 5, 8, 5, 3, 5, 3]
    assert [len(T.NB4[t]) for t in range(9)] == [2, 3, 2, 3, 4, 3, 2, 3, 2]
    for t in range(9):
        assert T.NB8[t] == [u for u in range(9) if _adjacent(t, u, True)]
        assert T.NB4[t] == [u for u in range(9) if _adjacent(t, u, False)]


def test_hand_worked_kernels():
    """Section 4.2 steps 1-4 followed by hand.
    Kernel A, importances 1 4 9 / 16 81 25 / 36 49 64 (weights 1..9 with the 9 at the centre): first position the
    centre (4), best neighbour position 8; candidates = {1,3,5,7} (cross of the centre) united with {5,7}; the best
    pair is {5,7}: pattern {4,5,7,8} = 0b110110000.
    Kernel B: first position 0, best neighbour 1, candidates {3} + {2,4}; best pair {2,3}: pattern {0,1,2,3}."""
    W = np.array([[[1, 2, 3, 4, 9, 5, 6, 7, 8]], [[9, 8, 1, 7, 0.5, 0.2, 0.1, 0.3, 0.4]]], dtype=np.float32)
    m = T.dppg_candidate_masks(W, None)
    assert m.tolist() == [[0b110110000], [0b000001111]]
    # with gradients the importance is (g*w)^2: a gradient that zeroes the centre moves the first position
    G = np.ones_like(W)
    G[0, 0, 4] = 0.0
    m2 = T.dppg_candidate_masks(W, G)
    # kernel A now: first 8, best neighbour 7 (49 > 25 > 0), candidates {5,7}->{5} + {4,6,8}->{4,6}: {4,5,6};
    # best pair by importance 36 (6) and 25 (5): pattern {5,6,7,8}
    assert m2[0, 0] == (1 << 5) | (1 << 6) | (1 << 7) | (1 << 8)


def test_reachable_patterns_exhaustive():
    """Every candidate pattern the construction can produce: 44 of the 126 four-tap masks, 32 with the centre."""
    reach = set()
    for t1 in range(9):
        for t2 in range(9):
            if not _adjacent(t1, t2, True):
                continue
            cand = {u for u in range(9) if (_adjacent(t1, u, False) or _adjacent(t2, u, False)) and u not in (t1, t2)}
            assert len(cand) >= 2
            for a, b in itertools.combinations(sorted(cand), 2):
                reach.add((1 << t1) | (1 << t2) | (1 << a) | (1 << b))
    assert len(reach) == 44 and sum(1 for m in reach if m & 16) == 32
    rng = np.random.default_rng(3)
    W = rng.standard_normal((40, 50, 9)).astype(np.float32)
    G = rng.standard_normal((40, 50, 9)).astype(np.float32)
    got = set(int(m) for m in T.dppg_candidate_masks(W, G).reshape(-1))
    assert got <= reach
    assert len(got) == 44          # 2000 random kernels reach every one of them
    # the 12-pattern benchmark pool consists of masks the construction can produce
    from paper_2011_10170_amd import inputs as I
    assert all(int(m) in reach for m in I.make_library(12))


def test_candidate_masks_against_brute_force():
    rng = np.random.default_rng(11)
    W = rng.standard_normal((6, 7, 9)).astype(np.float32)
    G = rng.standard_normal((6, 7, 9)).astype(np.float32)
    got = T.dppg_candidate_masks(W, G)
    for f in range(6):
        for c in range(7):
            s = [np.float32(np.float32(G[f, c, t] * W[f, c, t]) * np.float32(G[f, c, t] * W[f, c, t])) for t in range(9)]
            t1 = max(range(9), key=lambda t: (s[t], -t))
            t2 = max((u for u in range(9) if _adjacent(t1, u, True)), key=lambda t: (s[t], -t))
            cand = {u for u in range(9) if (_adjacent(t1, u, False) or _adjacent(t2, u, False)) and u not in (t1, t2)}
            best, best_m = None, None
            for taps in itertools.combinations(range(9), 4):          # all 126 masks
                if t1 not in taps or t2 not in taps:
                    continue
                if not set(taps) - {t1, t2} <= cand:
                    continue
                a, b, c2, d = taps
                score = np.float32(np.float32(np.float32(s[a] + s[b]) + s[c2]) + s[d])
                if best is None or score > best:
                    best, best_m = score, sum(1 << t for t in taps)
            assert got[f, c] == best_m
            assert bin(int(got[f, c])).count("1") == 4 and (got[f, c] >> t1) & 1 and (got[f, c] >> t2) & 1


def test_pool_counts_and_order():
    rng = np.random.default_rng(5)
    hist = np.zeros(512, dtype=np.uint32)
    total = 0
    for it in range(3):                                   # step 5: repeated accumulation
        W = rng.standard_normal((8, 16, 9)).astype(np.float32)
        G = rng.standard_normal((8, 16, 9)).astype(np.float32)
        hist = T.dppg_accumulate(hist, W, G)
        total += 8 * 16
    assert int(hist.sum()) == total                        # one count per kernel per round
    pool, counts = T.dppg_pool(hist, 8)
    assert len(pool) == 8 and len(set(pool.tolist())) == 8
    assert all(counts[i] >= counts[i + 1] for i in range(7))
    assert int(counts[-1]) >= max(int(hist[m]) for m in range(512) if m not in set(pool.tolist()))
    # ties go to the lower mask; fewer produced patterns than asked: only those
    h = np.zeros(512, dtype=np.uint32)
    h[[15, 23, 432]] = [2, 2, 5]
    assert T.dppg_pool(h, 2)[0].tolist() == [432, 15]
    assert T.dppg_pool(h, 8)[0].tolist() == [432, 15, 23]


def test_finalisation_counters():
    P = 5
    counts = np.zeros((2, 3, P), dtype=np.uint32)
    seq = [np.array([[0, 1, 2], [3, 4, 0]]), np.array([[0, 2, 2], [3, 1, 0]]), np.array([[1, 2, 3], [4, 1, 0]])]
    for pid in seq:
        counts = T.finalize_count(counts, pid.astype(np.uint8))
    assert int(counts.sum()) == 3 * 6
    # kernel (0,1) saw 1,2,2 -> 2; kernel (1,1) saw 4,1,1 -> 1; kernel (0,2) saw 2,2,3 -> 2; (1,0) saw 3,3,4 -> 3
    assert T.finalize_pick(counts).tolist() == [[0, 2, 2], [3, 1, 0]]
    # a tie keeps the lower pattern id
    tie = np.zeros((1, 1, P), dtype=np.uint32)
    tie[0, 0, [1, 3]] = 2
    assert T.finalize_pick(tie)[0, 0] == 1


def _case(seed, F=5, C=6, P=8):
    rng = np.random.default_rng(seed)
    lib = I.make_library(P)
    W = rng.standard_normal((F, C, 9))
    pid = rng.integers(0, P, size=(F, C)).astype(np.uint8)
    keep = (rng.random((F, C)) < 0.5).astype(np.uint8)
    return W, pid, keep, lib


def test_group_lasso_gradient_finite_differences():
    W, pid, keep, lib = _case(1)
    lp, li = 0.3, 0.7
    g = T.group_lasso_grad(W, pid, keep, lib, lp, li)
    eps = 1e-6
    rng = np.random.default_rng(2)
    for _ in range(40):
        f, c, t = rng.integers(0, 5), rng.integers(0, 6), rng.integers(0, 9)
        Wp, Wm = W.copy(), W.copy()
        Wp[f, c, t] += eps
        Wm[f, c, t] -= eps
        fd = (T.group_lasso_penalty(Wp, pid, keep, lib, lp, li) - T.group_lasso_penalty(Wm, pid, keep, lib, lp, li)) / (2 * eps)
        assert abs(fd - g[f, c, t]) < 1e-6


def test_group_lasso_gradient_autograd():
    torch = pytest.importorskip("torch")
    W, pid, keep, lib = _case(4)
    lp, li = 1.25, 0.5
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    bits = torch.tensor([[[(int(lib[pid[f, c]]) >> t) & 1 for t in range(9)] for c in range(6)] for f in range(5)],
                        dtype=torch.float64)
    # the kernel term is summed over the unimportant kernels only: a group that is identically zero has no
    # derivative at 0 in autograd (the method's subgradient there is 0)
    unimportant = torch.tensor(keep == 0)
    pen = lp * (Wt * (1 - bits)).pow(2).sum(dim=2).sqrt().sum() + li * Wt[unimportant].pow(2).sum(dim=1).sqrt().sum()
    pen.backward()
    assert abs(float(pen.detach()) - T.group_lasso_penalty(W, pid, keep, lib, lp, li)) < 1e-9
    assert np.allclose(Wt.grad.numpy(), T.group_lasso_grad(W, pid, keep, lib, lp, li), atol=1e-12)


def test_group_lasso_invariants():
    W, pid, keep, lib = _case(9)
    lp, li = 0.2, 0.9
    g = T.group_lasso_grad(W, pid, keep, lib, lp, li)
    not_p, not_i = T.group_lasso_masks(pid, keep, lib)
    # weights inside the pattern of an important kernel are not penalised
    assert not g[(not_p == 0) & (not_i == 0)].any()
    # the pattern term alone has norm lambda_P in every kernel, the kernel term norm lambda_I in unimportant ones
    gp = T.group_lasso_grad(W, pid, keep, lib, lp, 0.0)
    gi = T.group_lasso_grad(W, pid, keep, lib, 0.0, li)
    assert np.allclose(np.sqrt((gp * gp).sum(axis=2)), lp)
    assert np.allclose(np.sqrt((gi * gi).sum(axis=2)), li * (keep == 0))
    assert np.allclose(gp + gi, g)
    # positive scaling of the weights leaves the gradient unchanged (the norm is 1-homogeneous)
    assert np.allclose(T.group_lasso_grad(3.5 * W, pid, keep, lib, lp, li), g)
    # zero groups have zero gradient, not NaN
    Wz = W.copy()
    Wz[0, 0] = 0.0
    assert np.isfinite(T.group_lasso_grad(Wz, pid, keep, lib, lp, li)).all()
    assert not T.group_lasso_grad(Wz, pid, keep, lib, lp, li)[0, 0].any()

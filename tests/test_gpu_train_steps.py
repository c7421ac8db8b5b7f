"""GPU parity of the training-side steps (pool generation, finalisation counters, modified group lasso) against
oracle/pc_oracle_train.py, through the C ABI. Masks, counts and picks are compared bit-exactly; the group-lasso
gradient (float32 on the GPU, float64 in the oracle) to a relative L2 error of 1e-6: every element is a few
correctly rounded float32 operations (9 squares and additions, one square root, one division, one product),
i.e. a relative error of a few 2^-24."""
import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests._harness import rel_l2, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2011_10170_amd import binding
    binding.load()
    return binding


@pytest.fixture(scope="module")
def ctx(B):
    import torch
    c = B.pc_create(0, torch.cuda.current_stream().cuda_stream)
    yield c
    B.pc_destroy(c)


@pytest.fixture(scope="module")
def T():
    from oracle import pc_oracle_train
    return pc_oracle_train


SHAPES = [(1, 1), (3, 5), (29, 37), (64, 64), (130, 257), (512, 512)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("with_grad", [True, False])
def test_pool_generation_bit_exact(B, ctx, T, shape, with_grad):
    import torch
    F, C = shape
    Wn = I.gen_weights(F, C, I.BASE_SEED, ("dppg", shape))
    Gn = I.gen_weight_grads(F, C, I.BASE_SEED, ("dppg", shape)) if with_grad else None
    ref_masks = T.dppg_candidate_masks(Wn, Gn)
    hist = torch.zeros(512, dtype=torch.int32, device="cuda")
    masks = torch.full((F, C), -1, dtype=torch.int16, device="cuda")
    Wd = to_dev(Wn)
    Gd = to_dev(Gn) if with_grad else None
    ref_hist = np.zeros(512, dtype=np.uint32)
    for rounds in range(2):                                  # the pool accumulates over calls
        B.pc_dppg_accumulate(ctx, Wd, Gd, F, C, hist, masks)
        ref_hist = T.dppg_accumulate(ref_hist, Wn, Gn)
    torch.cuda.synchronize()
    assert np.array_equal(masks.cpu().numpy().view(np.uint16), ref_masks)
    assert np.array_equal(hist.cpu().numpy().view(np.uint32), ref_hist)
    for n in (4, 8, 12, 126):
        pool, scores = B.pc_dppg_pool(ctx, hist, n)
        rp, rs = T.dppg_pool(ref_hist, n)
        assert pool == rp.tolist() and scores == rs.tolist()
    # without the per-kernel output the counts are the same
    hist2 = torch.zeros(512, dtype=torch.int32, device="cuda")
    B.pc_dppg_accumulate(ctx, Wd, Gd, F, C, hist2, None)
    B.pc_dppg_accumulate(ctx, Wd, Gd, F, C, hist2, None)
    torch.cuda.synchronize()
    assert torch.equal(hist2, hist)


def test_pool_generation_ties_and_zero_weights(B, ctx, T):
    """Quantised weights: equal importances everywhere, so every arg max falls back to its tie rule."""
    import torch
    rng = np.random.default_rng(21)
    F, C = 17, 300
    for lo, hi in ((0, 1), (-1, 2), (-2, 3)):
        Wn = rng.integers(lo, hi, size=(F, C, 9)).astype(np.float32)
        Gn = rng.integers(-1, 2, size=(F, C, 9)).astype(np.float32)
        masks = torch.full((F, C), -1, dtype=torch.int16, device="cuda")
        hist = torch.zeros(512, dtype=torch.int32, device="cuda")
        B.pc_dppg_accumulate(ctx, to_dev(Wn), to_dev(Gn), F, C, hist, masks)
        torch.cuda.synchronize()
        assert np.array_equal(masks.cpu().numpy().view(np.uint16), T.dppg_candidate_masks(Wn, Gn))
        assert int(hist.sum().item()) == F * C


@pytest.mark.parametrize("shape,P", [((3, 5), 4), ((29, 37), 12), ((64, 300), 16), ((7, 9), 126)])
def test_finalisation_counters_bit_exact(B, ctx, T, shape, P):
    import torch
    F, C = shape
    rng = np.random.default_rng(31)
    counts = torch.zeros((F, C, P), dtype=torch.int32, device="cuda")
    ref = np.zeros((F, C, P), dtype=np.uint32)
    for batch in range(5):
        pid = rng.integers(0, min(P, 3 + batch), size=(F, C)).astype(np.uint8)
        B.pc_finalize_count(ctx, to_dev(pid), F, C, P, counts)
        ref = T.finalize_count(ref, pid)
    pick = torch.full((F, C), 255, dtype=torch.uint8, device="cuda")
    B.pc_finalize_pick(ctx, counts, F, C, P, pick)
    torch.cuda.synchronize()
    assert np.array_equal(counts.cpu().numpy().view(np.uint32), ref)
    assert np.array_equal(pick.cpu().numpy(), T.finalize_pick(ref))


def test_finalisation_follows_selection(B, ctx, T):
    """Counters fed by pc_pattern_select over batches with changing gradients, as in Section 4.3."""
    import torch
    from oracle import pc_oracle as oracle
    F, C, P = 24, 40, 8
    lib = I.make_library(P)
    Wn = I.gen_weights(F, C, I.BASE_SEED, "fin")
    Wd = to_dev(Wn)
    counts = torch.zeros((F, C, P), dtype=torch.int32, device="cuda")
    ref = np.zeros((F, C, P), dtype=np.uint32)
    pid = torch.empty((F, C), dtype=torch.uint8, device="cuda")
    keep = torch.empty((F, C), dtype=torch.uint8, device="cuda")
    for batch in range(4):
        Gn = I.gen_weight_grads(F, C, I.BASE_SEED, ("fin", batch))
        B.pc_pattern_select(ctx, Wd, to_dev(Gn), F, C, lib, 0, C, 0, pid, keep)
        B.pc_finalize_count(ctx, pid, F, C, P, counts)
        ref = T.finalize_count(ref, oracle.select(Wn, Gn, lib, C)[0])
    final = torch.empty((F, C), dtype=torch.uint8, device="cuda")
    B.pc_finalize_pick(ctx, counts, F, C, P, final)
    torch.cuda.synchronize()
    assert np.array_equal(final.cpu().numpy(), T.finalize_pick(ref))


@pytest.mark.parametrize("shape,P", [((1, 1), 4), ((3, 5), 8), ((29, 37), 12), ((130, 257), 16), ((512, 512), 8)])
def test_group_lasso_gradient(B, ctx, T, shape, P):
    import torch
    F, C = shape
    lib = I.make_library(P)
    rng = np.random.default_rng(41)
    Wn = I.gen_weights(F, C, I.BASE_SEED, ("gl", shape))
    pid = rng.integers(0, P, size=(F, C)).astype(np.uint8)
    keep = (rng.random((F, C)) < 0.4).astype(np.uint8)
    dW0 = rng.standard_normal((F, C, 9)).astype(np.float32)
    lp, li = 0.37, 1.6
    ref = dW0.astype(np.float64) + T.group_lasso_grad(Wn, pid, keep, lib, lp, li)
    ref_pen = T.group_lasso_penalty(Wn, pid, keep, lib, np.float32(lp), np.float32(li))
    dW = to_dev(dW0.copy())
    pen = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    B.pc_group_lasso_grad(ctx, to_dev(Wn), to_dev(pid), to_dev(keep), F, C, lib, lp, li, dW, pen)
    torch.cuda.synchronize()
    got = dW.cpu().numpy()
    assert rel_l2(got, ref) <= 1e-6
    assert abs(float(pen.item()) - ref_pen) <= 1e-6 * abs(ref_pen)
    # the added part alone, and where it must be zero: inside the pattern of an important kernel
    add = got.astype(np.float64) - dW0
    not_p, not_i = T.group_lasso_masks(pid, keep, lib)
    assert not add[(not_p == 0) & (not_i == 0)].any()
    assert rel_l2(add, T.group_lasso_grad(Wn, pid, keep, lib, lp, li)) <= 1e-5   # (cancellation against dW0 costs a digit)
    # without the penalty output, and run twice: identical bits
    dW2 = to_dev(dW0.copy())
    B.pc_group_lasso_grad(ctx, to_dev(Wn), to_dev(pid), to_dev(keep), F, C, lib, lp, li, dW2, None)
    torch.cuda.synchronize()
    assert np.array_equal(dW2.cpu().numpy(), got)


def test_group_lasso_zero_groups(B, ctx, T):
    """Kernels that are identically zero, and hard-pruned kernels (zero outside the pattern), add nothing: no NaN."""
    import torch
    F, C, P = 4, 6, 8
    lib = I.make_library(P)
    Wn = I.gen_weights(F, C, I.BASE_SEED, "glz")
    pid = np.zeros((F, C), dtype=np.uint8)
    keep = np.ones((F, C), dtype=np.uint8)
    keep[1] = 0
    Wn[0] = 0.0
    Wn[1, :3] = 0.0
    for t in range(9):
        if not (int(lib[0]) >> t) & 1:
            Wn[2, :, t] = 0.0                                # filter 2 is already hard-pruned to pattern 0
    dW = torch.zeros((F, C, 9), dtype=torch.float32, device="cuda")
    B.pc_group_lasso_grad(ctx, to_dev(Wn), to_dev(pid), to_dev(keep), F, C, lib, 0.5, 0.25, dW, None)
    torch.cuda.synchronize()
    got = dW.cpu().numpy()
    assert np.isfinite(got).all()
    assert not got[0].any() and not got[1, :3].any() and not got[2].any()
    assert rel_l2(got, T.group_lasso_grad(Wn, pid, keep, lib, 0.5, 0.25)) <= 1e-6


def test_batch_calls_equal_the_oracle_layer_by_layer(B, ctx, T):
    """The training-side steps over 35 layers of mixed sizes in one call each (more than one launch takes): masks,
    pool counts, finalisation counts and picks bit-exact, the group-lasso gradient and its total penalty within the
    single call's tolerance."""
    import torch
    rng = np.random.default_rng(51)
    P = 8
    lib = I.make_library(P)
    shapes = [(int(rng.integers(1, 50)), int(rng.integers(1, 90))) for _ in range(33)] + [(130, 257), (64, 64)]
    Ws = [I.gen_weights(F, C, I.BASE_SEED, ("tsb", i)) for i, (F, C) in enumerate(shapes)]
    Gs = [I.gen_weight_grads(F, C, I.BASE_SEED, ("tsb", i)) for i, (F, C) in enumerate(shapes)]
    Fs, Cs = [f for f, _ in shapes], [c for _, c in shapes]
    Wd, Gd = [to_dev(w) for w in Ws], [to_dev(g) for g in Gs]
    Gd[3] = None
    # pool generation
    hist = torch.zeros(512, dtype=torch.int32, device="cuda")
    masks = [torch.full((F, C), -1, dtype=torch.int16, device="cuda") for F, C in shapes]
    B.pc_dppg_accumulate_batch(ctx, Wd, Gd, Fs, Cs, hist, masks)
    torch.cuda.synchronize()
    ref_hist = np.zeros(512, dtype=np.uint32)
    for i, (w, g) in enumerate(zip(Ws, Gs)):
        gg = None if i == 3 else g
        assert np.array_equal(masks[i].cpu().numpy().view(np.uint16), T.dppg_candidate_masks(w, gg)), i
        ref_hist = T.dppg_accumulate(ref_hist, w, gg)
    assert np.array_equal(hist.cpu().numpy().view(np.uint32), ref_hist)
    hist2 = torch.zeros(512, dtype=torch.int32, device="cuda")
    B.pc_dppg_accumulate_batch(ctx, Wd, Gd, Fs, Cs, hist2, None)
    torch.cuda.synchronize()
    assert torch.equal(hist2, hist)
    # finalisation counters over three batches, then the pick
    counts = [torch.zeros((F, C, P), dtype=torch.int32, device="cuda") for F, C in shapes]
    ref_counts = [np.zeros((F, C, P), dtype=np.uint32) for F, C in shapes]
    for batch in range(3):
        pids = [rng.integers(0, min(P, 3 + batch), size=(F, C)).astype(np.uint8) for F, C in shapes]
        B.pc_finalize_count_batch(ctx, [to_dev(p) for p in pids], Fs, Cs, P, counts)
        ref_counts = [T.finalize_count(r, p) for r, p in zip(ref_counts, pids)]
    picks = [torch.full((F, C), 255, dtype=torch.uint8, device="cuda") for F, C in shapes]
    B.pc_finalize_pick_batch(ctx, counts, Fs, Cs, P, picks)
    torch.cuda.synchronize()
    for i in range(len(shapes)):
        assert np.array_equal(counts[i].cpu().numpy().view(np.uint32), ref_counts[i]), i
        assert np.array_equal(picks[i].cpu().numpy(), T.finalize_pick(ref_counts[i])), i
    # group lasso: 32 layers with the penalty, all 35 without
    pid_h = [rng.integers(0, P, size=(F, C)).astype(np.uint8) for F, C in shapes]
    keep_h = [(rng.random((F, C)) < 0.4).astype(np.uint8) for F, C in shapes]
    dW0 = [rng.standard_normal((F, C, 9)).astype(np.float32) for F, C in shapes]
    lp, li = 0.37, 1.6
    pd, kd = [to_dev(p) for p in pid_h], [to_dev(k) for k in keep_h]
    dW = [to_dev(d.copy()) for d in dW0]
    pen = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    sel = list(range(3, 35))
    pick = lambda xs: [xs[i] for i in sel]
    B.pc_group_lasso_grad_batch(ctx, pick(Wd), pick(pd), pick(kd), pick(Fs), pick(Cs), lib, lp, li, pick(dW), pen)
    torch.cuda.synchronize()
    ref_pen = 0.0
    for i in sel:
        ref = dW0[i].astype(np.float64) + T.group_lasso_grad(Ws[i], pid_h[i], keep_h[i], lib, lp, li)
        assert rel_l2(dW[i].cpu().numpy(), ref) <= 1e-6, i
        ref_pen += T.group_lasso_penalty(Ws[i], pid_h[i], keep_h[i], lib, np.float32(lp), np.float32(li))
    assert abs(float(pen.item()) - ref_pen) <= 1e-6 * abs(ref_pen)
    dW2 = [to_dev(d.copy()) for d in dW0]
    B.pc_group_lasso_grad_batch(ctx, Wd, pd, kd, Fs, Cs, lib, lp, li, dW2, None)
    torch.cuda.synchronize()
    for i in sel:
        assert torch.equal(dW2[i], dW[i]), i
    with pytest.raises(B.PcError):
        B.pc_group_lasso_grad_batch(ctx, Wd, pd, kd, Fs, Cs, lib, lp, li, dW2, pen)     # 35 layers with a penalty


def test_argument_checks(B, ctx):
    import torch
    t = torch.zeros(512, dtype=torch.int32, device="cuda")
    with pytest.raises(B.PcError):
        B.pc_dppg_accumulate(ctx, None, None, 4, 4, t)
    with pytest.raises(B.PcError):
        B.pc_dppg_pool(ctx, t, 0)
    with pytest.raises(B.PcError):
        B.pc_finalize_count(ctx, t, 4, 4, 127, t)
    with pytest.raises(B.PcError):
        B.pc_group_lasso_grad(ctx, t, t, t, 4, 4, [15, 15], 0.1, 0.1, t)

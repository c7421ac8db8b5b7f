"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (default kernel choice). The oracle cannot run these layers in full, so selection is compared in
full (bit-exact) and the three passes on sampled outputs the oracle computes one by one, each held to its
own per-element bound: a stratified sample (one output in every stratum of one image row x 16 to 32 pixels x 16
to 32 channels, so every accumulator tile of every kernel tile is touched) plus image corners and edges; for
the weight gradient one kept tap in every 32 x 32 block of (filter, channel). Activations larger than
inputs.PERIOD repeat cyclically (generation time); weights are always fully generated."""
import sys

import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests._harness import Case, GpuLayer, assert_close, oracle_masks, stratified_indices, TOL_L2, TOL_L2_DW

pytestmark = pytest.mark.gpu

N_WSAMPLES = 192


def _unique_layers():
    out = []
    for name in I.WORKLOAD_ORDER[1:]:
        wl = I.WORKLOADS[name]
        seen = set()
        for li, L in enumerate(wl.layers):
            if L in seen:
                continue
            seen.add(L)
            out.append(pytest.param(name, li, id="%s-L%d-%dx%d-%dto%d-s%d" % (name, li, L.H, L.W, L.C, L.F, L.stride)))
    return out


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2011_10170_amd import binding
    binding.load()
    return binding


@pytest.fixture(scope="module")
def ctx(B):
    import torch
    c = B.pc_create(0, torch.cuda.current_stream().cuda_stream)
    yield c
    B.pc_destroy(c)


def _border_pixels(N, H, W, CH, rng):
    """Flat NHWC indices at corners and edge midpoints of a few images, a few channels each."""
    ys = sorted({0, H // 2, H - 1})
    xs = sorted({0, W // 2, W - 1})
    out = []
    for n in sorted({0, N // 2, N - 1}):
        for y in ys:
            for x in xs:
                for ch in rng.integers(0, CH, size=3):
                    out.append(((n * H + y) * W + x) * CH + int(ch))
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("name,li", _unique_layers())
def test_full_size_layer(B, ctx, oracle, name, li):
    wl = I.WORKLOADS[name]
    L = wl.layers[li]
    print("full-size", name, li, L, flush=True)
    sys.stdout.flush()
    _check_layer_sampled(B, ctx, oracle, L, wl.dtype, wl.P, wl.keep, ("full", name, li), 1000 + li)


@pytest.mark.timeout(600)
def test_tensors_beyond_2_gib(B, ctx, oracle):
    """An activation tensor of more than 2^31 bytes: the kernels that address through 32-bit buffer offsets step
    aside and the passes run on the kernels with 64-bit addressing. Sampled outputs include the last image."""
    L = I.Layer(5, 1024, 1024, 256, 8, 1)
    assert L.N * L.H * L.W * L.C * 2 > (1 << 31)
    print("beyond 2 GiB", L, flush=True)
    _check_layer_sampled(B, ctx, oracle, L, "bf16", 8, 0.3, ("huge",), 77)


def sample_kept_taps(oracle, case, pid, kp, rng, n_random=N_WSAMPLES):
    """Kept taps to compare: one in every 32 x 32 block of (filter, channel) that holds a kept kernel, plus
    n_random anywhere. Returns (flat [F][C][9] indices, compact slots, entry 0..3 of the slot)."""
    L = case.layer
    sf, sc = oracle.compact_order(pid, kp, case.P)
    nnzk = sf.size
    block = (sf.astype(np.int64) // 32) * ((L.C + 31) // 32) + sc.astype(np.int64) // 32
    perm = rng.permutation(nnzk)
    _, first = np.unique(block[perm], return_index=True)
    slots = np.concatenate([perm[first], rng.integers(0, nnzk, size=n_random)])
    js = rng.integers(0, 4, size=slots.size)
    widx = np.empty(slots.size, dtype=np.int64)
    for i, (s_, j) in enumerate(zip(slots, js)):
        f, c = int(sf[s_]), int(sc[s_])
        taps = [t for t in range(9) if (int(case.lib[pid[f, c]]) >> t) & 1]
        widx[i] = (f * L.C + c) * 9 + taps[int(j)]
    return widx, slots, js


def _check_layer_sampled(B, ctx, oracle, L, dtype, P, keep, tag, seed):
    rng = np.random.default_rng(seed)
    case = Case(L, dtype, P, I.kept_per_filter(keep, L.C), tag=tag)
    pid, kp, M, Wm = oracle_masks(oracle, case)
    g = GpuLayer(B, ctx, case)
    try:
        assert g.variant == B.PC_VARIANT_MFMA
        gpid, gkeep = g.masks()
        assert np.array_equal(gpid, pid) and np.array_equal(gkeep, kp)
        assert g.nnzk == int(kp.sum()) == L.F * I.kept_per_filter(keep, L.C)
        assert np.array_equal(g.unpack(), Wm)

        aW, ady = np.abs(Wm), np.abs(case.dy)       # x is non-negative already
        y = g.fwd().reshape(-1)
        idx = np.concatenate([stratified_indices((L.N, L.Ho, L.Wo, L.F), rng), _border_pixels(L.N, L.Ho, L.Wo, L.F, rng)])
        assert_close(y[idx], oracle.conv_fwd_at(case.x, Wm, L.stride, idx), oracle.conv_fwd_at(case.x, aW, L.stride, idx),
                     dtype, TOL_L2[dtype], "fwd, %d samples" % idx.size)
        del y

        dx = g.bwd_data().reshape(-1)
        idx = np.concatenate([stratified_indices((L.N, L.H, L.W, L.C), rng), _border_pixels(L.N, L.H, L.W, L.C, rng)])
        assert_close(dx[idx], oracle.conv_bwd_data_at(case.dy, Wm, case.x.shape, L.stride, idx),
                     oracle.conv_bwd_data_at(ady, aW, case.x.shape, L.stride, idx), dtype, TOL_L2[dtype],
                     "bwd_data, %d samples" % idx.size)
        del dx

        dw, guard = g.bwd_weight()
        widx, slots, js = sample_kept_taps(oracle, case, pid, kp, rng)
        assert_close(dw[slots, js], oracle.conv_bwd_weight_at(case.x, case.dy, L.F, L.stride, widx),
                     oracle.conv_bwd_weight_at(case.x, ady, L.F, L.stride, widx), "f32", TOL_L2_DW,
                     "bwd_weight, %d samples" % widx.size)
        # nothing is written at pruned positions
        dense = g.scatter(guard.body)
        assert np.all(dense[M == 0] == 0.0)
    finally:
        g.close()

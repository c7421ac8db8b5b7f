"""GPU parity on seeded random layer shapes with the automatic kernel choice: ragged batch sizes, 1-pixel and odd
maps, channel counts that are no multiple of a tile (3, 24, 40, 72, 320, ...), both strides, both dtypes, pools of
4 to 16 patterns, keep ratios from 0.1 to 1. Masks bit-exact; forward and backward-data on sampled outputs the
oracle computes one by one; backward-weight in full."""
import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests._harness import Case, GpuLayer, assert_close, oracle_masks, TOL_L2, TOL_L2_DW

pytestmark = pytest.mark.gpu


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


def _draw(rng, big):
    N = int(rng.choice([1, 2, 3, 5, 8, 13, 16, 32] + ([48, 64] if big else [])))
    H = int(rng.choice([1, 2, 3, 4, 7, 8, 9, 14, 16, 20, 28] + ([40, 56] if big else [])))
    W = int(rng.choice([1, 2, 4, 5, 8, 12, 16, 17, 28, 33] + ([47, 56, 64] if big else [])))
    C = int(rng.choice([3, 8, 16, 24, 32, 40, 64, 72, 96, 128, 192, 256, 320] + ([384, 512] if big else [])))
    F = int(rng.choice([4, 8, 16, 24, 32, 64, 72, 128, 160, 256] + ([384, 512] if big else [])))
    stride = int(rng.choice([1, 1, 1, 2]))
    return N, H, W, C, F, stride


@pytest.mark.parametrize("seed,big", [(101, False), (102, False), (103, True)])
def test_random_layers(B, ctx, oracle, seed, big):
    rng = np.random.default_rng(seed)
    done = 0
    while done < (25 if big else 40):
        N, H, W, C, F, stride = _draw(rng, big)
        if N * H * W * C * F > (4e9 if big else 6e8):
            continue
        P = int(rng.choice([4, 8, 12, 16]))
        keep = float(rng.choice([0.1, 0.3, 0.5, 1.0]))
        dtype = str(rng.choice(["bf16", "bf16", "f32"])) if not big else "bf16"
        layer = I.Layer(N, H, W, C, F, stride)
        case = Case(layer, dtype, P, I.kept_per_filter(keep, C), tag=("random", seed, done))
        print("random case", seed, done, (N, H, W, C, F, stride), "P", P, "keep", keep, dtype, flush=True)
        pid, kp, M, Wm = oracle_masks(oracle, case)
        g = GpuLayer(B, ctx, case)
        try:
            gpid, gkeep = g.masks()
            assert np.array_equal(gpid, pid) and np.array_equal(gkeep, kp)
            tol = TOL_L2[dtype]
            aW, ady = np.abs(Wm), np.abs(case.dy)       # x is non-negative already
            y = g.fwd().reshape(-1)
            idx = rng.integers(0, y.size, size=min(4000, y.size))
            assert_close(y[idx], oracle.conv_fwd_at(case.x, Wm, stride, idx), oracle.conv_fwd_at(case.x, aW, stride, idx),
                         dtype, tol, "fwd")
            dx = g.bwd_data().reshape(-1)
            idx = rng.integers(0, dx.size, size=min(4000, dx.size))
            assert_close(dx[idx], oracle.conv_bwd_data_at(case.dy, Wm, case.x.shape, stride, idx),
                         oracle.conv_bwd_data_at(ady, aW, case.x.shape, stride, idx), dtype, tol, "bwd_data")
            dw, guard = g.bwd_weight()
            dense = g.scatter(guard.body)
            assert np.all(dense[M == 0] == 0.0)
            assert_close(dense, oracle.conv_bwd_weight(case.x, case.dy, M, stride), oracle.conv_bwd_weight(case.x, ady, M, stride),
                         "f32", TOL_L2_DW, "bwd_weight")
        finally:
            g.close()
        done += 1

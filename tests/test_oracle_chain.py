"""Pins of oracle/pc_oracle_chain.py (ReLU + max pooling between two layers, Section 5.2's sigma and sigma') against
things other than itself: a hand-worked map, PyTorch-CPU pooling and autograd, finite differences, invariants."""
import numpy as np
import pytest

from oracle import pc_oracle_chain as T


def test_hand_worked_map():
    # one image, 4x5 map (odd width: the last column is dropped), one channel
    z = np.array([[1.0, 3.0, -1.0, -2.0, 9.0],
                  [2.0, 3.0, -4.0, -0.5, 9.0],
                  [0.0, -1.0, 5.0, 5.0, 9.0],
                  [-2.0, 0.0, 5.0, 7.0, 9.0]], dtype=np.float32).reshape(1, 4, 5, 1)
    a, sel = T.act_pool_fwd(z, 2)
    # windows: {1,3,2,3} -> 3, first of the two 3s is position 1; {-1,-2,-4,-.5} -> nothing passes;
    #          {0,-1,-2,0} -> maximum 0 is not positive; {5,5,5,7} -> 7 at position 3
    assert a.reshape(2, 2).tolist() == [[3.0, 0.0], [0.0, 7.0]]
    assert sel.reshape(2, 2).tolist() == [[1, 255], [255, 3]]
    da = np.array([[10.0, 20.0], [30.0, 40.0]], dtype=np.float32).reshape(1, 2, 2, 1)
    dz = T.act_pool_bwd(da, sel, 4, 5, 2).reshape(4, 5)
    want = np.zeros((4, 5), dtype=np.float32)
    want[0, 1] = 10.0
    want[3, 3] = 40.0
    assert np.array_equal(dz, want)
    # without pooling: plain ReLU and its derivative
    a1, s1 = T.act_pool_fwd(z, 1)
    assert np.array_equal(a1, np.maximum(z, 0)) and not np.signbit(a1).any()
    assert np.array_equal(s1 == 0, z > 0) and set(np.unique(s1)) <= {0, 255}
    d1 = T.act_pool_bwd(np.full_like(z, 2.0), s1, 4, 5, 1)
    assert np.array_equal(d1, np.where(z > 0, 2.0, 0.0).astype(np.float32))


def test_all_equal_positive_window_takes_first_position():
    z = np.full((1, 2, 2, 3), 4.0, dtype=np.float32)
    a, sel = T.act_pool_fwd(z, 2)
    assert (a == 4.0).all() and (sel == 0).all()


@pytest.mark.parametrize("shape", [(2, 4, 4, 3), (1, 7, 5, 4), (3, 2, 9, 1), (2, 6, 6, 8)])
@pytest.mark.parametrize("pool", [1, 2])
def test_against_torch_pooling_and_autograd(shape, pool):
    import torch
    import torch.nn.functional as Fn
    rng = np.random.default_rng(5)
    z = rng.standard_normal(shape)                                   # float64: no ties
    a, sel = T.act_pool_fwd(z, pool)
    da = rng.standard_normal(a.shape)
    dz = T.act_pool_bwd(da, sel, shape[1], shape[2], pool)
    zt = torch.from_numpy(z).permute(0, 3, 1, 2).clone().requires_grad_(True)     # NCHW for torch
    at = Fn.relu(zt)
    if pool == 2:
        at = Fn.max_pool2d(at, 2)
    assert np.array_equal(at.detach().permute(0, 2, 3, 1).numpy(), a)
    at.backward(torch.from_numpy(da).permute(0, 3, 1, 2))
    assert np.array_equal(zt.grad.permute(0, 2, 3, 1).numpy(), dz)


def test_finite_differences_and_invariants():
    rng = np.random.default_rng(6)
    z = rng.standard_normal((2, 6, 4, 3))
    a, sel = T.act_pool_fwd(z, 2)
    da = rng.standard_normal(a.shape)
    dz = T.act_pool_bwd(da, sel, 6, 4, 2)
    eps = 1e-6
    for _ in range(40):
        i = tuple(int(rng.integers(0, s)) for s in z.shape)
        zp = z.copy()
        zp[i] += eps
        zm = z.copy()
        zm[i] -= eps
        num = ((T.act_pool_fwd(zp, 2)[0] - T.act_pool_fwd(zm, 2)[0]) * da).sum() / (2 * eps)
        assert abs(num - dz[i]) <= 1e-6 * max(1.0, abs(dz[i]))
    # at most one nonzero per window, and what passes sums to the passed errors
    nz = (dz != 0).reshape(2, 3, 2, 2, 2, 3).sum(axis=(2, 4))
    assert nz.max() <= 1
    assert np.isclose(dz.sum(), da[sel != T.NONE].sum())
    assert np.array_equal(nz == 1, sel != T.NONE)

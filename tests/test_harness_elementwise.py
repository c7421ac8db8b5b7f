"""The comparison the GPU parity tests use, tried on the CPU: the per-element bound catches a single wrong
output that the relative L2 norm of the tensor lets through, and the stratified sample reaches every block."""
import numpy as np

from paper_2011_10170_amd import inputs as I
from tests._harness import (Case, assert_close, elementwise_excess, oracle_masks, rel_l2, stratified_indices, TOL_L2)

import pytest


def _case(oracle):
    L = I.Layer(2, 12, 12, 32, 16, 1)
    case = Case(L, "bf16", 8, 10, tag="harness")
    pid, kp, M, Wm = oracle_masks(oracle, case)
    ref = oracle.conv_fwd(case.x, Wm, 1)
    mag = oracle.conv_fwd(np.abs(case.x), np.abs(Wm), 1)
    return case, Wm, ref, mag


def test_correctly_rounded_result_passes(oracle):
    case, Wm, ref, mag = _case(oracle)
    got = oracle.bf16_round(ref)          # what a kernel with exact accumulation and one bf16 rounding stores
    worst, _ = elementwise_excess(got, ref, mag, "bf16")
    assert 0.5 < worst <= 1.0             # half a unit in the last place reaches 2^-8 relative at the low end of a binade
    assert_close(got, ref, mag, "bf16", TOL_L2["bf16"], "rounded")


def test_one_wrong_element_fails_where_the_norm_does_not(oracle):
    case, Wm, ref, mag = _case(oracle)
    got = oracle.bf16_round(ref).copy()
    flat = got.reshape(-1)
    # one output with one of its 40 products missing: far inside the norm bound, outside its own bound
    j = int(np.argmax(mag.reshape(-1)))
    flat[j] -= mag.reshape(-1)[j] / 40.0
    assert rel_l2(got, ref) <= TOL_L2["bf16"]
    worst, at = elementwise_excess(got, ref, mag, "bf16")
    assert at == j and worst > 1.0
    with pytest.raises(AssertionError):
        assert_close(got, ref, mag, "bf16", TOL_L2["bf16"], "perturbed")
    # a completely wrong element (another element's value) and a NaN fail too
    got = oracle.bf16_round(ref).copy()
    got.reshape(-1)[5] = got.reshape(-1)[77] + 1.0
    assert elementwise_excess(got, ref, mag, "bf16")[0] > 1.0
    got = oracle.bf16_round(ref).copy()
    got.reshape(-1)[9] = np.nan
    assert elementwise_excess(got, ref, mag, "bf16")[0] > 1.0


def test_float32_bound_is_tight_enough_for_a_dropped_term(oracle):
    L = I.Layer(1, 6, 6, 8, 8, 1)
    case = Case(L, "f32", 4, 4, tag="harness32")
    pid, kp, M, Wm = oracle_masks(oracle, case)
    ref = oracle.conv_fwd(case.x, Wm, 1)
    mag = oracle.conv_fwd(np.abs(case.x), np.abs(Wm), 1)
    assert elementwise_excess(ref, ref, mag, "f32")[0] == 0.0
    got = ref.copy()
    j = int(np.argmax(mag.reshape(-1)))
    got.reshape(-1)[j] += mag.reshape(-1)[j] * 1e-5
    assert elementwise_excess(got, ref, mag, "f32")[0] > 1.0


@pytest.mark.parametrize("shape", [(2, 5, 37, 40), (3, 1, 1, 3), (1, 64, 64, 64), (32, 224, 224, 64)])
def test_stratified_sample_touches_every_block(shape):
    rng = np.random.default_rng(0)
    idx = stratified_indices(shape, rng)
    N, H, W, CH = shape
    assert idx.min() >= 0 and idx.max() < N * H * W * CH
    c = idx % CH
    x = (idx // CH) % W
    y = (idx // (CH * W)) % H
    n = idx // (CH * W * H)
    blocks = set(zip(n.tolist(), y.tolist(), (x // 32).tolist(), (c // 32).tolist()))
    assert len(blocks) == N * H * ((W + 31) // 32) * ((CH + 31) // 32)
    assert idx.size <= max(150000, len(blocks))

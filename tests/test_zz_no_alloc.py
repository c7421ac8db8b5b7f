"""The entry point that allocates nothing, pc_conv_bwd_weight_noalloc, through the C ABI: its output equals that of
pc_conv_bwd_weight bit for bit (same kernels, same split; only the place of the partial sums differs) and stays
within the oracle's bound, on two calls in a row that share the GPU's fixed buffer, the second with a smaller
input; a layer whose scratch need exceeds the fixed buffer is rejected before anything runs."""
import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests._harness import Case, GpuLayer, Guarded, assert_close, oracle_masks, TOL_L2_DW

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


def _both(B, ctx, oracle, layer, dtype, P, n_keep, tag):
    import torch
    case = Case(layer, dtype, P, n_keep, tag=tag)
    print("no-alloc case", tag, layer, dtype, flush=True)
    g = GpuLayer(B, ctx, case)
    try:
        ref = Guarded(g.nnzk * 4, torch.float32)
        B.pc_conv_bwd_weight(ctx, g.desc, g.pk, g.x, g.dy, ref.ptr)
        out = Guarded(g.nnzk * 4, torch.float32)
        B.pc_conv_bwd_weight_noalloc(ctx, g.desc, g.pk, g.x, g.dy, out.ptr)
        torch.cuda.synchronize()
        assert out.margins_intact() and ref.margins_intact()
        assert torch.isfinite(out.body).all()
        assert torch.equal(out.body, ref.body), "differs from pc_conv_bwd_weight"
        pid, kp, M, Wm = oracle_masks(oracle, case)
        dense = g.scatter(out.body)
        assert_close(dense, oracle.conv_bwd_weight(case.x, case.dy, M, layer.stride),
                     oracle.conv_bwd_weight(case.x, np.abs(case.dy), M, layer.stride), "f32", TOL_L2_DW, "no-alloc bwd_weight")
    finally:
        g.close()


def test_two_calls_in_a_row_second_smaller(B, ctx, oracle):
    # matrix-core kernels, several pixel splits: the partial sums of both calls go through the fixed buffer
    _both(B, ctx, oracle, I.Layer(8, 16, 16, 64, 128, 1), "bf16", 8, 19, "noalloc_a")
    _both(B, ctx, oracle, I.Layer(3, 7, 9, 40, 24, 2), "bf16", 8, 12, "noalloc_b")
    # the gather kernels (float32), and a first layer whose 3 channels are copied to 8-channel rows in the buffer
    _both(B, ctx, oracle, I.Layer(8, 32, 32, 16, 16, 1), "f32", 4, 8, "noalloc_c")
    _both(B, ctx, oracle, I.Layer(2, 16, 16, 3, 64, 1), "bf16", 8, 1, "noalloc_d")


def test_a_layer_beyond_the_fixed_buffer_is_rejected(B, ctx):
    """N*H*W*16 bytes for the 8-channel copy of a 3-channel input: 51 MB at N = 64, 224 x 224; nothing is launched."""
    import torch
    L = I.Layer(64, 224, 224, 3, 64, 1)
    lib = I.make_library(8)
    W = torch.randn((L.F, L.C, 9), device="cuda")
    pid = torch.empty((L.F, L.C), dtype=torch.uint8, device="cuda")
    keep = torch.empty((L.F, L.C), dtype=torch.uint8, device="cuda")
    B.pc_pattern_select(ctx, W, None, L.F, L.C, lib, B.PC_KEEP_PER_FILTER, 1, B.PC_SCORE_RETAINED, pid, keep)
    pk = B.pc_pack(ctx, W, pid, keep, L.F, L.C, lib, B.PC_BF16)
    try:
        x = torch.zeros((L.N, L.H, L.W, L.C), dtype=torch.bfloat16, device="cuda")
        dy = torch.zeros((L.N, L.Ho, L.Wo, L.F), dtype=torch.bfloat16, device="cuda")
        dw = torch.full((L.F, 4), 5.0, dtype=torch.float32, device="cuda")
        desc = B.make_desc(L.N, L.H, L.W, L.C, L.F, 1, B.PC_BF16)
        with pytest.raises(B.PcError) as ei:
            B.pc_conv_bwd_weight_noalloc(ctx, desc, pk, x, dy, dw)
        assert ei.value.status == B.PC_ERR_UNSUPPORTED
        torch.cuda.synchronize()
        assert bool((dw == 5.0).all().item())
        B.pc_conv_bwd_weight(ctx, desc, pk, x, dy, dw)      # the allocating entry point takes it
        torch.cuda.synchronize()
        assert bool((dw == 0.0).all().item())
    finally:
        B.pc_packed_free(pk)

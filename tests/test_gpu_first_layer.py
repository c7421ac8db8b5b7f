"""GPU parity of the first-layer kernels (stride 1, at most 4 input channels): every output element of the three
passes against the oracle, on shapes with ragged rows, columns and tiles, 1 to 4 input channels and 1 to 4 row tiles
of 32 filters; the fused ReLU of the forward launch; and that the automatic choice really takes these kernels."""
import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests.test_gpu_parity import run_case

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

# (N, H, W, C, F, stride): the backward-data kernel takes 32 and 64 filters, the forward kernel up to 128
FIRST_LAYER_SHAPES = [
    (2, 9, 37, 3, 64, 1),       # ragged rows and columns
    (3, 16, 32, 1, 32, 1),      # one channel, one row tile
    (1, 8, 40, 4, 96, 1),       # four channels, three row tiles (backward-data on the general kernels)
    (2, 17, 33, 2, 64, 1),
    (1, 5, 300, 3, 128, 1),     # two column tiles, four row tiles
    (4, 32, 32, 3, 64, 1),      # the CIFAR first layer
    (1, 1, 1, 3, 32, 1),        # a single pixel
]


@pytest.mark.parametrize("keep", [0.3, 1.0])
@pytest.mark.parametrize("shape", FIRST_LAYER_SHAPES)
def test_first_layer_passes(B, ctx, oracle, shape, keep):
    run_case(B, ctx, oracle, shape, "bf16", 8, keep, B.PC_VARIANT_MFMA, ("first_layer", keep))


@pytest.mark.parametrize("shape", [(2, 9, 37, 3, 64, 1), (3, 16, 32, 1, 32, 1)])
def test_first_layer_kernels_forced(B, ctx, oracle, shape):
    """Override code 23 fails rather than falling back to another kernel."""
    B.pc_set_plan_override(ctx, 23, 0)
    try:
        run_case(B, ctx, oracle, shape, "bf16", 8, 0.4, B.PC_VARIANT_MFMA, "first_layer_forced")
    finally:
        B.pc_set_plan_override(ctx, -1, 0)


def test_first_layer_kernels_are_the_automatic_choice_and_fuse_the_relu(B, ctx):
    import torch
    from tests._harness import Case, GpuLayer
    layer = I.Layer(3, 20, 45, 3, 64, 1)
    case = Case(layer, "bf16", 8, I.kept_per_filter(0.4, layer.C), tag="first_layer_auto")
    g = GpuLayer(B, ctx, case)
    try:
        L = layer
        y = torch.empty((L.N, L.Ho, L.Wo, L.F), dtype=torch.bfloat16, device="cuda")
        a = torch.full_like(y, float("nan"))
        dx = torch.empty((L.N, L.H, L.W, L.C), dtype=torch.bfloat16, device="cuda")
        dz = torch.full_like(dx, float("nan"))
        B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, y)
        assert B.pc_last_kernel(ctx).startswith("pc_thin_fwd_kernel")
        B.pc_conv_fwd_relu(ctx, g.desc, g.pk, g.x, a)
        B.pc_conv_bwd_data(ctx, g.desc, g.pk, g.dy, dx)
        assert B.pc_last_kernel(ctx).startswith("pc_thin_bwd_data_kernel")
        B.pc_conv_bwd_data_relu(ctx, g.desc, g.pk, g.dy, g.x, dz)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), torch.where(y > 0, y, torch.zeros_like(y)).view(torch.int16))
        assert torch.equal(dz.view(torch.int16), torch.where(g.x > 0, dx, torch.zeros_like(dx)).view(torch.int16))
        # a forced general kernel gives the same values up to the float32 order of additions
        from tests._harness import rel_l2, from_dev_f32
        B.pc_set_plan_override(ctx, 6, 0)
        yg = torch.empty_like(y)
        dxg = torch.empty_like(dx)
        B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, yg)
        assert B.pc_last_kernel(ctx).startswith("pc_mfma_conv_kernel")
        B.pc_conv_bwd_data(ctx, g.desc, g.pk, g.dy, dxg)
        torch.cuda.synchronize()
        assert rel_l2(from_dev_f32(y), from_dev_f32(yg)) <= 3e-3 and rel_l2(from_dev_f32(dx), from_dev_f32(dxg)) <= 3e-3
    finally:
        B.pc_set_plan_override(ctx, -1, 0)
        g.close()

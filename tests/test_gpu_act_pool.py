"""GPU parity of the step between two chained layers (ReLU + optional 2x2 max pooling, and its backward pass)
against oracle/pc_oracle_chain.py, through the C ABI. Both passes only compare and copy, so every output
(activations, selection bytes, propagated errors) is compared bit for bit, in float32 and in bfloat16. Inputs
with many ties (bfloat16 rounding, small integers) exercise the first-maximum rule; odd extents, channel counts
that do not fill a 16-byte access and misaligned pointers exercise the element-wise kernels."""
import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests._harness import CANARY, Guarded, to_dev

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


@pytest.fixture(scope="module")
def T():
    from oracle import pc_oracle_chain
    return pc_oracle_chain


def _values(shape, dtype, kind, seed):
    """(host array handed to the device, the same values as float32 for the oracle)."""
    rng = np.random.default_rng(seed)
    if kind == "normal":
        v = rng.standard_normal(shape).astype(np.float32)
    else:                                                   # small integers: ties in almost every window
        v = rng.integers(-2, 3, size=shape).astype(np.float32)
    if dtype == "bf16":
        bits = I.f32_to_bf16_bits(v)
        return bits, I.bf16_bits_to_f32(bits)
    return v, v


def _bits(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy().view(np.uint32)


def _host_bits(a32, dtype):
    return I.f32_to_bf16_bits(a32) if dtype == "bf16" else np.ascontiguousarray(a32).view(np.uint32)


class GuardedBytes:
    """uint8 device buffer with sentinel margins (the harness class fills floating-point sentinels)."""

    def __init__(self, n: int):
        import torch
        self.n = n
        self.buf = torch.full((n + 2 * CANARY,), 7, dtype=torch.uint8, device="cuda")
        self.body = self.buf[CANARY:CANARY + n]
        self.body.fill_(99)
        self.ptr = self.buf.data_ptr() + CANARY

    def margins_intact(self) -> bool:
        import torch
        m = torch.cat([self.buf[:CANARY], self.buf[CANARY + self.n:]])
        return bool((m == 7).all().item())


def _run(B, ctx, T, shape, dtype, pool, kind, seed, misalign=0):
    import torch
    N, H, W, C = shape
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    pdt = B.PC_BF16 if dtype == "bf16" else B.PC_F32
    zh, z32 = _values(shape, dtype, kind, seed)
    ref_a, ref_sel = T.act_pool_fwd(z32, pool)
    Ho, Wo = H // pool, W // pool
    n_out = N * Ho * Wo * C
    zd = to_dev(zh)
    a = Guarded(n_out + misalign, tdt)
    sel = GuardedBytes(n_out + misalign)
    esz = 2 if dtype == "bf16" else 4
    B.pc_act_pool_fwd(ctx, zd, N, H, W, C, pdt, pool, a.ptr + misalign * esz, sel.ptr + misalign)
    torch.cuda.synchronize()
    assert a.margins_intact() and sel.margins_intact()
    got_a = _bits(a.body[misalign:])
    got_sel = sel.body[misalign:].cpu().numpy()
    assert np.array_equal(got_sel, ref_sel.reshape(-1))
    assert np.array_equal(got_a, _host_bits(ref_a, dtype).reshape(-1))
    # backward with the selection bytes the forward call wrote
    dah, da32 = _values(ref_a.shape, dtype, "normal", seed + 1)
    ref_dz = T.act_pool_bwd(da32, ref_sel, H, W, pool)
    dz = Guarded(N * H * W * C + misalign, tdt)
    B.pc_act_pool_bwd(ctx, to_dev(dah), sel.ptr + misalign, N, H, W, C, pdt, pool, dz.ptr + misalign * esz)
    torch.cuda.synchronize()
    assert dz.margins_intact()
    assert np.array_equal(_bits(dz.body[misalign:]), _host_bits(ref_dz, dtype).reshape(-1))


SHAPES = [(1, 1, 1, 1), (1, 2, 2, 1), (2, 4, 4, 3), (1, 7, 5, 4), (3, 9, 9, 8), (2, 6, 6, 16), (5, 33, 17, 24),
          (2, 3, 2, 40), (4, 16, 16, 64), (3, 5, 8, 13)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("pool", [1, 2])
def test_act_pool_bit_exact(B, ctx, T, shape, dtype, pool):
    if pool == 2 and (shape[1] < 2 or shape[2] < 2):
        pytest.skip("no 2x2 window in this map")
    for kind in ("normal", "ties"):
        _run(B, ctx, T, shape, dtype, pool, kind, seed=sum(shape) * 8 + pool * 2 + (kind == "ties"))


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_misaligned_pointers_take_the_elementwise_kernels(B, ctx, T, dtype):
    for mis in (1, 3):
        _run(B, ctx, T, (2, 6, 10, 16), dtype, 2, "ties", seed=7, misalign=mis)
        _run(B, ctx, T, (2, 6, 10, 16), dtype, 1, "normal", seed=8, misalign=mis)


@pytest.mark.parametrize("shape,pool", [((128, 32, 32, 64), 2), ((128, 16, 16, 128), 1), ((128, 2, 2, 512), 2),
                                        ((32, 224, 224, 64), 2), ((32, 14, 14, 512), 1)])
def test_full_size_maps(B, ctx, T, shape, pool):
    """The maps of the VGG-16 workloads at their batch sizes (CIFAR batch 128, ImageNet batch 32), bfloat16."""
    _run(B, ctx, T, shape, "bf16", pool, "normal", seed=11)


def test_argument_checks(B, ctx):
    import torch
    t = torch.zeros(64, dtype=torch.float32, device="cuda")
    s = torch.zeros(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.PcError):
        B.pc_act_pool_fwd(ctx, t, 1, 4, 4, 4, B.PC_F32, 3, t, s)
    with pytest.raises(B.PcError):
        B.pc_act_pool_fwd(ctx, t, 1, 1, 4, 4, B.PC_F32, 2, t, s)
    with pytest.raises(B.PcError):
        B.pc_act_pool_fwd(ctx, None, 1, 4, 4, 4, B.PC_F32, 2, t, s)
    with pytest.raises(B.PcError):
        B.pc_act_pool_bwd(ctx, t, s, 0, 4, 4, 4, B.PC_F32, 2, t)
    with pytest.raises(B.PcError):
        B.pc_act_pool_bwd(ctx, t, s, 1, 4, 4, 4, 7, 2, t)


def test_three_layer_chain_f32(B, ctx, T, oracle):
    """conv -> ReLU/pool -> conv -> ReLU -> conv -> ReLU/pool and the whole backward pass, float32, against the same
    chain of oracle calls. Float32 rounding can flip a comparison only between nearly equal values, so the chain as
    a whole is held to the float32 tolerance of a single pass (relative L2 error 1e-4)."""
    import torch
    from tests._harness import rel_l2
    N, H, W = 3, 12, 10
    chans = [5, 16, 24, 8]
    pools = [2, 1, 2]
    lib = I.make_library(8)
    Ls, packs, Wms, Ms = [], [], [], []
    h, w = H, W
    for li in range(3):
        L = I.Layer(N, h, w, chans[li], chans[li + 1], 1)
        Wn = I.gen_weights(L.F, L.C, I.BASE_SEED, ("chain", li))
        k = I.kept_per_filter(0.6, L.C)
        pid, keep = oracle.select(Wn, None, lib, k)
        M = oracle.mask(pid, keep, lib)
        Wms.append(oracle.apply_mask(Wn, M))
        Ms.append(M)
        pd, kd = torch.empty((L.F, L.C), dtype=torch.uint8, device="cuda"), torch.empty((L.F, L.C), dtype=torch.uint8, device="cuda")
        Wd = to_dev(Wn)
        B.pc_pattern_select(ctx, Wd, None, L.F, L.C, lib, B.PC_KEEP_PER_FILTER, k, B.PC_SCORE_RETAINED, pd, kd)
        packs.append(B.pc_pack(ctx, Wd, pd, kd, L.F, L.C, lib, B.PC_F32))
        Ls.append(L)
        h, w = h // pools[li], w // pools[li]
    x0 = I.gen_activations((N, H, W, chans[0]), I.BASE_SEED, ("chain", "x"), True, "f32")[1]
    # oracle chain
    xs, zs, sels = [x0], [], []
    for li in range(3):
        z = oracle.conv_fwd(xs[-1], Wms[li], 1)
        a, sel = T.act_pool_fwd(z, pools[li])
        zs.append(z); sels.append(sel); xs.append(a)
    da = I.gen_activations(xs[-1].shape, I.BASE_SEED, ("chain", "da"), False, "f32")[1]
    ref_dw = [None] * 3
    g = da
    for li in (2, 1, 0):
        L = Ls[li]
        dz = T.act_pool_bwd(g, sels[li], L.Ho, L.Wo, pools[li])
        ref_dw[li] = oracle.conv_bwd_weight(xs[li], dz, Ms[li], 1)
        g = oracle.conv_bwd_data(dz, Wms[li], xs[li].shape, 1)
    ref_dx0 = g
    # the same chain through the library
    dxs = [to_dev(x0)]
    dsel = []
    for li in range(3):
        L = Ls[li]
        desc = B.make_desc(L.N, L.H, L.W, L.C, L.F, 1, B.PC_F32)
        z = torch.empty((N, L.Ho, L.Wo, L.F), dtype=torch.float32, device="cuda")
        B.pc_conv_fwd(ctx, desc, packs[li], dxs[-1], z)
        q = pools[li]
        a = torch.empty((N, L.Ho // q, L.Wo // q, L.F), dtype=torch.float32, device="cuda")
        s = torch.empty(a.shape, dtype=torch.uint8, device="cuda")
        B.pc_act_pool_fwd(ctx, z, N, L.Ho, L.Wo, L.F, B.PC_F32, q, a, s)
        dxs.append(a); dsel.append(s)
    torch.cuda.synchronize()
    assert rel_l2(dxs[-1].cpu().numpy(), xs[-1]) <= 1e-4
    gd = to_dev(da)
    for li in (2, 1, 0):
        L = Ls[li]
        desc = B.make_desc(L.N, L.H, L.W, L.C, L.F, 1, B.PC_F32)
        dz = torch.empty((N, L.Ho, L.Wo, L.F), dtype=torch.float32, device="cuda")
        B.pc_act_pool_bwd(ctx, gd, dsel[li], N, L.Ho, L.Wo, L.F, B.PC_F32, pools[li], dz)
        nnzk, _ = B.pc_packed_info(ctx, packs[li])
        dw = torch.empty((nnzk, 4), dtype=torch.float32, device="cuda")
        B.pc_conv_bwd_weight(ctx, desc, packs[li], dxs[li], dz, dw)
        dense = torch.zeros((L.F, L.C, 9), dtype=torch.float32, device="cuda")
        B.pc_scatter_dense(ctx, packs[li], dw, dense)
        gd = torch.empty((N, L.H, L.W, L.C), dtype=torch.float32, device="cuda")
        B.pc_conv_bwd_data(ctx, desc, packs[li], dz, gd)
        torch.cuda.synchronize()
        assert rel_l2(dense.cpu().numpy(), ref_dw[li]) <= 1e-4
    assert rel_l2(gd.cpu().numpy(), ref_dx0) <= 1e-4
    for pk in packs:
        B.pc_packed_free(pk)


FUSED_LAYERS = [I.Layer(4, 8, 8, 64, 64, 1), I.Layer(2, 9, 7, 128, 96, 1), I.Layer(3, 6, 6, 3, 64, 1), I.Layer(3, 6, 6, 64, 3, 1),
                I.Layer(2, 9, 9, 64, 64, 2), I.Layer(2, 5, 5, 40, 72, 1)]


@pytest.mark.parametrize("layer", FUSED_LAYERS)
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_conv_with_fused_relu_equals_the_two_calls(B, ctx, T, oracle, layer, dtype):
    """pc_conv_fwd_relu and pc_conv_bwd_data_relu against pc_conv_fwd / pc_conv_bwd_data followed by the ReLU step on
    the stored values (bit for bit: the step only zeroes elements), and against the oracle chain within the conv
    tolerance. Layers the fused kernels take, and layers that fall back to a second launch (3 channels out,
    stride-2 backward, float32)."""
    import torch
    from tests._harness import Case, GpuLayer, oracle_masks, rel_l2, from_dev_f32
    case = Case(layer, dtype, 8, I.kept_per_filter(0.4, layer.C), tag=("fused", layer.C, layer.F, layer.stride))
    g = GpuLayer(B, ctx, case)
    try:
        tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
        L = layer
        y = torch.empty((L.N, L.Ho, L.Wo, L.F), dtype=tdt, device="cuda")
        a = torch.full_like(y, float("nan"))
        B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, y)
        B.pc_conv_fwd_relu(ctx, g.desc, g.pk, g.x, a)
        torch.cuda.synchronize()
        want = torch.where(y > 0, y, torch.zeros_like(y))
        assert torch.equal(a.view(torch.int16 if dtype == "bf16" else torch.int32), want.view(torch.int16 if dtype == "bf16" else torch.int32))
        pid, kp, M, Wm = oracle_masks(oracle, case)
        ref = np.maximum(oracle.conv_fwd(case.x, Wm, L.stride), 0)
        assert rel_l2(from_dev_f32(a), ref) <= (2e-2 if dtype == "bf16" else 1e-4)
        # backward: the mask is this layer's input; once as it is (post-ReLU: zeros and positives), once with negatives
        dx = torch.empty((L.N, L.H, L.W, L.C), dtype=tdt, device="cuda")
        B.pc_conv_bwd_data(ctx, g.desc, g.pk, g.dy, dx)
        for mask in (g.x, (g.x.float() - 0.3).to(tdt)):
            dz = torch.full_like(dx, float("nan"))
            B.pc_conv_bwd_data_relu(ctx, g.desc, g.pk, g.dy, mask, dz)
            torch.cuda.synchronize()
            want = torch.where(mask > 0, dx, torch.zeros_like(dx))
            assert torch.equal(dz.view(torch.int16 if dtype == "bf16" else torch.int32),
                               want.view(torch.int16 if dtype == "bf16" else torch.int32))
    finally:
        g.close()


@pytest.mark.parametrize("cfg", [7, 8, 9, 13, 14, 15, 16, 19, 20, 21])
def test_fused_relu_in_every_tile_configuration(B, ctx, cfg):
    """The fused step in both store paths of the wave-specialised kernel (reduction split and pixel split) and
    every tile shape: bit-identical to the plain launch of the same configuration followed by the step."""
    import torch
    from tests._harness import Case, GpuLayer
    layer = I.Layer(6, 10, 9, 128, 160, 1)
    case = Case(layer, "bf16", 8, I.kept_per_filter(0.3, layer.C), tag=("fused_cfg", cfg))
    g = GpuLayer(B, ctx, case)
    try:
        B.pc_set_plan_override(ctx, cfg, 0)
        L = layer
        y = torch.empty((L.N, L.Ho, L.Wo, L.F), dtype=torch.bfloat16, device="cuda")
        a = torch.full_like(y, float("nan"))
        dx = torch.empty((L.N, L.H, L.W, L.C), dtype=torch.bfloat16, device="cuda")
        dz = torch.full_like(dx, float("nan"))
        try:
            B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, y)
        except B.PcError:
            pytest.skip("this configuration does not take the layer")
        B.pc_conv_fwd_relu(ctx, g.desc, g.pk, g.x, a)
        B.pc_conv_bwd_data(ctx, g.desc, g.pk, g.dy, dx)
        B.pc_conv_bwd_data_relu(ctx, g.desc, g.pk, g.dy, g.x, dz)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), torch.where(y > 0, y, torch.zeros_like(y)).view(torch.int16))
        assert torch.equal(dz.view(torch.int16), torch.where(g.x > 0, dx, torch.zeros_like(dx)).view(torch.int16))
    finally:
        B.pc_set_plan_override(ctx, -1, 0)
        g.close()


@pytest.mark.parametrize("keep", [0.2, 0.6])
def test_fused_relu_in_the_structured_sparse_kernel(B, ctx, keep):
    """The fused step at the store of the structured-sparse kernel, with the overflow weights as lists (keep 0.2) and
    through the second operand part (keep 0.6: the lists do not fit): bit-identical to the plain launch followed by
    the step, and the plain launch equals the zero-filled kernel's result up to the float32 order of additions."""
    import torch
    from tests._harness import Case, GpuLayer, rel_l2, from_dev_f32
    layer = I.Layer(6, 10, 9, 128, 160, 1)
    case = Case(layer, "bf16", 16, I.kept_per_filter(keep, layer.C), tag=("fused_sparse", keep))
    g = GpuLayer(B, ctx, case, variant=B.PC_VARIANT_MFMA_SPARSE)
    gd = GpuLayer(B, ctx, case, variant=B.PC_VARIANT_MFMA)
    try:
        assert g.variant == B.PC_VARIANT_MFMA_SPARSE
        B.pc_set_plan_override(ctx, 22, 0)
        L = layer
        y = torch.empty((L.N, L.Ho, L.Wo, L.F), dtype=torch.bfloat16, device="cuda")
        a = torch.full_like(y, float("nan"))
        dx = torch.empty((L.N, L.H, L.W, L.C), dtype=torch.bfloat16, device="cuda")
        dz = torch.full_like(dx, float("nan"))
        B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, y)
        assert B.pc_last_kernel(ctx).startswith("pc_mfma_conv_sp_kernel")
        B.pc_conv_fwd_relu(ctx, g.desc, g.pk, g.x, a)
        B.pc_conv_bwd_data(ctx, g.desc, g.pk, g.dy, dx)
        B.pc_conv_bwd_data_relu(ctx, g.desc, g.pk, g.dy, g.x, dz)
        torch.cuda.synchronize()
        assert torch.equal(a.view(torch.int16), torch.where(y > 0, y, torch.zeros_like(y)).view(torch.int16))
        assert torch.equal(dz.view(torch.int16), torch.where(g.x > 0, dx, torch.zeros_like(dx)).view(torch.int16))
        B.pc_set_plan_override(ctx, -1, 0)
        yd = torch.empty_like(y)
        dxd = torch.empty_like(dx)
        B.pc_conv_fwd(ctx, gd.desc, gd.pk, gd.x, yd)
        B.pc_conv_bwd_data(ctx, gd.desc, gd.pk, gd.dy, dxd)
        torch.cuda.synchronize()
        assert rel_l2(from_dev_f32(y), from_dev_f32(yd)) <= 3e-3 and rel_l2(from_dev_f32(dx), from_dev_f32(dxd)) <= 3e-3
    finally:
        B.pc_set_plan_override(ctx, -1, 0)
        g.close()
        gd.close()

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

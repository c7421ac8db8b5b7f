"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs. Masks and pattern ids must be bit-exact; conv outputs within 1e-4 relative L2 (float32)
or 2e-2 (bf16 inputs, float32 accumulation); float32 weight gradients within 1e-4 in both cases."""
import sys

import numpy as np
import pytest

from paper_2011_10170_amd import inputs as I
from tests._harness import Case, GpuLayer, assert_close, oracle_masks, rel_l2, to_dev, TOL_L2 as TOL, TOL_L2_DW as TOL_DW

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


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


# N, H, W, C, F, stride: small enough for the full oracle, spanning several tiles with ragged tails
SMALL = [
    (8, 32, 32, 16, 16, 1),     # the single-layer float32 configuration
    (2, 13, 19, 5, 7, 1),
    (3, 9, 11, 6, 10, 2),
    (1, 1, 1, 3, 4, 1),
    (2, 2, 2, 8, 8, 2),
    (1, 40, 37, 12, 20, 1),
    (1, 12, 12, 200, 24, 1),    # more channels than one LDS pass holds
    (2, 33, 35, 7, 18, 2),
    (5, 4, 4, 32, 48, 1),
    (20, 2, 2, 16, 32, 1),
    (2, 16, 16, 3, 64, 1),      # first-layer shape: 3 input channels
]
MEDIUM_BF16 = [
    (4, 16, 16, 64, 64, 1),
    (4, 16, 16, 64, 128, 2),
    (8, 4, 4, 128, 128, 1),
    (16, 2, 2, 64, 64, 1),
    (2, 28, 28, 32, 96, 1),
    (2, 14, 14, 96, 32, 2),
    (3, 7, 7, 64, 64, 1),
]


def run_case(B, ctx, oracle, shape, dtype, P, keep, variant, tag, keep_mode=0):
    N, H, W, C, F, stride = shape
    layer = I.Layer(N, H, W, C, F, stride)
    n_keep = I.kept_per_filter(keep, C) if keep_mode == 0 else max(1, int(keep * F * C + 0.5))
    case = Case(layer, dtype, P, n_keep, tag=(tag, shape, dtype))
    say("case", tag, shape, dtype, "P", P, "keep", keep, "variant", variant, "keep_mode", keep_mode)
    pid, kp, M, Wm = oracle_masks(oracle, case, keep_mode=keep_mode)
    g = GpuLayer(B, ctx, case, variant=variant, keep_mode=keep_mode)
    try:
        gpid, gkeep = g.masks()
        assert np.array_equal(gpid, pid), "pattern ids differ"
        assert np.array_equal(gkeep, kp), "keep mask differs"
        assert g.nnzk == int(kp.sum())
        assert np.array_equal(g.unpack(), Wm), "unpacked weights differ from W (.) M"
        # every output element against the oracle, each within its own bound (the oracle on absolute values gives
        # the magnitude of the sum behind every element), beside the relative L2 norm of the whole tensor
        aW, ax, ady = np.abs(Wm), np.abs(case.x), np.abs(case.dy)
        y_ref = oracle.conv_fwd(case.x, Wm, stride)
        assert_close(g.fwd(), y_ref, oracle.conv_fwd(ax, aW, stride), dtype, TOL[dtype], "fwd")
        dx_ref = oracle.conv_bwd_data(case.dy, Wm, case.x.shape, stride)
        assert_close(g.bwd_data(), dx_ref, oracle.conv_bwd_data(ady, aW, case.x.shape, stride), dtype, TOL[dtype], "bwd_data")
        dw_ref_dense = oracle.conv_bwd_weight(case.x, case.dy, M, stride)
        dw_mag_dense = oracle.conv_bwd_weight(ax, ady, M, stride)
        sf, sc = oracle.compact_order(pid, kp, P)
        dw_ref = oracle.gather_compact(dw_ref_dense, pid, case.lib, sf, sc)
        dw_mag = oracle.gather_compact(dw_mag_dense, pid, case.lib, sf, sc)
        dw, guard = g.bwd_weight()
        assert_close(dw, dw_ref, dw_mag, "f32", TOL_DW, "bwd_weight")
        dense = g.scatter(guard.body)
        assert np.all(dense[M == 0] == 0.0)
        assert_close(dense, dw_ref_dense, dw_mag_dense, "f32", TOL_DW, "bwd_weight scattered")
        return g.variant
    finally:
        g.close()


@pytest.mark.parametrize("shape", SMALL)
def test_small_f32(B, ctx, oracle, shape):
    run_case(B, ctx, oracle, shape, "f32", 4 if shape[3] == 16 else 8, 0.5, B.PC_VARIANT_AUTO, "small")


@pytest.mark.parametrize("shape", SMALL)
def test_small_bf16_valu(B, ctx, oracle, shape):
    run_case(B, ctx, oracle, shape, "bf16", 8, 0.4, B.PC_VARIANT_VALU, "small")


@pytest.mark.parametrize("shape", SMALL)
def test_small_bf16_auto(B, ctx, oracle, shape):
    """The default kernel choice for bf16 (matrix-core kernels), on odd channel counts and ragged tiles."""
    run_case(B, ctx, oracle, shape, "bf16", 8, 0.4, B.PC_VARIANT_AUTO, "small_auto")


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5, 6])
@pytest.mark.parametrize("split", [0, 3])
def test_every_mfma_tile_configuration(B, ctx, oracle, cfg, split):
    """Each built tile configuration of the forward/backward-data kernel, with and without split-K."""
    B.pc_set_plan_override(ctx, cfg, split)
    try:
        for shape in [(3, 12, 20, 72, 96, 1), (2, 9, 9, 40, 24, 2)]:
            run_case(B, ctx, oracle, shape, "bf16", 8, 0.3, B.PC_VARIANT_MFMA, ("cfg", cfg, split))
    finally:
        B.pc_set_plan_override(ctx, -1, 0)


# Shapes for the wave-specialised forward/backward-data kernel (channel counts that are multiples of 8): a
# partial last channel chunk, tiny images, a strided layer, and more tiles than workgroups.
WAVE_SPEC = [
    (3, 12, 20, 72, 96, 1),
    (2, 9, 9, 40, 24, 2),
    (20, 2, 2, 128, 64, 1),
    (5, 4, 4, 192, 80, 1),
    (12, 32, 32, 64, 128, 1),
]


@pytest.mark.parametrize("cfg", [7, 8, 9, 13, 14, 15, 16, 17, 18, 19, 20, 21])
@pytest.mark.parametrize("shape", WAVE_SPEC)
def test_wave_specialised_kernel(B, ctx, oracle, cfg, shape):
    """The persistent kernel with loader wavefronts: the reduction split over four MFMA wavefronts for each of
    its pixel-tile widths (7, 8, 9: 128, 64 and 32 pixels; 14, 21: 32 and 64 pixels with 128-channel chunks; 15: the same with 32 output channels), and the
    pixel split (13: 512-pixel tiles, 16: 256-pixel tiles; 17, 18: the same with 16-channel chunks; 19: 512-pixel
    tiles of 32 output channels; 20: 256-pixel tiles with 64-channel chunks)."""
    B.pc_set_plan_override(ctx, cfg, 0)
    try:
        run_case(B, ctx, oracle, shape, "bf16", 8, 0.3, B.PC_VARIANT_MFMA, ("wave_spec", cfg))
    finally:
        B.pc_set_plan_override(ctx, -1, 0)


# The structured-sparse kernel (packs made under PC_VARIANT_MFMA_SPARSE): keep ratios from nearly every group of 4
# channels within the instruction's 2-of-4 form (0.05) to none of them (1.0: every kept kernel's neighbours are kept
# too, so the second operand part carries half of the weights); partial channel chunks, more tiles than workgroups.
SPARSE_SHAPES = [
    (3, 12, 20, 72, 96, 1),
    (20, 2, 2, 128, 64, 1),
    (5, 4, 4, 192, 80, 1),
    (12, 32, 32, 64, 128, 1),
    (2, 28, 28, 256, 64, 1),
]


@pytest.mark.parametrize("keep", [0.05, 0.2, 0.45, 1.0])
@pytest.mark.parametrize("shape", SPARSE_SHAPES)
def test_structured_sparse_kernel(B, ctx, oracle, keep, shape):
    B.pc_set_plan_override(ctx, 22, 0)       # fail rather than fall back to another kernel
    try:
        v = run_case(B, ctx, oracle, shape, "bf16", 16, keep, B.PC_VARIANT_MFMA_SPARSE, ("sparse", keep))
        assert v == B.PC_VARIANT_MFMA_SPARSE
        assert B.pc_last_kernel(ctx).startswith("pc_mfma_wgrad")      # the weight gradient ran last
    finally:
        B.pc_set_plan_override(ctx, -1, 0)


def test_structured_sparse_variant_other_layers(B, ctx, oracle):
    """Layers the structured-sparse kernel does not take (few channels, stride 2) use the pack's dense tiles."""
    for shape in [(2, 16, 16, 3, 64, 1), (3, 9, 11, 40, 24, 2), (2, 14, 14, 96, 32, 2)]:
        run_case(B, ctx, oracle, shape, "bf16", 8, 0.3, B.PC_VARIANT_MFMA_SPARSE, "sparse_other")


# Filter counts that are multiples of 8 (what the wave-specialised kernel takes): several pixel tiles per
# workgroup, strided and tiny-image layers, partial channel tiles, short image groups; both backward-weight
# kernels (10 = cooperative, 11 = wave-specialised).
WGRAD_SHAPES = [
    (8, 12, 20, 72, 96, 1),
    (16, 9, 9, 40, 24, 2),
    (24, 2, 2, 128, 64, 1),
    (8, 4, 4, 192, 80, 1),
    (16, 32, 32, 64, 128, 1),
    (32, 8, 8, 64, 64, 1),
    (12, 6, 10, 16, 24, 1),     # the last image group is short
    (3, 5, 5, 8, 8, 2),
    (16, 16, 16, 3, 64, 1),     # first-layer shape: the input is copied to 8-channel rows
    (8, 7, 9, 12, 24, 1),
]


@pytest.mark.parametrize("cfg", [10, 11])
@pytest.mark.parametrize("shape", WGRAD_SHAPES)
def test_backward_weight_kernels(B, ctx, oracle, cfg, shape):
    B.pc_set_plan_override(ctx, cfg, 0)
    try:
        run_case(B, ctx, oracle, shape, "bf16", 8, 0.3, B.PC_VARIANT_MFMA, ("wgrad", cfg))
    finally:
        B.pc_set_plan_override(ctx, -1, 0)


@pytest.mark.parametrize("shape", MEDIUM_BF16)
def test_medium_bf16_valu(B, ctx, oracle, shape):
    run_case(B, ctx, oracle, shape, "bf16", 12, 0.3, B.PC_VARIANT_VALU, "medium")


@pytest.mark.parametrize("shape", MEDIUM_BF16)
def test_medium_bf16_auto(B, ctx, oracle, shape):
    run_case(B, ctx, oracle, shape, "bf16", 16, 0.25, B.PC_VARIANT_AUTO, "medium")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 9, 9, 24, 40, 1), (3, 8, 8, 64, 64, 2), (2, 6, 6, 130, 96, 1)])
def test_per_layer_keep_unbalanced_rows(B, ctx, oracle, shape, dtype):
    """Kept kernels chosen over the whole layer: filters keep different numbers of kernels (some possibly none)."""
    N, H, W, C, F, stride = shape
    run_case(B, ctx, oracle, shape, dtype, 8, 0.15, B.PC_VARIANT_AUTO, "perlayer", keep_mode=1)
    layer_case = Case(I.Layer(*shape), dtype, 8, max(1, int(0.15 * F * C + 0.5)), tag=("perlayer", shape, dtype))
    _, kp, _, _ = oracle_masks(oracle, layer_case, keep_mode=1)
    assert len(set(kp.sum(axis=1).tolist())) > 1          # the rows really are unbalanced


def test_full_pool_and_every_pattern_f32(B, ctx, oracle):
    run_case(B, ctx, oracle, (2, 10, 10, 24, 16, 1), "f32", 126, 0.5, B.PC_VARIANT_AUTO, "p126")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_degenerate_keep_counts(B, ctx, oracle, dtype):
    """n_keep = 0 prunes everything (outputs are zero, no slots); n_keep = C is pattern-only pruning."""
    layer = I.Layer(2, 6, 7, 5, 6, 1)
    for n_keep in (0, 5):
        case = Case(layer, dtype, 8, n_keep, tag=("degenerate", n_keep))
        pid, kp, M, Wm = oracle_masks(oracle, case)
        g = GpuLayer(B, ctx, case)
        try:
            gpid, gkeep = g.masks()
            assert np.array_equal(gpid, pid) and np.array_equal(gkeep, kp)
            assert g.nnzk == n_keep * layer.F
            y = g.fwd()
            dx = g.bwd_data()
            if n_keep == 0:
                assert not y.any() and not dx.any()
                dw, _ = g.bwd_weight()
                assert dw.size == 0
            else:
                assert rel_l2(y, oracle.conv_fwd(case.x, Wm, 1)) <= TOL[dtype]
                assert rel_l2(dx, oracle.conv_bwd_data(case.dy, Wm, case.x.shape, 1)) <= TOL[dtype]
        finally:
            g.close()


@pytest.mark.parametrize("score_mode", [0, 1])
@pytest.mark.parametrize("keep_mode", [0, 1])
@pytest.mark.parametrize("with_grad", [True, False])
def test_select_modes_bit_exact(B, ctx, oracle, score_mode, keep_mode, with_grad):
    layer = I.Layer(1, 4, 4, 37, 29, 1)
    n_keep = 11 if keep_mode == 0 else 333
    case = Case(layer, "f32", 12, n_keep, tag=("modes", score_mode, keep_mode, with_grad))
    pid, kp, _, _ = oracle_masks(oracle, case, score_mode=score_mode, keep_mode=keep_mode, with_grad=with_grad)
    g = GpuLayer(B, ctx, case, score_mode=score_mode, keep_mode=keep_mode, with_grad=with_grad)
    try:
        gpid, gkeep = g.masks()
        assert np.array_equal(gpid, pid) and np.array_equal(gkeep, kp)
    finally:
        g.close()


def test_select_ties_and_zero_weights(B, ctx, oracle):
    """All-zero and constant weights: every score ties; lowest pattern id and lowest channels win."""
    import torch
    F, C, P = 3, 10, 8
    lib = I.make_library(P)
    for fill in (0.0, 1.0):
        Wn = np.full((F, C, 9), fill, np.float32)
        pid, kp = oracle.select(Wn, None, lib, 4)
        Wd = to_dev(Wn)
        gp = torch.empty((F, C), dtype=torch.uint8, device="cuda")
        gk = torch.empty((F, C), dtype=torch.uint8, device="cuda")
        B.pc_pattern_select(ctx, Wd, None, F, C, lib, 0, 4, 0, gp, gk)
        torch.cuda.synchronize()
        assert np.array_equal(gp.cpu().numpy(), pid) and np.array_equal(gk.cpu().numpy(), kp)


def test_select_full_layer_sizes_bit_exact(B, ctx, oracle):
    """Selection at the largest layer of the benchmark stacks (512x512 kernels), both score modes."""
    import torch
    F = C = 512
    for P, keep in ((8, 0.3), (16, 0.2)):
        lib = I.make_library(P)
        Wn = I.gen_weights(F, C, I.BASE_SEED, ("sel_full", P))
        Gn = I.gen_weight_grads(F, C, I.BASE_SEED, ("sel_full", P))
        k = I.kept_per_filter(keep, C)
        Wd, Gd = to_dev(Wn), to_dev(Gn)
        for sm in (0, 1):
            pid, kp = oracle.select(Wn, Gn, lib, k, score_mode=sm)
            gp = torch.empty((F, C), dtype=torch.uint8, device="cuda")
            gk = torch.empty((F, C), dtype=torch.uint8, device="cuda")
            B.pc_pattern_select(ctx, Wd, Gd, F, C, lib, 0, k, sm, gp, gk)
            torch.cuda.synchronize()
            assert np.array_equal(gp.cpu().numpy(), pid)
            assert np.array_equal(gk.cpu().numpy(), kp)
            assert int(kp.sum()) == F * k


def test_runs_are_bit_reproducible(B, ctx, oracle):
    layer = I.Layer(4, 16, 16, 64, 64, 1)
    for dtype in ("f32", "bf16"):
        case = Case(layer, dtype, 8, 19, tag=("repro", dtype))
        g = GpuLayer(B, ctx, case)
        try:
            a = (g.fwd(), g.bwd_data(), g.bwd_weight()[0])
            b = (g.fwd(), g.bwd_data(), g.bwd_weight()[0])
            for u, v in zip(a, b):
                assert np.array_equal(u, v)
        finally:
            g.close()


def test_update_values_and_repack(B, ctx, oracle):
    """pc_update_values re-gathers from new dense weights with the same tables; pc_pack can re-pack
    an existing handle with a new selection."""
    layer = I.Layer(2, 8, 8, 16, 24, 1)
    case = Case(layer, "f32", 8, 6, tag="upd")
    pid, kp, M, Wm = oracle_masks(oracle, case)
    g = GpuLayer(B, ctx, case)
    try:
        W2 = I.gen_weights(layer.F, layer.C, 99, "upd2")
        B.pc_update_values(ctx, g.pk, to_dev(W2))
        Wm2 = oracle.apply_mask(W2, M)
        assert np.array_equal(g.unpack(), Wm2)
        assert rel_l2(g.fwd(), oracle.conv_fwd(case.x, Wm2, 1)) <= 1e-4
        assert rel_l2(g.bwd_data(), oracle.conv_bwd_data(case.dy, Wm2, case.x.shape, 1)) <= 1e-4
        # new selection from the new weights, packed into the same handle
        pid3, kp3 = oracle.select(W2, None, case.lib, 9)
        M3 = oracle.mask(pid3, kp3, case.lib)
        W2d = to_dev(W2)
        B.pc_pattern_select(ctx, W2d, None, layer.F, layer.C, case.lib, 0, 9, 0, g.pid, g.keep)
        pk2 = B.pc_pack(ctx, W2d, g.pid, g.keep, layer.F, layer.C, case.lib, g.dt, reuse=g.pk)
        assert pk2 == g.pk
        g.nnzk, _ = B.pc_packed_info(ctx, g.pk)
        assert g.nnzk == 9 * layer.F
        assert np.array_equal(g.unpack(), oracle.apply_mask(W2, M3))
        assert rel_l2(g.fwd(), oracle.conv_fwd(case.x, oracle.apply_mask(W2, M3), 1)) <= 1e-4
    finally:
        g.close()


def test_select_long_rows_with_partial_ties(B, ctx, oracle):
    """Rows longer than one workgroup pass, scores from a small discrete set: the cut falls inside a run of equal
    scores in most rows, so the lowest channels of the run must win (per-filter and per-layer modes)."""
    import torch
    rng = np.random.default_rng(7)
    lib = I.make_library(12)
    for F, C, n_keep in ((5, 700, 123), (3, 1300, 1), (4, 513, 512), (2, 8192, 3000), (2, 9000, 77)):
        Wn = rng.integers(-3, 4, size=(F, C, 9)).astype(np.float32) * 0.25
        Gn = rng.integers(-2, 3, size=(F, C, 9)).astype(np.float32)
        Wd, Gd = to_dev(Wn), to_dev(Gn)
        for sm in (0, 1):
            pid, kp = oracle.select(Wn, Gn, lib, n_keep, score_mode=sm)
            gp = torch.full((F, C), 255, dtype=torch.uint8, device="cuda")
            gk = torch.full((F, C), 255, dtype=torch.uint8, device="cuda")
            B.pc_pattern_select(ctx, Wd, Gd, F, C, lib, 0, n_keep, sm, gp, gk)
            torch.cuda.synchronize()
            assert np.array_equal(gp.cpu().numpy(), pid), (F, C, n_keep, sm)
            assert np.array_equal(gk.cpu().numpy(), kp), (F, C, n_keep, sm)
            assert int(kp.sum()) == F * min(n_keep, C)


def test_select_per_layer_long_segments(B, ctx, oracle):
    """Per-layer keep mode on layers of more than 8192 kernels (the radix select runs across workgroups): random
    scores, scores with many ties at the cut, and the degenerate counts."""
    import torch
    rng = np.random.default_rng(17)
    lib = I.make_library(8)
    cases = []
    for F, C in ((29, 700), (128, 130), (512, 512)):
        Wq = rng.integers(-3, 4, size=(F, C, 9)).astype(np.float32) * 0.25
        Gq = rng.integers(-2, 3, size=(F, C, 9)).astype(np.float32)
        cases.append((Wq, Gq, [1, F * C // 3, F * C - 1, 0, F * C]))
        cases.append((I.gen_weights(F, C, I.BASE_SEED, ("perlayer", F)), I.gen_weight_grads(F, C, I.BASE_SEED, ("perlayer", F)),
                      [F * C * 3 // 10]))
    for Wn, Gn, counts in cases:
        F, C = Wn.shape[:2]
        Wd, Gd = to_dev(Wn), to_dev(Gn)
        for n_keep in counts:
            for sm in (0, 1):
                pid, kp = oracle.select(Wn, Gn, lib, n_keep, keep_mode=1, score_mode=sm)
                gp = torch.full((F, C), 255, dtype=torch.uint8, device="cuda")
                gk = torch.full((F, C), 255, dtype=torch.uint8, device="cuda")
                B.pc_pattern_select(ctx, Wd, Gd, F, C, lib, 1, n_keep, sm, gp, gk)
                torch.cuda.synchronize()
                assert np.array_equal(gp.cpu().numpy(), pid), (F, C, n_keep, sm)
                assert np.array_equal(gk.cpu().numpy(), kp), (F, C, n_keep, sm)
                assert int(kp.sum()) == n_keep


@pytest.mark.parametrize("shape", [(2, 9, 9, 40, 72, 1), (2, 8, 8, 6, 40, 1), (3, 7, 5, 130, 33, 2)])
def test_update_values_bf16_tiles(B, ctx, oracle, shape):
    """pc_update_values on a bf16 pack rebuilds the matrix-core operand tiles from the tables of the pack."""
    layer = I.Layer(*shape)
    case = Case(layer, "bf16", 8, I.kept_per_filter(0.4, layer.C), tag=("upd_bf16", shape))
    pid, kp, M, Wm = oracle_masks(oracle, case)
    g = GpuLayer(B, ctx, case)
    try:
        W2 = I.gen_weights(layer.F, layer.C, 123, ("upd_bf16_2", shape))
        B.pc_update_values(ctx, g.pk, to_dev(W2))
        Wm2 = oracle.apply_mask(oracle.bf16_round(W2), M)
        assert np.array_equal(g.unpack(), Wm2)
        assert rel_l2(g.fwd(), oracle.conv_fwd(case.x, Wm2, layer.stride)) <= 2e-2
        assert rel_l2(g.bwd_data(), oracle.conv_bwd_data(case.dy, Wm2, case.x.shape, layer.stride)) <= 2e-2
    finally:
        g.close()


@pytest.mark.parametrize("shape", [(8, 8, 8, 64, 64, 1), (5, 6, 6, 130, 72, 1), (16, 4, 4, 256, 512, 1), (3, 9, 9, 3, 64, 2)])
def test_backward_weight_without_count_readback(B, ctx, oracle, shape):
    """After a re-pack the host does not know the kept-kernel count; backward-weight then sizes its partial planes
    by the capacity of the pack and must give the same gradient, without forcing a read-back."""
    import torch
    layer = I.Layer(*shape)
    case = Case(layer, "bf16", 8, I.kept_per_filter(0.3, layer.C), tag=("nocount", shape))
    pid, kp, M, Wm = oracle_masks(oracle, case)
    g = GpuLayer(B, ctx, case)
    try:
        ref = oracle.conv_bwd_weight(case.x, case.dy, M, layer.stride)
        dw_known, guard = g.bwd_weight()
        assert rel_l2(g.scatter(guard.body), ref) <= 1e-4
        pk2 = B.pc_pack(ctx, g.W, g.pid, g.keep, layer.F, layer.C, case.lib, g.dt, reuse=g.pk)   # count unknown again
        assert pk2 == g.pk
        dw_cap, guard2 = g.bwd_weight()
        assert np.array_equal(dw_cap, dw_known)
        assert B.pc_packed_info(ctx, g.pk)[0] == g.nnzk
    finally:
        g.close()


def test_select_and_pack_replay_in_a_graph(B, oracle):
    """A step that re-selects and re-packs can be captured into a HIP graph: replays with other work between them
    give the masks, the pack and the layer outputs of the eager calls."""
    import torch
    layer = I.Layer(4, 8, 8, 64, 64, 1)
    case = Case(layer, "bf16", 8, 19, tag="graph")
    pid, kp, M, Wm = oracle_masks(oracle, case)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = B.pc_create(0, stream.cuda_stream)
        g = GpuLayer(B, ctx, case)
        try:
            y = torch.empty((layer.N, layer.Ho, layer.Wo, layer.F), dtype=torch.bfloat16, device="cuda")
            dw = torch.empty((g.nnzk, 4), dtype=torch.float32, device="cuda")

            def step():
                B.pc_pattern_select(ctx, g.W, g.G, layer.F, layer.C, case.lib, 0, case.n_keep, 0, g.pid, g.keep)
                B.pc_pack(ctx, g.W, g.pid, g.keep, layer.F, layer.C, case.lib, g.dt, reuse=g.pk)
                B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, y)
                B.pc_conv_bwd_weight(ctx, g.desc, g.pk, g.x, g.dy, dw)

            step()
            stream.synchronize()
            y_eager, dw_eager = y.clone(), dw.clone()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                step()
            for rep in range(3):
                g.pid.fill_(255); g.keep.fill_(255); y.zero_(); dw.zero_()
                (torch.ones(1 << 16, device="cuda") * 2).sum().item()       # unrelated eager work between replays
                graph.replay()
                stream.synchronize()
                assert np.array_equal(g.pid.cpu().numpy(), pid) and np.array_equal(g.keep.cpu().numpy(), kp), rep
                assert torch.equal(y, y_eager) and torch.equal(dw, dw_eager), rep
            assert B.pc_packed_info(ctx, g.pk)[0] == g.nnzk
            assert np.array_equal(g.unpack(), Wm)
        finally:
            g.close()
            B.pc_destroy(ctx)


def test_bwd_weight_on_a_second_context_and_stream(B, oracle):
    """A pack belongs to no context: a second context on a second stream runs pc_conv_bwd_weight while the first
    runs pc_conv_bwd_data (fork after the forward call, join at the end), and selects and packs every layer ahead
    of the first context's forward calls, eagerly and replayed from a HIP graph. Outputs equal those of the
    one-stream eager calls bit for bit."""
    import torch
    shapes = [I.Layer(16, 8, 8, 64, 128, 1), I.Layer(16, 4, 4, 128, 128, 1), I.Layer(8, 16, 16, 24, 64, 2)]
    main, side = torch.cuda.Stream(), torch.cuda.Stream()
    with torch.cuda.stream(main):
        ctx = B.pc_create(0, main.cuda_stream)
        ctx_w = B.pc_create(0, side.cuda_stream)
        gs = []
        try:
            for li, layer in enumerate(shapes):
                case = Case(layer, "bf16", 8, I.kept_per_filter(0.3, layer.C), tag=("two_streams", li))
                g = GpuLayer(B, ctx, case)
                g.y = torch.empty((layer.N, layer.Ho, layer.Wo, layer.F), dtype=torch.bfloat16, device="cuda")
                g.dx = torch.empty((layer.N, layer.H, layer.W, layer.C), dtype=torch.bfloat16, device="cuda")
                g.dw = torch.empty((g.nnzk, 4), dtype=torch.float32, device="cuda")
                gs.append(g)

            def prep(g, cx):
                L, c = g.case.layer, g.case
                B.pc_pattern_select(cx, g.W, g.G, L.F, L.C, c.lib, 0, c.n_keep, 0, g.pid, g.keep)
                B.pc_pack(cx, g.W, g.pid, g.keep, L.F, L.C, c.lib, g.dt, reuse=g.pk)

            def step(two):
                ready = []
                if two:                                      # selection and packing of every layer on the side stream first
                    side.wait_stream(main)
                    for g in gs:
                        prep(g, ctx_w)
                        ev = torch.cuda.Event()
                        ev.record(side)
                        ready.append(ev)
                for li, g in enumerate(gs):
                    if two:
                        main.wait_event(ready[li])
                    else:
                        prep(g, ctx)
                    B.pc_conv_fwd(ctx, g.desc, g.pk, g.x, g.y)
                    if two:
                        side.wait_stream(main)
                    B.pc_conv_bwd_data(ctx, g.desc, g.pk, g.dy, g.dx)
                    B.pc_conv_bwd_weight(ctx_w if two else ctx, g.desc, g.pk, g.x, g.dy, g.dw)
                if two:
                    main.wait_stream(side)

            def outputs():
                torch.cuda.synchronize()
                return [t.clone() for g in gs for t in (g.y, g.dx, g.dw)]

            def clear():
                for g in gs:
                    g.y.zero_(); g.dx.zero_(); g.dw.zero_(); g.pid.fill_(255); g.keep.fill_(255)

            step(False)
            ref = outputs()
            for g, (y, dx, dw) in zip(gs, zip(ref[0::3], ref[1::3], ref[2::3])):
                L, c = g.case.layer, g.case
                pid, kp, M, Wm = oracle_masks(oracle, c)
                assert rel_l2(g.scatter(dw), oracle.conv_bwd_weight(c.x, c.dy, M, L.stride)) <= 1e-4
            clear()
            step(True)                                       # eager, two streams (also grows the side context's scratch)
            assert all(torch.equal(a, b) for a, b in zip(outputs(), ref))
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=main):
                step(True)
            for rep in range(3):
                clear()
                (torch.ones(1 << 16, device="cuda") * 2).sum().item()
                graph.replay()
                assert all(torch.equal(a, b) for a, b in zip(outputs(), ref)), rep
        finally:
            torch.cuda.synchronize()
            for g in gs:
                g.close()
            B.pc_destroy(ctx_w)
            B.pc_destroy(ctx)


def test_select_and_pack_batch(B, ctx, oracle):
    """pc_pattern_select_batch and pc_pack_batch over layers of mixed shapes, dtypes and kernel families (one row too
    long for the one-workgroup kernel, one float32 layer on the gather kernels): masks bit-exact against the oracle,
    the re-packed handles hold W (.) M, their kept-kernel counts are right and a forward pass through each is within
    tolerance. The handles were first packed with other masks (selection with gradients), so a stale table would show."""
    import torch
    shapes = [(2, 6, 6, 3, 64, "bf16"), (2, 6, 6, 64, 64, "bf16"), (2, 5, 4, 64, 128, "bf16"), (2, 4, 4, 24, 40, "f32"),
              (1, 4, 4, 256, 256, "bf16"), (1, 2, 2, 9000, 8, "bf16"), (3, 3, 3, 40, 72, "bf16")]
    gs, cases = [], []
    try:
        for li, (N, H, W_, C, F, dtype) in enumerate(shapes):
            layer = I.Layer(N, H, W_, C, F, 1)
            case = Case(layer, dtype, 8, I.kept_per_filter(0.3, C), tag=("batch", li))
            cases.append(case)
            gs.append(GpuLayer(B, ctx, case))                       # select with gradients + pack, one layer at a time
        for g in gs:
            g.pid.fill_(255); g.keep.fill_(255)
        lib = cases[0].lib
        B.pc_pattern_select_batch(ctx, [g.W for g in gs], None, [c.layer.F for c in cases], [c.layer.C for c in cases], lib,
                                  B.PC_KEEP_PER_FILTER, [c.n_keep for c in cases], B.PC_SCORE_RETAINED,
                                  [g.pid for g in gs], [g.keep for g in gs])
        B.pc_pack_batch(ctx, [g.W for g in gs], [g.pid for g in gs], [g.keep for g in gs], lib, [g.pk for g in gs])
        for g, case in zip(gs, cases):
            L = case.layer
            pid, kp, M, Wm = oracle_masks(oracle, case, with_grad=False)
            gpid, gkeep = g.masks()
            assert np.array_equal(gpid, pid) and np.array_equal(gkeep, kp), L
            assert B.pc_packed_info(ctx, g.pk)[0] == int(kp.sum())
            assert np.array_equal(g.unpack(), Wm), L
            tol = 2e-2 if case.dtype == "bf16" else 1e-4
            assert rel_l2(g.fwd(), oracle.conv_fwd(case.x, Wm, 1)) <= tol, L
            dw, guard = g.bwd_weight()
            assert rel_l2(g.scatter(guard.body), oracle.conv_bwd_weight(case.x, case.dy, M, 1)) <= 1e-4, L
        # new weights, unchanged tables, all handles in one call (the per-iteration conversion of Section 5.1)
        W2 = [I.gen_weights(c.layer.F, c.layer.C, I.BASE_SEED, ("batch_new", li)) for li, c in enumerate(cases)]
        W2d = [to_dev(w) for w in W2]
        B.pc_update_values_batch(ctx, [g.pk for g in gs], W2d)
        for g, case, w2 in zip(gs, cases, W2):
            pid, kp, M, _ = oracle_masks(oracle, case, with_grad=False)
            src = oracle.bf16_round(w2) if case.dtype == "bf16" else w2
            assert np.array_equal(g.unpack(), oracle.apply_mask(src, M)), case.layer
            tol = 2e-2 if case.dtype == "bf16" else 1e-4
            assert rel_l2(g.fwd(), oracle.conv_fwd(case.x, oracle.apply_mask(src, M), 1)) <= tol, case.layer
            dx_ref = oracle.conv_bwd_data(case.dy, oracle.apply_mask(src, M), case.x.shape, 1)
            assert rel_l2(g.bwd_data(), dx_ref) <= tol, case.layer
    finally:
        for g in gs:
            g.close()


def test_select_and_pack_batch_of_many_layers(B, ctx, oracle):
    """More layers than one launch takes (40 > 32), with gradients and with one gradient pointer missing."""
    import torch
    rng = np.random.default_rng(77)
    gs, cases = [], []
    try:
        for li in range(40):
            F, C = int(rng.integers(1, 40)), int(rng.integers(1, 70))
            case = Case(I.Layer(1, 3, 3, C, F, 1), "f32" if li % 5 == 0 else "bf16", 8, I.kept_per_filter(0.4, C), tag=("many", li))
            cases.append(case)
            gs.append(GpuLayer(B, ctx, case, with_grad=False))
        for g in gs:
            g.pid.fill_(255); g.keep.fill_(255)
        Gs = [to_dev(c.G) for c in cases]
        Gs[7] = None
        lib = cases[0].lib
        B.pc_pattern_select_batch(ctx, [g.W for g in gs], Gs, [c.layer.F for c in cases], [c.layer.C for c in cases], lib,
                                  B.PC_KEEP_PER_FILTER, [c.n_keep for c in cases], B.PC_SCORE_RETAINED,
                                  [g.pid for g in gs], [g.keep for g in gs])
        B.pc_pack_batch(ctx, [g.W for g in gs], [g.pid for g in gs], [g.keep for g in gs], lib, [g.pk for g in gs])
        for li, (g, case) in enumerate(zip(gs, cases)):
            pid, kp, M, Wm = oracle_masks(oracle, case, with_grad=li != 7)
            gpid, gkeep = g.masks()
            assert np.array_equal(gpid, pid) and np.array_equal(gkeep, kp), li
            assert np.array_equal(g.unpack(), Wm), li
        with pytest.raises(B.PcError):
            B.pc_pack_batch(ctx, [gs[0].W, gs[0].W], [gs[0].pid] * 2, [gs[0].keep] * 2, lib, [gs[0].pk, gs[0].pk])
    finally:
        for g in gs:
            g.close()


def test_bwd_weight_batch_equals_the_single_calls(B, ctx, oracle):
    """pc_conv_bwd_weight_batch over layers of every kind (3 input channels: padded copy; a filter count the
    wave-specialised kernel does not take; a float32 layer on the gather kernels; stride 2; a layer with as many tiles
    as CUs, i.e. no split; a pack whose count is not known on the host): within tolerance of the oracle and of
    pc_conv_bwd_weight layer by layer (the split of a layer, hence the float32 order of additions, may differ), and
    the same bits from call to call."""
    import torch
    shapes = [(8, 8, 8, 3, 64, 1, "bf16"), (8, 8, 8, 64, 64, 1, "bf16"), (4, 6, 6, 40, 36, 1, "bf16"), (2, 5, 5, 16, 24, 1, "f32"),
              (8, 9, 9, 64, 128, 2, "bf16"), (2, 2, 2, 1024, 1024, 1, "bf16"), (16, 4, 4, 256, 128, 1, "bf16")]
    gs, cases = [], []
    try:
        for li, (N, H, W_, C, F, st, dtype) in enumerate(shapes):
            case = Case(I.Layer(N, H, W_, C, F, st), dtype, 8, I.kept_per_filter(0.3, C), tag=("wgb", li))
            cases.append(case)
            gs.append(GpuLayer(B, ctx, case))
        single = []
        for g in gs:
            dw, guard = g.bwd_weight()
            single.append(guard.body.clone())
        # the last pack again without a read-back of its count: planes strided by the capacity
        g = gs[-1]
        B.pc_pack(ctx, g.W, g.pid, g.keep, cases[-1].layer.F, cases[-1].layer.C, cases[-1].lib, g.dt, reuse=g.pk)
        from tests._harness import Guarded
        outs = [Guarded(g.nnzk * 4, torch.float32) for g in gs]
        B.pc_conv_bwd_weight_batch(ctx, [g.desc for g in gs], [g.pk for g in gs], [g.x for g in gs], [g.dy for g in gs],
                                   [o.ptr for o in outs])
        torch.cuda.synchronize()
        for g, case, o, ref in zip(gs, cases, outs, single):
            assert o.margins_intact(), case.layer
            assert rel_l2(o.body.cpu().numpy(), ref.cpu().numpy()) <= 1e-5, case.layer
            pid, kp, M, Wm = oracle_masks(oracle, case)
            assert rel_l2(g.scatter(o.body), oracle.conv_bwd_weight(case.x, case.dy, M, case.layer.stride)) <= 1e-4, case.layer
        again = [Guarded(g.nnzk * 4, torch.float32) for g in gs]
        B.pc_conv_bwd_weight_batch(ctx, [g.desc for g in gs], [g.pk for g in gs], [g.x for g in gs], [g.dy for g in gs],
                                   [o.ptr for o in again])
        torch.cuda.synchronize()
        assert all(torch.equal(a.body, o.body) for a, o in zip(again, outs))
    finally:
        for g in gs:
            g.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("workload", ["vgg16_cifar", "resnet18_cifar", "resnet50_imagenet", "vgg16_imagenet"])
def test_bwd_weight_batch_full_size(B, ctx, oracle, workload):
    """All layers of a benchmark workload at its batch size in one call -- the launch bench.py times, with the
    per-layer splits that exist only at full size -- against the oracle: for every layer one kept tap in every
    32 x 32 block of (filter, channel) plus 192 anywhere, each within its per-element bound. Layers of equal shape
    share their seeded inputs (every layer still has its own output buffer). Also close to the single-layer call."""
    import torch
    from tests.test_gpu_fullsize import sample_kept_taps
    wl = I.WORKLOADS[workload]
    rng = np.random.default_rng(4242)
    by_shape = {}
    gs, outs = [], []
    try:
        for li, L in enumerate(wl.layers):
            if L not in by_shape:
                say("  layer", li, L)
                case = Case(L, wl.dtype, wl.P, I.kept_per_filter(wl.keep, L.C), tag=("wgfull", workload, li))
                by_shape[L] = GpuLayer(B, ctx, case)
            gs.append(by_shape[L])
        outs = [torch.full((g.nnzk, 4), float("nan"), dtype=torch.float32, device="cuda") for g in gs]
        B.pc_conv_bwd_weight_batch(ctx, [g.desc for g in gs], [g.pk for g in gs], [g.x for g in gs], [g.dy for g in gs], outs)
        torch.cuda.synchronize()
        checked = {}
        for li, (g, o) in enumerate(zip(gs, outs)):
            L, case = g.case.layer, g.case
            assert torch.isfinite(o).all(), (workload, li)
            if L in checked:                                  # same inputs, same plan: the same bits
                assert torch.equal(o, outs[checked[L]]), (workload, li)
                continue
            checked[L] = li
            pid, kp = g.masks()
            dw = o.cpu().numpy()
            widx, slots, js = sample_kept_taps(oracle, case, pid, kp, rng)
            assert_close(dw[slots, js], oracle.conv_bwd_weight_at(case.x, case.dy, L.F, L.stride, widx),
                         oracle.conv_bwd_weight_at(case.x, np.abs(case.dy), L.F, L.stride, widx), "f32", TOL_DW,
                         "%s layer %d grouped bwd_weight, %d samples" % (workload, li, widx.size))
            single = torch.full((g.nnzk, 4), float("nan"), dtype=torch.float32, device="cuda")
            B.pc_conv_bwd_weight(ctx, g.desc, g.pk, g.x, g.dy, single)
            torch.cuda.synchronize()
            assert rel_l2(dw, single.cpu().numpy()) <= 1e-5, (workload, li)
    finally:
        for g in by_shape.values():
            g.close()


def test_bwd_weight_batch_of_more_layers_than_one_launch_takes(B, ctx, oracle):
    """23 layers (a launch takes 20, and so does the grouped reduction): every layer within tolerance of its own call
    and of the oracle."""
    import torch
    rng = np.random.default_rng(91)
    gs, cases = [], []
    try:
        for li in range(23):
            C, F = int(rng.choice([8, 16, 40, 64])), int(rng.choice([8, 24, 64, 72]))
            layer = I.Layer(int(rng.choice([2, 8, 16])), int(rng.choice([3, 4, 8])), int(rng.choice([3, 4, 8])), C, F, 1)
            case = Case(layer, "bf16", 8, I.kept_per_filter(0.5, C), tag=("wgb23", li))
            cases.append(case)
            gs.append(GpuLayer(B, ctx, case))
        refs = []
        for g in gs:
            refs.append(g.bwd_weight()[1].body.clone())
        outs = [torch.full((g.nnzk, 4), float("nan"), dtype=torch.float32, device="cuda") for g in gs]
        B.pc_conv_bwd_weight_batch(ctx, [g.desc for g in gs], [g.pk for g in gs], [g.x for g in gs], [g.dy for g in gs], outs)
        torch.cuda.synchronize()
        for li, (g, case, o, r) in enumerate(zip(gs, cases, outs, refs)):
            assert torch.isfinite(o).all(), li
            assert rel_l2(o.cpu().numpy(), r.cpu().numpy()) <= 1e-5, li
            pid, kp, M, Wm = oracle_masks(oracle, case)
            assert rel_l2(g.scatter(o), oracle.conv_bwd_weight(case.x, case.dy, M, 1)) <= 1e-4, li
    finally:
        for g in gs:
            g.close()


def test_graph_survives_a_later_growth_of_the_scratch_buffer(B, oracle):
    """A graph captured while the context's scratch buffer was small is replayed after a larger layer made the buffer
    grow: the superseded buffer is kept until pc_destroy, so the replay gives the eager result."""
    import torch
    small = Case(I.Layer(8, 8, 8, 64, 64, 1), "bf16", 8, 19, tag="grow_small")
    big = Case(I.Layer(16, 8, 8, 512, 512, 1), "bf16", 8, 154, tag="grow_big")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ctx = B.pc_create(0, stream.cuda_stream)
        gs = GpuLayer(B, ctx, small)
        gb = GpuLayer(B, ctx, big)
        try:
            dw = torch.empty((gs.nnzk, 4), dtype=torch.float32, device="cuda")
            B.pc_conv_bwd_weight(ctx, gs.desc, gs.pk, gs.x, gs.dy, dw)          # scratch reaches the small layer's size
            stream.synchronize()
            ref = dw.clone()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                B.pc_conv_bwd_weight(ctx, gs.desc, gs.pk, gs.x, gs.dy, dw)
            dwb = torch.empty((gb.nnzk, 4), dtype=torch.float32, device="cuda")
            # re-packed without a read-back of the count: the partial planes are strided by the capacity, 4 x 512 x 512
            # slots of 16 bytes, several times the small layer's need, so a larger buffer replaces the first
            B.pc_pack(ctx, gb.W, gb.pid, gb.keep, 512, 512, big.lib, gb.dt, reuse=gb.pk)
            B.pc_conv_bwd_weight(ctx, gb.desc, gb.pk, gb.x, gb.dy, dwb)
            B.pc_conv_bwd_weight_batch(ctx, [gs.desc, gb.desc], [gs.pk, gb.pk], [gs.x, gb.x], [gs.dy, gb.dy],
                                       [torch.empty_like(dw), torch.empty_like(dwb)])  # and a larger one again
            stream.synchronize()
            for rep in range(2):
                dw.zero_()
                graph.replay()
                stream.synchronize()
                assert torch.equal(dw, ref), rep
            pid, kp, M, Wm = oracle_masks(oracle, big)
            assert rel_l2(gb.scatter(dwb), oracle.conv_bwd_weight(big.x, big.dy, M, 1)) <= 1e-4
        finally:
            gs.close()
            gb.close()
            B.pc_destroy(ctx)


def test_mismatched_descriptor_is_rejected(B, ctx, oracle):
    layer = I.Layer(1, 4, 4, 8, 8, 1)
    case = Case(layer, "f32", 4, 4, tag="mismatch")
    g = GpuLayer(B, ctx, case)
    try:
        import torch
        y = torch.zeros(1 * 4 * 4 * 8, device="cuda")
        bad = B.make_desc(1, 4, 4, 9, 8, 1, B.PC_F32)
        with pytest.raises(B.PcError) as ei:
            B.pc_conv_fwd(ctx, bad, g.pk, g.x, y)
        assert ei.value.status == B.PC_ERR_INVALID_ARG
        bad = B.make_desc(1, 4, 4, 8, 8, 1, B.PC_BF16)
        with pytest.raises(B.PcError):
            B.pc_conv_fwd(ctx, bad, g.pk, g.x, y)
        bad = B.make_desc(1, 4, 4, 8, 8, 3, B.PC_F32)
        with pytest.raises(B.PcError) as ei:
            B.pc_conv_fwd(ctx, bad, g.pk, g.x, y)
        assert ei.value.status == B.PC_ERR_BAD_SHAPE
        with pytest.raises(B.PcError) as ei:
            B.pc_pattern_select(ctx, g.W, None, 8, 8, [0b111], 0, 1, 0, g.pid, g.keep)
        assert ei.value.status == B.PC_ERR_BAD_LIBRARY
        with pytest.raises(B.PcError):
            B.pc_pattern_select(ctx, g.W, None, 8, 8, case.lib, 0, 9, 0, g.pid, g.keep)   # n_keep > C
    finally:
        g.close()

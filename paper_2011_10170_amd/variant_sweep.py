"""Per-layer operator choice as a function of sparsity (the analogue of the paper's sparsity sweep, Section 5.2 /
Figure 10, and of its compile-time choice between the sparse and the dense operator, Section 5.4).

For one bf16 layer shape and a range of connectivity keep ratios it times the three passes with the
pattern-grouped gather kernels (only kept taps are multiplied: time follows the density keep * 4/9) and with the
matrix-core kernels (zero-filled tiles: time independent of the density), and prints the ratio at which they
cross. Synthetic seeded inputs; every call runs in the library's kernels.

    python -m paper_2011_10170_amd.variant_sweep --shape 128,8,8,256,256,1 --patterns 8
"""
from __future__ import annotations

import argparse
import sys


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="128,8,8,256,256,1", help="N,H,W,C,F,stride")
    ap.add_argument("--patterns", type=int, default=8)
    ap.add_argument("--keeps", default="0.02,0.05,0.1,0.15,0.2,0.3,0.5,0.75,1.0")
    ap.add_argument("--reps", type=int, default=10)
    args = ap.parse_args()

    import torch
    from . import binding as B
    from . import inputs as I

    if not torch.cuda.is_available():
        print("variant_sweep: no GPU visible", file=sys.stderr)
        return 2
    B.load()
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)
    ctx = B.pc_create(0, stream.cuda_stream)
    N, H, W_, C, F, stride = (int(v) for v in args.shape.split(","))
    L = I.Layer(N, H, W_, C, F, stride)
    lib = I.make_library(args.patterns)

    def dev(a):
        import numpy as np
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    Wd = dev(I.gen_weights(F, C, I.BASE_SEED, "sweep"))
    Gd = dev(I.gen_weight_grads(F, C, I.BASE_SEED, "sweep"))
    x = dev(I.gen_activations((N, H, W_, C), I.BASE_SEED, ("sweep", "x"), True, "bf16")[1])
    dy = dev(I.gen_activations((N, L.Ho, L.Wo, F), I.BASE_SEED, ("sweep", "dy"), False, "bf16")[1])
    y = torch.empty_like(dy)
    dx = torch.empty_like(x)
    desc = B.make_desc(N, H, W_, C, F, stride, B.PC_BF16)
    pid = torch.empty((F, C), dtype=torch.uint8, device="cuda")
    keep = torch.empty((F, C), dtype=torch.uint8, device="cuda")

    def time_passes(pk, dw):
        def step():
            B.pc_conv_fwd(ctx, desc, pk, x, y)
            B.pc_conv_bwd_data(ctx, desc, pk, dy, dx)
            B.pc_conv_bwd_weight(ctx, desc, pk, x, dy, dw)
        step()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            step()
        g.replay()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(args.reps):
            g.replay()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / args.reps

    print("layer N=%d %dx%d %d->%d stride %d, %d patterns, bf16; us for fwd + bwd_data + bwd_weight" % (
        N, H, W_, C, F, stride, args.patterns))
    print("%6s %8s %9s %10s %10s %8s" % ("keep", "density", "sparsity", "gather us", "matrix us", "ratio"))
    rows = []
    for ks in args.keeps.split(","):
        kr = float(ks)
        k = I.kept_per_filter(kr, C)
        B.pc_pattern_select(ctx, Wd, Gd, F, C, lib, B.PC_KEEP_PER_FILTER, k, B.PC_SCORE_RETAINED, pid, keep)
        t = {}
        for name, var in (("valu", B.PC_VARIANT_VALU), ("mfma", B.PC_VARIANT_MFMA)):
            B.pc_set_variant(ctx, var)
            pk = B.pc_pack(ctx, Wd, pid, keep, F, C, lib, B.PC_BF16)
            nnzk, _ = B.pc_packed_info(ctx, pk)
            dw = torch.empty((max(nnzk, 1), 4), dtype=torch.float32, device="cuda")
            t[name] = time_passes(pk, dw)
            torch.cuda.synchronize()
            B.pc_packed_free(pk)
        dens = k / C * 4.0 / 9.0
        rows.append((dens, t["valu"], t["mfma"]))
        print("%6.2f %8.3f %9.3f %10.1f %10.1f %8.2f" % (k / C, dens, 1.0 - dens, t["valu"], t["mfma"], t["valu"] / t["mfma"]), flush=True)
    cross = None
    for (d0, v0, m0), (d1, v1, m1) in zip(rows, rows[1:]):
        if (v0 - m0) * (v1 - m1) <= 0 and v1 != v0:
            # linear interpolation of (gather - matrix) between the two densities
            f0, f1 = v0 - m0, v1 - m1
            cross = d0 + (d1 - d0) * (0 - f0) / (f1 - f0) if f1 != f0 else d0
            break
    if cross is not None:
        print("crossover: the gather kernels win below a weight density of about %.3f (sparsity above %.1f %%)" % (cross, 100 * (1 - cross)))
    elif rows and rows[0][1] > rows[0][2]:
        print("the matrix-core kernels win at every density of the sweep (lowest: %.3f)" % rows[0][0])
    else:
        print("the gather kernels win at every density of the sweep")
    B.pc_destroy(ctx)
    return 0


if __name__ == "__main__":
    sys.exit(main())

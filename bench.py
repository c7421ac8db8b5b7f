#!/usr/bin/env python3
"""Benchmark of the pattern-sparse convolution hot path on one MI355X.

One step = pc_conv_fwd + pc_conv_bwd_data + pc_conv_bwd_weight over every layer of the workload
(plus pc_pattern_select + pc_pack over all layers when the workload's step includes re-selection), on
seeded synthetic inputs already resident in HBM. Prints ONE JSON line on stdout; a per-layer table
goes to stderr. The default workload is the largest single-GPU configuration: the VGG-16 / ImageNet
stack at batch 32 with re-selection and re-packing inside the step.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload vgg16_imagenet] [--variant auto|valu|mfma]
    python bench.py --sweep          # also: gather vs matrix-core kernels over keep ratios (the "sweep" object)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_BF16_MFMA_TFLOPS = 2500.0
PEAK_F32_VALU_TFLOPS = 157.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="vgg16_imagenet")
    ap.add_argument("--variant", default="auto", choices=["auto", "valu", "mfma", "sparse"],
                    help="kernel family of the packs: automatic, the gather kernels, the zero-filled matrix-core kernels, or the "
                         "structured-sparse matrix-core kernels for the layers they take")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every step from the host instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy-mb", type=int, default=0,
                    help="also run one plain device copy of this many MiB (reference for scaling HBM counters)")
    ap.add_argument("--cpu-sample-batch", type=int, default=0,
                    help="images per layer the CPU oracle is timed on (0: as many as take it about 15 s at 5 nonzero GFLOP/s)")
    ap.add_argument("--sweep", action="store_true",
                    help="also time one bf16 layer over a range of keep ratios with the gather kernels and with the "
                         "matrix-core kernels (the per-layer operator choice of Section 5.2 / 5.4); adds the 'sweep' object")
    ap.add_argument("--sweep-shape", default="128,8,8,256,256,1", help="N,H,W,C,F,stride of the swept layer")
    ap.add_argument("--update-values", action="store_true",
                    help="re-gather the kept weights of every layer in the step (pc_update_values: the per-iteration conversion of Section 5.1)")
    ap.add_argument("--no-paper-context", action="store_true", help="skip the paper's demonstration layer (profiles of the workload alone)")
    ap.add_argument("--wgrad-streams", type=int, default=1,
                    help="enqueue bwd_weight on this many side streams in turn (one context each), forked after the layer's "
                         "forward call and joined at the end of the step: it overlaps bwd_data of the same layer and what follows")
    ap.add_argument("--no-prep-overlap", action="store_true",
                    help="keep selection and packing (or the value update) of a step on the main stream, before each layer's "
                         "forward call, instead of running them for all layers on the side stream from the start of the step")
    ap.add_argument("--wgrad", default="auto", choices=["auto", "group", "layer"],
                    help="group: one pc_conv_bwd_weight_batch call for all layers at the end of the step (a layer's weight "
                         "gradient needs only its own x and dy, so it can wait until all of them exist); layer: "
                         "pc_conv_bwd_weight per layer, on the side stream when there is one; auto: the faster of the two "
                         "in a short trial before the timed steps")
    ap.add_argument("--no-batch-prep", action="store_true",
                    help="select and pack layer by layer (pc_pattern_select, pc_pack) instead of all layers per launch "
                         "(pc_pattern_select_batch, pc_pack_batch)")
    ap.add_argument("--chained", action="store_true", help="(the default where the workload is a chain of layers; kept for old command lines)")
    ap.add_argument("--no-chained", action="store_true",
                    help="skip the second measurement of a VGG workload: its layers as one network, forward through every "
                         "layer with ReLU and 2x2 max pooling between them, then backward in reverse order")
    ap.add_argument("--train-steps", action="store_true",
                    help="also time pool generation, finalisation counters and the group-lasso gradient over the workload's layers")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the batch would shard across GPUs with one "
              "all-reduce of the compact weight gradient); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2011_10170_amd import binding as B
    from paper_2011_10170_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    B.load()   # raises if the HIP library is missing: there is no fallback
    wl = I.WORKLOADS[args.workload]
    dt = B.PC_BF16 if wl.dtype == "bf16" else B.PC_F32
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    esz = 2 if wl.dtype == "bf16" else 4
    stream = torch.cuda.Stream()          # every library call and every event of this run uses this stream
    torch.cuda.set_stream(stream)
    ctx = B.pc_create(0, stream.cuda_stream)
    B.pc_set_variant(ctx, {"auto": B.PC_VARIANT_AUTO, "valu": B.PC_VARIANT_VALU, "mfma": B.PC_VARIANT_MFMA, "sparse": B.PC_VARIANT_MFMA_SPARSE}[args.variant])
    # a pack belongs to no context: another context on another stream may use it, ordered by events
    streams_w = [torch.cuda.Stream() for _ in range(args.wgrad_streams)]
    ctxs_w = [B.pc_create(0, s.cuda_stream) for s in streams_w]
    lib = I.make_library(wl.P)

    def up(arr):
        if arr.dtype == np.uint16:
            return torch.from_numpy(arr.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(np.ascontiguousarray(arr)).cuda()

    # ---- set-up: inputs to HBM, selection and packing once
    t_setup = time.time()
    layers = []
    for li, L in enumerate(wl.layers):
        tag = (wl.name, li)
        W = up(I.gen_weights(L.F, L.C, I.BASE_SEED, tag))
        G = up(I.gen_weight_grads(L.F, L.C, I.BASE_SEED, tag))
        x = up(I.gen_activations((L.N, L.H, L.W, L.C), I.BASE_SEED, (tag, "x"), True, wl.dtype)[1])
        dy = up(I.gen_activations((L.N, L.Ho, L.Wo, L.F), I.BASE_SEED, (tag, "dy"), False, wl.dtype)[1])
        k = I.kept_per_filter(wl.keep, L.C)
        pid = torch.empty((L.F, L.C), dtype=torch.uint8, device="cuda")
        keep = torch.empty((L.F, L.C), dtype=torch.uint8, device="cuda")
        B.pc_pattern_select(ctx, W, G, L.F, L.C, lib, B.PC_KEEP_PER_FILTER, k, B.PC_SCORE_RETAINED, pid, keep)
        pk = B.pc_pack(ctx, W, pid, keep, L.F, L.C, lib, dt)
        nnzk, variant = B.pc_packed_info(ctx, pk)
        assert nnzk == k * L.F
        layers.append(dict(
            L=L, W=W, G=G, x=x, dy=dy, k=k, pid=pid, keep=keep, pk=pk, nnzk=nnzk, variant=variant,
            desc=B.make_desc(L.N, L.H, L.W, L.C, L.F, L.stride, dt),
            y=torch.empty((L.N, L.Ho, L.Wo, L.F), dtype=tdt, device="cuda"),
            dx=torch.empty((L.N, L.H, L.W, L.C), dtype=tdt, device="cuda"),
            dw=torch.empty((max(nnzk, 1), 4), dtype=torch.float32, device="cuda"),
            flops=8.0 * L.N * L.Ho * L.Wo * nnzk,                  # nonzero MACs x 2, per pass
            dense_flops=18.0 * L.N * L.Ho * L.Wo * L.F * L.C,      # what a zero-filled contraction issues
            act_in=L.N * L.H * L.W * L.C * esz, act_out=L.N * L.Ho * L.Wo * L.F * esz,
        ))
    torch.cuda.synchronize()
    log("set-up %.1f s, %d layers, workload %s" % (time.time() - t_setup, len(layers), wl.name))

    def run_pass(d, which, ctx=ctx):
        if which == "select":
            B.pc_pattern_select(ctx, d["W"], d["G"], d["L"].F, d["L"].C, lib, B.PC_KEEP_PER_FILTER, d["k"],
                                B.PC_SCORE_RETAINED, d["pid"], d["keep"])
        elif which == "update":
            B.pc_update_values(ctx, d["pk"], d["W"])
        elif which == "pack":
            B.pc_pack(ctx, d["W"], d["pid"], d["keep"], d["L"].F, d["L"].C, lib, dt, reuse=d["pk"])
        elif which == "fwd":
            B.pc_conv_fwd(ctx, d["desc"], d["pk"], d["x"], d["y"])
        elif which == "bwd_data":
            B.pc_conv_bwd_data(ctx, d["desc"], d["pk"], d["dy"], d["dx"])
        else:
            B.pc_conv_bwd_weight(ctx, d["desc"], d["pk"], d["x"], d["dy"], d["dw"])

    passes = (["select", "pack"] if wl.with_select else (["update"] if args.update_values else [])) + ["fwd", "bwd_data", "bwd_weight"]

    prep = [w for w in passes if w in ("select", "pack", "update")]
    batch_prep = bool(prep) and not args.no_batch_prep
    mode = {"wgrad": "group" if args.wgrad == "auto" else args.wgrad}

    def wgrad_batch(c, lo, hi):
        ls = layers[lo:hi]
        B.pc_conv_bwd_weight_batch(c, [d["desc"] for d in ls], [d["pk"] for d in ls], [d["x"] for d in ls],
                                   [d["dy"] for d in ls], [d["dw"] for d in ls])

    def run_batch(which, ctx=ctx):
        if which == "update":
            B.pc_update_values_batch(ctx, [d["pk"] for d in layers], [d["W"] for d in layers])
        elif which == "select":
            B.pc_pattern_select_batch(ctx, [d["W"] for d in layers], [d["G"] for d in layers], [d["L"].F for d in layers],
                                      [d["L"].C for d in layers], lib, B.PC_KEEP_PER_FILTER, [d["k"] for d in layers],
                                      B.PC_SCORE_RETAINED, [d["pid"] for d in layers], [d["keep"] for d in layers])
        else:
            B.pc_pack_batch(ctx, [d["W"] for d in layers], [d["pid"] for d in layers], [d["keep"] for d in layers], lib,
                            [d["pk"] for d in layers])

    def step(events=None):
        overlap = bool(ctxs_w) and events is None
        # selection and packing need only W and G, which exist when the step starts. Layer by layer
        # (--no-batch-prep, or the value update) they are enqueued on the side stream for all layers first, and the
        # main stream waits for a layer's pack before its forward call
        prep_side = overlap and bool(prep) and not args.no_prep_overlap
        ready = []
        if batch_prep:
            # all layers per launch: three launches at the start of the step, nothing left to overlap
            for which in prep:
                if events is not None:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                run_batch(which)
                if events is not None:
                    e1.record(stream)
                    events.append((-1, which, e0, e1, {"select": "pc_pattern_select_batch", "pack": "pc_pack_batch",
                                                       "update": "pc_update_values_batch"}[which]))
        elif prep_side:
            streams_w[0].wait_stream(stream)
            for d in layers:
                for which in prep:
                    run_pass(d, which, ctxs_w[0])
                ev = torch.cuda.Event()
                ev.record(streams_w[0])
                ready.append(ev)
        wg = mode["wgrad"]
        for li, d in enumerate(layers):
            if ready:
                stream.wait_event(ready[li])
            for which in passes:
                if (batch_prep or prep_side) and which in prep:
                    continue
                if wg != "layer" and which == "bwd_weight":
                    continue
                if events is not None:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                if overlap and which == "bwd_data":
                    streams_w[li % len(ctxs_w)].wait_stream(stream)    # fork: x, dy and the pack of this layer are ready
                if overlap and which == "bwd_weight":
                    B.pc_conv_bwd_weight(ctxs_w[li % len(ctxs_w)], d["desc"], d["pk"], d["x"], d["dy"], d["dw"])
                else:
                    run_pass(d, which)
                if events is not None:
                    e1.record(stream)
                    events.append((li, which, e0, e1, B.pc_last_kernel(ctx) if which in ("fwd", "bwd_data", "bwd_weight")
                                   else {"select": "pc_pattern_select", "pack": "pc_pack", "update": "pc_update_values"}[which]))
        if wg == "group":
            if events is not None:
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
            wgrad_batch(ctx, 0, len(layers))
            if events is not None:
                e1.record(stream)
                events.append((-1, "bwd_weight", e0, e1, B.pc_last_kernel(ctx)))
        if overlap:
            for s_w in streams_w:
                stream.wait_stream(s_w)                # join: the step ends when every stream has drained

    # The step is launch-bound on the host (dozens of short kernels), so it is captured once into a HIP graph
    # and replayed; no call of the step reads anything back to the host, re-selection and re-packing included.
    use_graph = not args.no_graph
    for _ in range(max(1, args.warmup if not use_graph else 1)):
        step()
    torch.cuda.synchronize()
    graph = None
    if use_graph:
        def capture():
            step()                                         # eager once: scratch buffers reach their size outside the capture
            torch.cuda.synchronize()
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr, stream=stream):
                step()
            torch.cuda.synchronize()
            return gr
        if args.wgrad == "auto":
            # where the weight gradients run is a launch choice: try both placements for a few replays, keep the faster.
            # Every candidate first runs eagerly, so that each context's scratch buffer has its final size before
            # any graph is captured (no allocation may happen during a capture).
            cands = ["group", "layer"]
            for cand in cands:
                mode["wgrad"] = cand
                step()
            torch.cuda.synchronize()
            graphs = {}
            for cand in cands:
                mode["wgrad"] = cand
                graphs[cand] = capture()
            trial = {c: float("inf") for c in cands}
            mode["trial_ms"] = trial
            for _ in range(2):                                  # alternate, keep each candidate's best
                for cand in cands:
                    for _ in range(5):
                        graphs[cand].replay()
                    torch.cuda.synchronize()
                    tt = time.perf_counter()
                    for _ in range(10):
                        graphs[cand].replay()
                    torch.cuda.synchronize()
                    trial[cand] = min(trial[cand], (time.perf_counter() - tt) * 1e2)
            mode["wgrad"] = min(trial, key=trial.get)
            log("weight-gradient placement: " + ", ".join("%s %.4f ms" % (c, v) for c, v in trial.items()) + " -> " + mode["wgrad"])
            graph = graphs[mode["wgrad"]]
            del graphs
        else:
            graph = capture()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        if graph is not None:
            graph.replay()
        else:
            step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    total_flops = sum(3.0 * d["flops"] for d in layers)
    value = total_flops / (ms_per_step * 1e-3) / 1e12

    # ---- per-call durations inside the same step sequence (library kernels run on torch's current stream), and the
    # kernel symbol that served each call (pc_last_kernel)
    events = []
    n_inst = max(3, min(args.steps, 10))
    for _ in range(n_inst):
        step(events)
    torch.cuda.synchronize()
    per_call = {}
    sym_of = {}
    for li, which, e0, e1, sym in events:
        per_call.setdefault((li, which), []).append(e0.elapsed_time(e1))
        sym_of[(li, which)] = sym
    # Roofline time of a call = max(algorithmic bytes / HBM peak, nonzero flops / peak of the unit that multiplies):
    # the method's own work, i.e. |in| + |out| + the kept weights, and 8*N*Ho*Wo*nnzk flops per pass -- never the
    # zero-filled flops the matrix-core kernels issue (those give "mfma_util", reported beside it). The unit peak is
    # the bf16 matrix rate for the matrix-core kernels and the float32 vector rate for the gather kernels; select
    # and pack are priced by bytes alone.
    calls = []
    log("%-3s %-22s %-10s %9s %9s %8s %6s %6s  %s" % ("#", "layer", "pass", "us", "nz TF/s", "GB/s", "roof", "mfma", "kernel"))
    for (li, which), ts in sorted(per_call.items()):
        d = layers[li]
        L = d["L"]
        us = float(np.median(ts)) * 1e3
        sym = sym_of[(li, which)]
        if which in ("select", "pack", "update"):
            n_pos = sum(x["L"].F * x["L"].C for x in layers) if li < 0 else L.F * L.C   # li = -1: one call for all layers
            byts = n_pos * (74.0 if which == "select" else 38.0)
            fl = dfl = 0.0
            mfma = False
        elif li < 0:                                         # the weight gradients of all layers in one call
            mfma = all(x["variant"] in (B.PC_VARIANT_MFMA, B.PC_VARIANT_MFMA_SPARSE) for x in layers)
            fl, dfl = sum(x["flops"] for x in layers), sum(x["dense_flops"] for x in layers)
            byts = float(sum(x["act_in"] + x["act_out"] + 16 * x["nnzk"] for x in layers))
        else:
            mfma = d["variant"] in (B.PC_VARIANT_MFMA, B.PC_VARIANT_MFMA_SPARSE)
            fl, dfl = d["flops"], d["dense_flops"]
            wbytes = d["nnzk"] * (4 * esz + 2)
            byts = float(d["act_in"] + d["act_out"] + (16 * d["nnzk"] if which == "bwd_weight" else wbytes))
        unit_peak = PEAK_BF16_MFMA_TFLOPS if mfma else PEAK_F32_VALU_TFLOPS
        t_hbm_us = byts / (PEAK_HBM_GBS * 1e3)
        t_unit_us = fl / (unit_peak * 1e6)
        c = dict(li=li, which=which, sym=sym, family=sym.split("<")[0], us=us, bytes=byts, flops=fl, dense=dfl if mfma else 0.0,
                 mfma=mfma, unit_peak=unit_peak, t_roof=max(t_hbm_us, t_unit_us),
                 t_sparse=max(t_hbm_us, fl / (PEAK_F32_VALU_TFLOPS * 1e6)))
        calls.append(c)
        log("%-3d %-22s %-10s %9.1f %9.2f %8.0f %6.3f %6.3f  %s" % (
            li, "all %d layers" % len(layers) if li < 0 else "%dx%d %d->%d s%d" % (L.H, L.W, L.C, L.F, L.stride), which, us,
            fl / us / 1e6, byts / us / 1e3, c["t_roof"] / us, c["dense"] / us / 1e6 / PEAK_BF16_MFMA_TFLOPS, sym))

    def summarise(cs):
        us = sum(c["us"] for c in cs)
        byts, fl, dense = sum(c["bytes"] for c in cs), sum(c["flops"] for c in cs), sum(c["dense"] for c in cs)
        unit_peak = cs[0]["unit_peak"]
        t_hbm, t_unit = byts / (PEAK_HBM_GBS * 1e3), fl / (unit_peak * 1e6)
        if t_hbm >= t_unit:
            bound, unit, peak, ach = "hbm", "GB/s", PEAK_HBM_GBS, byts / us / 1e3
        else:
            bound, unit, peak = ("mfma" if cs[0]["mfma"] else "alu"), "TFLOP/s", unit_peak
            ach = fl / us / 1e6
        return dict(launches_per_step=len(cs), avg_launch_us=round(us / len(cs), 2), bound=bound, achieved=round(ach, 3), peak=peak,
                    unit=unit, frac=round(ach / peak, 4), algorithmic_mib_per_launch=round(byts / len(cs) / (1 << 20), 2),
                    nonzero_gflop_per_launch=round(fl / len(cs) / 1e9, 3), algorithmic_gbs=round(byts / us / 1e3, 1),
                    nonzero_tflops=round(fl / us / 1e6, 3),
                    mfma_util=round(dense / us / 1e6 / PEAK_BF16_MFMA_TFLOPS, 4) if cs[0]["mfma"] else None,
                    ideal_sparse_frac=round(sum(c["t_sparse"] for c in cs) / us, 4), total_us=round(us, 1))

    # the dominant kernel: the kernel family (symbol without template arguments) with the largest share of the step;
    # every instantiation of it is listed with the same figures, so each can be held against a line of a kernel trace
    fams, syms = {}, {}
    for c in calls:
        fams.setdefault(c["family"], []).append(c)
        syms.setdefault(c["sym"], []).append(c)
    dk, dcs = max(fams.items(), key=lambda kv: sum(c["us"] for c in kv[1]))
    dom = summarise(dcs)
    t_all = sum(c["us"] for c in calls)
    # HBM bytes per launch of that kernel from the committed rocprofv3 counter summary (None when absent): the rows of
    # the family, plus the helper kernels that belong to the same library calls
    traffic = None
    prof = os.path.join(ROOT, "profiles", "%s_hbm_counters.md" % wl.name)
    helpers = {"pc_mfma_wgrad_ws_kernel": ("pc_wgrad_reduce", "pc_pad_channels_kernel"),
               "pc_mfma_wgrad_ws_group_kernel": ("pc_wgrad_reduce", "pc_pad_channels_kernel"),
               "pc_mfma_wgrad_kernel": ("pc_wgrad_reduce",), "pc_wgrad_valu_kernel": ("pc_wgrad_reduce",),
               "pc_mfma_conv_ks_kernel": (), "pc_mfma_conv_kernel": ("pc_mfma_splitk_reduce_kernel",)}.get(dk, ())
    if os.path.exists(prof):
        tot_b, tot_n = 0.0, 0
        for line in open(prof):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) > 5 and (cells[1].split("<")[0] == dk or any(cells[1].startswith(h) for h in helpers)):
                try:
                    n_disp = int(cells[2])
                    tot_b += float(cells[5].split("=")[-1]) * n_disp
                except ValueError:
                    continue
                if cells[1].split("<")[0] == dk:
                    tot_n += n_disp
        if tot_n:
            traffic = {"hbm_mib_per_launch": round(tot_b / tot_n, 2), "source": "profiles/%s_hbm_counters.md" % wl.name,
                       "algorithmic_mib_per_launch": dom["algorithmic_mib_per_launch"],
                       "ratio": round(tot_b / tot_n / max(dom["algorithmic_mib_per_launch"], 1e-9), 3)}
    roofline = {"kernel": dk, "bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"],
                "frac": dom["frac"], "traffic": traffic}
    roofline.update({k: dom[k] for k in ("launches_per_step", "avg_launch_us", "algorithmic_mib_per_launch", "nonzero_gflop_per_launch",
                                          "algorithmic_gbs", "nonzero_tflops", "mfma_util", "ideal_sparse_frac")})
    roofline["share_of_step"] = round(dom["total_us"] / t_all, 3)
    roofline["definition"] = ("frac = achieved / peak for the bound that takes longer: algorithmic bytes (|in| + |out| + kept weights) "
                              "at the HBM peak, or nonzero flops 8*N*Ho*Wo*nnzk at the peak of the unit that multiplies; durations are "
                              "HIP events around each library call on its stream; mfma_util = zero-filled flops issued / bf16 matrix peak")
    # all calls of the step: the sum of their roofline times over the step time
    roofline["path_frac"] = round(sum(c["t_roof"] for c in calls) / (ms_per_step * 1e3), 4)
    # the same against max(algorithmic bytes / HBM peak, nonzero flops / float32 vector peak)
    roofline["path_ideal_sparse_frac"] = round(sum(c["t_sparse"] for c in calls) / (ms_per_step * 1e3), 4)
    roofline["path_mfma_util"] = round(sum(c["dense"] for c in calls) / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4)
    roofline["kernels"] = {}
    for sname, cs in sorted(syms.items(), key=lambda kv: -sum(c["us"] for c in kv[1])):
        sm = summarise(cs)
        roofline["kernels"][sname] = {k: sm[k] for k in ("launches_per_step", "avg_launch_us", "bound", "frac", "algorithmic_mib_per_launch",
                                                          "nonzero_gflop_per_launch", "mfma_util")}
        log("kernel %-46s launches %3d  avg %8.1f us  %4s frac %6.3f  nz %7.2f TF/s  alg %6.0f GB/s  mfma util %s" % (
            sname, sm["launches_per_step"], sm["avg_launch_us"], sm["bound"], sm["frac"], sm["nonzero_tflops"], sm["algorithmic_gbs"],
            sm["mfma_util"]))
    log("dominant kernel family %s: %d launches, %.1f us of %.1f us, bound %s, frac %.4f; whole step: path_frac %.4f" % (
        dk, dom["launches_per_step"], dom["total_us"], t_all, dom["bound"], dom["frac"], roofline["path_frac"]))

    if args.calib_copy_mb > 0:
        n = args.calib_copy_mb * (1 << 20) // 4
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        log("calibration copy: %d MiB read + %d MiB written" % (args.calib_copy_mb, args.calib_copy_mb))

    # ---- the same layers as one network: every layer's input is the previous layer's output after ReLU (and a 2x2
    # max pooling where the next map is half the size), the backward pass runs in reverse order; bwd_weight of a
    # layer is forked to the side stream once its error tensor exists. No gradient reaches the network's input.
    chained = None
    if not args.no_chained and len(wl.layers) > 1:
        ok = all(L.stride == 1 for L in wl.layers) and all(
            (b.C == a.F and b.H in (a.Ho, a.Ho // 2) and b.N == a.N) for a, b in zip(wl.layers, wl.layers[1:]))
        if not ok:
            if args.chained:
                log("--chained: workload %s is not a plain chain of stride-1 layers, skipped" % wl.name)
        else:
            nl = len(layers)
            for li, d in enumerate(layers):
                L = d["L"]
                nxt = wl.layers[li + 1] if li + 1 < nl else None
                d["pool"] = (2 if nxt.H == L.Ho // 2 and nxt.H != L.Ho else 1) if nxt is not None else (2 if L.Ho >= 2 else 1)
                q = d["pool"]
                d["a"] = torch.empty((L.N, L.Ho // q, L.Wo // q, L.F), dtype=tdt, device="cuda")
                d["sel"] = torch.empty((L.N, L.Ho // q, L.Wo // q, L.F), dtype=torch.uint8, device="cuda")
            last = layers[-1]
            da_last = up(I.gen_activations(tuple(last["a"].shape), I.BASE_SEED, (wl.name, "chain_da"), False, wl.dtype)[1])

            def chain_step(side, fuse=False):
                # fuse: where no pooling follows a layer, its ReLU runs inside the conv launch (pc_conv_fwd_relu) and
                # its derivative inside the next layer's backward-data launch (pc_conv_bwd_data_relu)
                xin = layers[0]["x"]
                for d in layers:
                    L = d["L"]
                    if fuse and d["pool"] == 1 and d is not layers[-1]:
                        B.pc_conv_fwd_relu(ctx, d["desc"], d["pk"], xin, d["a"])
                    else:
                        B.pc_conv_fwd(ctx, d["desc"], d["pk"], xin, d["y"])
                        B.pc_act_pool_fwd(ctx, d["y"], L.N, L.Ho, L.Wo, L.F, dt, d["pool"], d["a"], d["sel"])
                    d["xin"] = xin
                    xin = d["a"]
                # the error of the last layer's output through its ReLU / pooling; d["dy"] holds a layer's dz from here on
                last_d = layers[-1]
                B.pc_act_pool_bwd(ctx, da_last, last_d["sel"], last_d["L"].N, last_d["L"].Ho, last_d["L"].Wo, last_d["L"].F, dt,
                                  last_d["pool"], last_d["dy"])
                for li in range(nl - 1, -1, -1):
                    d = layers[li]
                    if side == "group":
                        pass                                                         # all weight gradients at the end
                    elif side:
                        streams_w[0].wait_stream(stream)
                        B.pc_conv_bwd_weight(ctxs_w[0], d["desc"], d["pk"], d["xin"], d["dy"], d["dw"])
                    else:
                        B.pc_conv_bwd_weight(ctx, d["desc"], d["pk"], d["xin"], d["dy"], d["dw"])
                    if li > 0:
                        prev = layers[li - 1]
                        Lp = prev["L"]
                        if fuse and prev["pool"] == 1:
                            B.pc_conv_bwd_data_relu(ctx, d["desc"], d["pk"], d["dy"], d["xin"], prev["dy"])
                        else:
                            B.pc_conv_bwd_data(ctx, d["desc"], d["pk"], d["dy"], d["dx"])
                            B.pc_act_pool_bwd(ctx, d["dx"], prev["sel"], Lp.N, Lp.Ho, Lp.Wo, Lp.F, dt, prev["pool"], prev["dy"])
                if side == "group":
                    B.pc_conv_bwd_weight_batch(ctx, [d["desc"] for d in layers], [d["pk"] for d in layers],
                                               [d["xin"] for d in layers], [d["dy"] for d in layers], [d["dw"] for d in layers])
                elif side:
                    stream.wait_stream(streams_w[0])

            def time_chain(side, fuse=False):
                chain_step(side, fuse)
                torch.cuda.synchronize()
                gch = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gch, stream=stream):
                    chain_step(side, fuse)
                for _ in range(3):
                    gch.replay()
                torch.cuda.synchronize()
                t0c = time.perf_counter()
                for _ in range(args.steps):
                    gch.replay()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0c) * 1e3 / args.steps

            ms_by_streams = {"per layer, one stream": time_chain(False), "weight gradients grouped": time_chain("group"),
                             "weight gradients grouped, ReLU fused": time_chain("group", True)}
            if ctxs_w:
                ms_by_streams["per layer, weight gradients on a side stream"] = time_chain(True)
            finite = bool(torch.isfinite(layers[0]["dw"]).all().item()) and bool(torch.isfinite(last["a"].float()).all().item())
            n_str, ms_chain = min(ms_by_streams.items(), key=lambda kv: kv[1])
            fl_chain = sum(3.0 * d["flops"] for d in layers) - layers[0]["flops"]
            # the act / pool calls alone (one graph), priced by their bytes: z in, a and sel out; da and sel in, dz out
            def act_only():
                for d in layers:
                    L = d["L"]
                    B.pc_act_pool_fwd(ctx, d["y"], L.N, L.Ho, L.Wo, L.F, dt, d["pool"], d["a"], d["sel"])
                for d in reversed(layers):
                    L = d["L"]
                    B.pc_act_pool_bwd(ctx, d["a"], d["sel"], L.N, L.Ho, L.Wo, L.F, dt, d["pool"], d["dy"])
            gact = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gact, stream=stream):
                act_only()
            gact.replay()
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                gact.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            us_act = e0.elapsed_time(e1) * 1e3 / 10
            by_act = sum(2 * (d["act_out"] + d["a"].numel() * (esz + 1)) for d in layers)
            chained = {"ms_per_step": round(ms_chain, 4), "value": round(fl_chain / (ms_chain * 1e-3) / 1e12, 4), "unit": "TFLOP/s",
                       "passes": "%d fwd + %d bwd_weight + %d bwd_data, ReLU / pooling between the layers" % (nl, nl, nl - 1),
                       "variant": n_str, "ms_per_step_by_variant": {str(k): round(v, 4) for k, v in ms_by_streams.items()},
                       "finite": finite,
                       "act_pool_us": round(us_act, 1), "act_pool_gbs": round(by_act / us_act / 1e3, 1),
                       "act_pool_hbm_frac": round(by_act / us_act / 1e3 / PEAK_HBM_GBS, 4)}
            log("chained network: %.4f ms per step (%.1f nonzero TFLOP/s; %s); all ReLU/pool calls alone "
                "%.1f us (%.0f GB/s algorithmic)" % (ms_chain, chained["value"], chained["variant"], us_act, by_act / us_act / 1e3))
            torch.cuda.synchronize()

    # ---- the training-side steps over the same layers (one graph of all layers per step kind), HBM-bound
    train_steps = None
    if args.train_steps:
        train_steps = {}
        hist = torch.zeros(512, dtype=torch.int32, device="cuda")
        for d in layers:
            L = d["L"]
            d["counts"] = torch.zeros((L.F, L.C, wl.P), dtype=torch.int32, device="cuda")
            d["gdense"] = torch.zeros((L.F, L.C, 9), dtype=torch.float32, device="cuda")
        pen = torch.zeros(1, dtype=torch.float64, device="cuda")
        kinds_ts = {
            "dppg_accumulate": (lambda d: B.pc_dppg_accumulate(ctx, d["W"], d["G"], d["L"].F, d["L"].C, hist, None), 72),
            "finalize_count": (lambda d: B.pc_finalize_count(ctx, d["pid"], d["L"].F, d["L"].C, wl.P, d["counts"]), 9),
            "finalize_pick": (lambda d: B.pc_finalize_pick(ctx, d["counts"], d["L"].F, d["L"].C, wl.P, d["pid"]), 4 * wl.P + 1),
            "group_lasso_grad": (lambda d: B.pc_group_lasso_grad(ctx, d["W"], d["pid"], d["keep"], d["L"].F, d["L"].C, lib,
                                                                 1e-4, 1e-4, d["gdense"], pen), 110),
        }
        n_kern = sum(d["L"].F * d["L"].C for d in layers)
        Fs, Cs = [d["L"].F for d in layers], [d["L"].C for d in layers]
        col = lambda key: [d[key] for d in layers]
        # all layers per call (one launch each; the group-lasso penalty adds a one-workgroup sum)
        batch_ts = {
            "dppg_accumulate": lambda: B.pc_dppg_accumulate_batch(ctx, col("W"), col("G"), Fs, Cs, hist, None),
            "finalize_count": lambda: B.pc_finalize_count_batch(ctx, col("pid"), Fs, Cs, wl.P, col("counts")),
            "finalize_pick": lambda: B.pc_finalize_pick_batch(ctx, col("counts"), Fs, Cs, wl.P, col("pid")),
            "group_lasso_grad": lambda: B.pc_group_lasso_grad_batch(ctx, col("W"), col("pid"), col("keep"), Fs, Cs, lib, 1e-4, 1e-4,
                                                                    col("gdense"), pen),
        }
        for name, (fn, bytes_per_kernel) in kinds_ts.items():
            def run_kind():
                if args.no_batch_prep or len(layers) > 32:
                    for d in layers:
                        fn(d)
                else:
                    batch_ts[name]()
            run_kind()
            torch.cuda.synchronize()
            gts = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gts, stream=stream):
                run_kind()
            gts.replay()
            torch.cuda.synchronize()
            e0 = torch.cuda.Event(enable_timing=True)
            e1 = torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                gts.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 10
            gbs = n_kern * bytes_per_kernel / us / 1e3
            train_steps[name] = {"us_all_layers": round(us, 1), "algorithmic_gbs": round(gbs, 1),
                                 "hbm_frac": round(gbs / PEAK_HBM_GBS, 4)}
            log("train step %-18s %2d layers %8.1f us  alg %7.0f GB/s (%d B per kernel position)" % (
                name, len(layers), us, gbs, bytes_per_kernel))
        # selection was overwritten by finalize_pick: restore the packs' masks for anything that follows
        for d in layers:
            run_pass(d, "select")
        torch.cuda.synchronize()

    # ---- context only: the paper's one absolute time for this path is the demonstration layer of its Section 5.1
    # (256 filters x 128 channels on a 224x224 map, batch 1: a 256x1152 by 1152x50176 SpMM, about 3000 us on one
    # Quadro RTX 5000, precision and sparsity not stated). The same layer shape through pc_conv_fwd here:
    paper_context = None
    if wl.dtype == "bf16" and not args.no_paper_context:
        Lp = I.Layer(1, 224, 224, 128, 256, 1)
        Wp = up(I.gen_weights(Lp.F, Lp.C, I.BASE_SEED, "paper_demo"))
        kp_n = I.kept_per_filter(wl.keep, Lp.C)
        pidp = torch.empty((Lp.F, Lp.C), dtype=torch.uint8, device="cuda")
        keepp = torch.empty((Lp.F, Lp.C), dtype=torch.uint8, device="cuda")
        B.pc_pattern_select(ctx, Wp, None, Lp.F, Lp.C, lib, B.PC_KEEP_PER_FILTER, kp_n, B.PC_SCORE_RETAINED, pidp, keepp)
        pkp = B.pc_pack(ctx, Wp, pidp, keepp, Lp.F, Lp.C, lib, dt)
        xp = up(I.gen_activations((1, 224, 224, 128), I.BASE_SEED, "paper_demo_x", True, wl.dtype)[1])
        yp = torch.empty((1, 224, 224, 256), dtype=tdt, device="cuda")
        descp = B.make_desc(1, 224, 224, 128, 256, 1, dt)
        for _ in range(3):
            B.pc_conv_fwd(ctx, descp, pkp, xp, yp)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(20):
            B.pc_conv_fwd(ctx, descp, pkp, xp, yp)
        e1.record(stream)
        torch.cuda.synchronize()
        us_p = e0.elapsed_time(e1) * 1e3 / 20
        B.pc_packed_free(pkp)
        paper_context = {"layer": "1x224x224, 128->256 (the 256x1152 by 1152x50176 product of Section 5.1)",
                         "fwd_us_here": round(us_p, 1), "keep": wl.keep, "dtype": wl.dtype,
                         "paper_us": 3000, "paper_hardware": "1x Quadro RTX 5000, precision and sparsity not stated",
                         "note": "context only, not a target"}
        log("paper's demonstration layer (Section 5.1), forward: %.1f us here (bf16, keep %.2f); paper: about 3000 us "
            "SpMM on one Quadro RTX 5000 (context only)" % (us_p, wl.keep))

    # ---- the per-layer operator choice as a function of sparsity (Section 5.2 / 5.4; the shape of the paper's
    # sparsity sweep): one bf16 layer over a range of keep ratios, the three passes with the pattern-grouped gather
    # kernels (only kept taps are multiplied) and with the matrix-core kernels (zero-filled tiles)
    sweep = None
    if args.sweep:
        sN, sH, sW, sC, sF, sS = (int(v) for v in args.sweep_shape.split(","))
        Ls = I.Layer(sN, sH, sW, sC, sF, sS)
        Ws = up(I.gen_weights(sF, sC, I.BASE_SEED, "sweep"))
        Gs = up(I.gen_weight_grads(sF, sC, I.BASE_SEED, "sweep"))
        xs_ = up(I.gen_activations((sN, sH, sW, sC), I.BASE_SEED, ("sweep", "x"), True, "bf16")[1])
        dys_ = up(I.gen_activations((sN, Ls.Ho, Ls.Wo, sF), I.BASE_SEED, ("sweep", "dy"), False, "bf16")[1])
        ys_, dxs_ = torch.empty_like(dys_), torch.empty_like(xs_)
        descs_ = B.make_desc(sN, sH, sW, sC, sF, sS, B.PC_BF16)
        pids_ = torch.empty((sF, sC), dtype=torch.uint8, device="cuda")
        keeps_ = torch.empty((sF, sC), dtype=torch.uint8, device="cuda")
        rows = []
        for kr in (0.02, 0.05, 0.1, 0.2, 0.3, 0.5, 1.0):
            ks = I.kept_per_filter(kr, sC)
            B.pc_pattern_select(ctx, Ws, Gs, sF, sC, lib, B.PC_KEEP_PER_FILTER, ks, B.PC_SCORE_RETAINED, pids_, keeps_)
            t_us = {}
            for vname, var in (("gather", B.PC_VARIANT_VALU), ("matrix", B.PC_VARIANT_MFMA), ("sparse", B.PC_VARIANT_MFMA_SPARSE),
                               ("auto", B.PC_VARIANT_AUTO)):
                B.pc_set_variant(ctx, var)
                pks = B.pc_pack(ctx, Ws, pids_, keeps_, sF, sC, lib, B.PC_BF16)
                nz, picked = B.pc_packed_info(ctx, pks)
                dws = torch.empty((max(nz, 1), 4), dtype=torch.float32, device="cuda")
                def sweep_step():
                    B.pc_conv_fwd(ctx, descs_, pks, xs_, ys_)
                    B.pc_conv_bwd_data(ctx, descs_, pks, dys_, dxs_)
                    B.pc_conv_bwd_weight(ctx, descs_, pks, xs_, dys_, dws)
                for _ in range(2):
                    sweep_step()
                torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(5):
                    sweep_step()
                e1.record(stream)
                torch.cuda.synchronize()
                t_us[vname] = round(e0.elapsed_time(e1) * 1e3 / 5, 1)
                if vname == "auto":
                    t_us["auto_picks"] = {B.PC_VARIANT_MFMA: "matrix", B.PC_VARIANT_MFMA_SPARSE: "sparse"}.get(picked, "gather")
                B.pc_packed_free(pks)
            B.pc_set_variant(ctx, {"auto": B.PC_VARIANT_AUTO, "valu": B.PC_VARIANT_VALU, "mfma": B.PC_VARIANT_MFMA, "sparse": B.PC_VARIANT_MFMA_SPARSE}[args.variant])
            rows.append({"keep": round(ks / sC, 4), "weight_density": round(ks / sC * 4.0 / 9.0, 4), "us": t_us})
            log("sweep keep %.3f density %.4f: gather %.1f us, matrix %.1f us, structured-sparse matrix %.1f us, auto %.1f us (%s)" % (
                ks / sC, ks / sC * 4 / 9, t_us["gather"], t_us["matrix"], t_us["sparse"], t_us["auto"], t_us["auto_picks"]))
        sweep = {"layer": "N=%d %dx%d %d->%d stride %d, bf16, %d patterns" % (sN, sH, sW, sC, sF, sS, wl.P),
                 "passes": "fwd+bwd_data+bwd_weight", "rows": rows}

    # ---- the CPU oracle on a bounded sample of the same workload (reported, not a target)
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import pc_oracle as oracle
        # a bounded sample: the oracle runs at a few nonzero GFLOP/s, so the batch is cut to what takes it about 15 s
        if args.cpu_sample_batch > 0:
            ns = min(args.cpu_sample_batch, wl.layers[0].N)
        else:
            per_image = total_flops / wl.layers[0].N
            ns = int(max(1, min(wl.layers[0].N, round(15.0 * 5e9 / per_image))))
        t_cpu, f_cpu = 0.0, 0.0
        for li, L in enumerate(wl.layers):
            tag = (wl.name, li)
            Wn = I.gen_weights(L.F, L.C, I.BASE_SEED, tag)
            Gn = I.gen_weight_grads(L.F, L.C, I.BASE_SEED, tag)
            k = I.kept_per_filter(wl.keep, L.C)
            xs = I.gen_activations((ns, L.H, L.W, L.C), I.BASE_SEED, (tag, "x", "cpu"), True, wl.dtype)[0]
            dys = I.gen_activations((ns, L.Ho, L.Wo, L.F), I.BASE_SEED, (tag, "dy", "cpu"), False, wl.dtype)[0]
            c0 = time.perf_counter()
            pid, kp = oracle.select(Wn, Gn, lib, k)
            M = oracle.mask(pid, kp, lib)
            Wm = oracle.apply_mask(oracle.bf16_round(Wn) if wl.dtype == "bf16" else Wn, M)
            c1 = time.perf_counter()
            oracle.conv_fwd(xs, Wm, L.stride)
            oracle.conv_bwd_data(dys, Wm, xs.shape, L.stride)
            oracle.conv_bwd_weight(xs, dys, M, L.stride)
            c2 = time.perf_counter()
            t_cpu += (c2 - c1) + ((c1 - c0) if wl.with_select else 0.0)
            f_cpu += 3.0 * 8.0 * ns * L.Ho * L.Wo * int(kp.sum())
        cpu = {"value": round(f_cpu / t_cpu / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "all %d layers of %s at batch %d (of %d), fwd+bwd_data+bwd_weight%s, %.1f s" % (
                   len(wl.layers), wl.name, ns, wl.layers[0].N, " + select" if wl.with_select else "", t_cpu)}

    out = {
        "metric": "effective nonzero-MAC TFLOP/s for pattern-conv fwd+bwd; % of MI355X roofline",
        "value": round(value, 4), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": wl.name, "layers": len(wl.layers), "batch": wl.layers[0].N, "patterns": wl.P,
                   "keep": wl.keep, "variant": args.variant, "passes": "+".join(passes), "launch": "hip_graph" if graph is not None else "host",
                   "streams": 1 + len(ctxs_w), "wgrad": mode["wgrad"],
                   "wgrad_trial_ms": {k: round(v, 4) for k, v in mode["trial_ms"].items()} if "trial_ms" in mode else None,
                   "nonzero_gflop_per_step": round(total_flops / 1e9, 3)},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if chained is not None:
        out["chained"] = chained
    if train_steps is not None:
        out["train_steps"] = train_steps
    if paper_context is not None:
        out["paper_context"] = paper_context
    if sweep is not None:
        out["sweep"] = sweep
    print(json.dumps(out), flush=True)
    for d in layers:
        B.pc_packed_free(d["pk"])
    for c_w in ctxs_w:
        B.pc_destroy(c_w)
    B.pc_destroy(ctx)
    return 0


if __name__ == "__main__":
    sys.exit(main())

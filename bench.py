#!/usr/bin/env python3
"""Benchmark: ResNet-50 convolution stack, column-wise 2:4 (T = 16), batch 64,
on one MI355X (the default; --workload selects the other workloads, which are
reported the same way but are not the headline).

A step is one pass of the hot path over one batch: all 53 convolutions
(fused im2col+pack, kept-column contraction, bias + ReLU) launched back to back
through the C ABI on one stream, each on its own resident synthetic input of the
standard shape.  Pruning, packing and the per-layer tuning are one-time set-up,
as in the paper (weights are pruned once, every candidate kernel is profiled
once per layer), and are reported separately.

Prints ONE JSON line on stdout; everything else goes to stderr.
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

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # dense MFMA peaks of MI355X
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dtype", choices=["f32", "bf16"], default="f32")
    ap.add_argument("--batch", type=int, default=None, help="default: the workload's own batch")
    ap.add_argument("--workload", default="resnet50",
                    choices=["resnet50", "resnet18", "resnet101", "sweep", "single",
                             "resnet50_net", "resnet18_net", "resnet101_net", "fusion"],
                    help="resnet50 (default, the headline: 53 layers 2:4 T16 batch 64) | resnet18 (batch 32) | "
                         "resnet101 (mixed sparsity, T32, batch 256, bf16) | sweep (15 N:M x T cells of one "
                         "3x3 layer + its dense form, batch 32) | single (one 3x3 layer, batch 1) | *_net: the "
                         "whole network on one input batch (residual adds fused into the closing convolution of "
                         "each block, pooling, classifier), reported in images/s | fusion: the k x k layers of "
                         "ResNet-50 fused (nm_conv2d) against unfused (nm_im2col to memory, then the same "
                         "contraction as a 1x1 convolution over it), the comparison of the paper's section 4.3")
    ap.add_argument("--tile", type=int, default=None,
                    help="experiment: tile size T of the ResNet workloads (1 = conventional row-wise N:M)")
    ap.add_argument("--nm", default=None, help="experiment: N:M of the ResNet-18/50 workloads, e.g. 1:4")
    ap.add_argument("--group", choices=["cin", "row"], default=None,
                    help="experiment: one group per kernel tap (M = Cin) or per row (M = K), half the columns kept")
    ap.add_argument("--tune-tile", default=None,
                    help="experiment: comma-separated tile sizes; the tuner prunes every pruned layer at each and "
                         "keeps the fastest per layer (nm_autotune_tile), e.g. 8,16,32")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tune", action="store_true", help="use the untuned default variant")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch the 53 kernels of a step one by one instead of replaying a HIP graph")
    ap.add_argument("--cache", default=None, help="tuning cache file to load/save")
    ap.add_argument("--report", default=None, help="write the per-layer table (JSON) here")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2507_17301_amd import binding as nm
    from paper_2507_17301_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    nm.lib()

    n_, m_ = (int(v) for v in args.nm.split(":")) if args.nm else (2, 4)
    t_ = args.tile or 16
    if args.workload.endswith("_net"):
        return whole_network(args, n_, m_, t_)
    if args.workload == "fusion":
        return fusion_ablation(args, n_, m_, t_)
    if args.workload == "resnet50":
        layers, B, seed0 = wl.resnet50_stack(n_, m_, t_), 64, 4000
        wname = f"resnet50_conv_stack_53layers_{n_}of{m_}_T{t_}"
    elif args.workload == "resnet18":
        layers, B, seed0 = wl.resnet18_stack(n_, m_, t_), 32, 3000
        wname = f"resnet18_conv_stack_20layers_{n_}of{m_}_T{t_}"
    elif args.workload == "resnet101":
        layers, B, seed0 = wl.resnet101_stack(args.tile or 32), 256, 5000
        wname = f"resnet101_conv_stack_104layers_mixed_T{args.tile or 32}"
        if "--dtype" not in sys.argv:
            args.dtype = "bf16"
    elif args.workload == "sweep":
        cells = wl.sweep_config2()
        layers, B, wname, seed0 = cells + [wl.dense_form(cells[1], "cfg2_dense_T16")], 32, "sweep_3x3_256ch_14x14_15cells_plus_dense", 0
    else:
        layers, B, wname, seed0 = [wl.single_conv_config1()], 1, "single_3x3_64ch_56x56_2of4_T16", 0
    if args.group:
        layers = wl.with_large_groups(layers, args.group)
        wname += "_groups_per_" + args.group
    if args.batch is not None:
        B = args.batch
    cand_tiles = [int(t) for t in args.tune_tile.split(",")] if args.tune_tile else None
    if cand_tiles:
        wname += "_T_per_layer_of_" + "_".join(str(t) for t in cand_tiles)
    headline = (args.workload == "resnet50" and B == 64 and not args.group and (n_, m_, t_) == (2, 4, 16)
                and not cand_tiles)
    bf16 = args.dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    esize = 2 if bf16 else 4

    # ---- one-time set-up: weights, pruning, tuning, resident inputs ---------
    if args.cache and os.path.exists(args.cache):
        nm.nm_cache_load(args.cache)
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    t0 = time.time()
    packed, xs, ys, biases, variants = [], [], [], [], []
    prune_s = 0.0
    for i, l in enumerate(layers):
        _, w, bias = wl.make_tensors(l, B, seed0 + i, with_input=False)
        tp = time.time()
        if cand_tiles and l.n < l.m:
            import dataclasses
            wp, best_t, t_ms = nm.nm_autotune_tile(w, l.n, l.m, cand_tiles, ndt, B, l.H, l.W, True,
                                                   l.stride, l.pad, l.dil, True)
            log(f"{l.name:>22s}  T -> {best_t:2d}   " +
                "  ".join(f"T{t}: {v * 1e3:7.1f} us" for t, v in zip(cand_tiles, t_ms)))
            layers[i] = l = dataclasses.replace(l, tile=best_t)
        else:
            wp = nm.nm_prune(w, l.n, l.m, l.tile, ndt)
        prune_s += time.time() - tp
        packed.append(wp)
        x = torch.rand((B, l.H, l.W, l.Cin), generator=gen, device=dev, dtype=torch.float32).to(tdt)
        xs.append(x)
        ys.append(torch.empty((B, l.Ho, l.Wo, l.Cout), device=dev, dtype=tdt))
        biases.append(torch.from_numpy(bias).to(dev))
    tune_s = 0.0
    for i, l in enumerate(layers):
        if args.no_tune:
            variants.append(None)
            continue
        tp = time.time()
        v, ms = nm.nm_autotune(ndt, B, l.H, l.W, l.Cin, packed[i], True, l.stride, l.pad, l.dil, True)
        tune_s += time.time() - tp
        variants.append(v)
    torch.cuda.synchronize()
    if args.cache:
        nm.nm_cache_save(args.cache)
    log(f"set-up {time.time() - t0:.1f}s (prune+pack {prune_s:.2f}s, tune {tune_s:.2f}s), "
        f"{len(layers)} layers, {nm.nm_cache_size()} tuned shapes")

    stream = torch.cuda.current_stream()

    # a plain device copy of known size (1 GiB read + 1 GiB written): the yardstick
    # for the FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    def step():
        for i, l in enumerate(layers):
            nm.nm_conv2d(xs[i], packed[i], biases[i], l.stride, l.pad, l.dil, True, y=ys[i],
                         stream=stream)

    # The launch-bound sequence of a step is captured once into a HIP graph (the
    # library only enqueues kernels, so it can be captured) and replayed per step.
    step()
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            nonlocal_stream = torch.cuda.current_stream()
            for i, l in enumerate(layers):
                nm.nm_conv2d(xs[i], packed[i], biases[i], l.stride, l.pad, l.dil, True, y=ys[i],
                             stream=nonlocal_stream)
    run_step = graph.replay if graph is not None else step

    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t_host0 = time.time()
    e0.record(stream)
    for _ in range(args.steps):
        run_step()
    e1.record(stream)
    torch.cuda.synchronize()
    t_host = time.time() - t_host0
    ms_step = e0.elapsed_time(e1) / args.steps
    ms_step_host = t_host * 1e3 / args.steps

    # ---- per-layer kernel durations, in the stack (HIP events on the launch stream):
    # an event after every layer of a few extra steps, so that each layer is timed
    # with the caches in the state the stack leaves them in
    inst_steps = 3
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(layers) + 1)]
             for _ in range(inst_steps)]
    for k in range(inst_steps):
        marks[k][0].record(stream)
        for i, l in enumerate(layers):
            nm.nm_conv2d(xs[i], packed[i], biases[i], l.stride, l.pad, l.dil, True, y=ys[i],
                         stream=stream)
            marks[k][i + 1].record(stream)
    torch.cuda.synchronize()
    per_layer = []
    for i, l in enumerate(layers):
        ms = sorted(marks[k][i].elapsed_time(marks[k][i + 1]) for k in range(inst_steps))[inst_steps // 2]
        eff = l.effective_flops(B)
        byts = l.algorithmic_bytes(B, esize, esize)
        t_flop = eff / (PEAK_TFLOPS[args.dtype] * 1e12) * 1e3
        t_mem = byts / (PEAK_HBM_GBS * 1e9) * 1e3
        per_layer.append({
            "layer": l.name, "variant": nm.nm_variant_name(variants[i]) if variants[i] is not None else "default",
            "ms": ms, "dense_gflops": l.dense_flops(B) / ms / 1e6, "eff_gflops": eff / ms / 1e6,
            "alg_bytes": byts, "gbs": byts / ms / 1e6, "t_min_ms": max(t_flop, t_mem),
            "bound": "mfma" if t_flop >= t_mem else "hbm", "frac": max(t_flop, t_mem) / ms,
        })

    dense = sum(l.dense_flops(B) for l in layers)
    eff = sum(l.effective_flops(B) for l in layers)
    byts = sum(l.algorithmic_bytes(B, esize, esize) for l in layers)
    kern_ms = sum(r["ms"] for r in per_layer)
    tmin_ms = sum(r["t_min_ms"] for r in per_layer)
    for r in per_layer:
        log(f"{r['layer']:>18s} {r['variant']:>34s} {r['ms'] * 1e3:9.1f} us  "
            f"{r['eff_gflops'] / 1e3:7.1f} eff TF/s {r['gbs']:8.0f} GB/s  {r['bound']:4s} {r['frac'] * 100:5.1f}%")
    log(f"sum of kernel times {kern_ms:.3f} ms, step {ms_step:.3f} ms (host {ms_step_host:.3f} ms), "
        f"sum of per-layer lower bounds {tmin_ms:.3f} ms -> {tmin_ms / kern_ms * 100:.1f}% of binding roofline")

    # The convolution kernel, all launches of a step taken together.  fp32 is bound by the
    # fp32 matrix cores (2*P*K'*Cout flops per launch); with bf16 tensors nearly every layer
    # sits below the ridge, so the bound is HBM (algorithmic bytes per launch).  The average
    # launch duration comes from the timed region itself: the launches of a step run back to
    # back on one stream, so step time / launches is the kernel's duration plus whatever gap
    # the launches leave (an upper bound on the duration; the kernel trace shows no gap).
    avg_ms = ms_step / len(layers)
    if bf16:
        roofline = {"bound": "hbm", "achieved": byts / ms_step / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": byts / ms_step / 1e6 / PEAK_HBM_GBS}
    else:
        roofline = {"bound": "mfma", "achieved": eff / ms_step / 1e9, "peak": PEAK_TFLOPS["f32"],
                    "unit": "TFLOP/s", "frac": eff / ms_step / 1e9 / PEAK_TFLOPS["f32"]}
    roofline.update({
        # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
        # counters read for the 1 GiB device copy above (profiles/); measured for the default workload only
        "traffic": {"f32": 112.5e6, "bf16": 54.7e6}[args.dtype] if headline else None,
        "kernel": "nm_conv_sp16_kernel" if bf16 else "nm_conv_kernel", "launches_per_step": len(layers),
        "avg_launch_ms": avg_ms,
        # with an event after every layer of three extra steps (adds the events' own cost)
        "avg_launch_ms_event_per_layer": kern_ms / len(layers),
        "frac_of_binding_roofline_per_layer": tmin_ms / kern_ms,
        "effective_tflops": eff / ms_step / 1e9,
        "algorithmic_gbytes_per_step": byts / 1e9, "achieved_gbs": byts / ms_step / 1e6,
    })

    if args.workload == "sweep":
        # sparse-over-dense speedup per cell: the dense form of the same layer through the same kernel family
        t_dense = per_layer[-1]["ms"]
        for r in per_layer[:-1]:
            r["speedup_over_dense"] = t_dense / r["ms"]
            log(f"{r['layer']:>18s}  {r['ms'] * 1e3:7.1f} us   x{r['speedup_over_dense']:.2f} over dense ({t_dense * 1e3:.1f} us)")

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(layers, B, bf16, seed0)

    out = {
        "metric": ("dense-equiv GFLOP/s, ResNet-50 conv stack 2:4 @batch 64" if headline
                   else f"dense-equiv GFLOP/s, {wname} @batch {B}"),
        "value": dense / ms_step / 1e6, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_img": ms_step / B,
        "effective_gflops": eff / ms_step / 1e6,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{wname}_batch{B}_{args.dtype}",
                   "batch": B, "layers": len(layers), "tuned": not args.no_tune,
                   "launch": "hip_graph_replay" if graph is not None else "one_launch_per_layer"},
        "setup": {"prune_pack_s": prune_s, "autotune_s": tune_s},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if args.report:
        with open(args.report, "w") as f:
            json.dump({"summary": out, "layers": per_layer}, f, indent=1)
    print(json.dumps(out), flush=True)


def whole_network(args, n_, m_, t_):
    """One input batch through the whole network; a step is one forward pass."""
    import torch
    from paper_2507_17301_amd import binding as nm
    from paper_2507_17301_amd import workloads as wl
    from paper_2507_17301_amd.network import Network

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    name = args.workload[:-4]
    if name == "resnet50":
        ops, B, seed0 = wl.resnet50_graph(n_, m_, t_), 64, 4000
    elif name == "resnet18":
        ops, B, seed0 = wl.resnet18_graph(n_, m_, t_), 32, 3000
    else:
        ops, B, seed0 = wl.resnet101_graph(args.tile or 32), 256, 5000
        if "--dtype" not in sys.argv:
            args.dtype = "bf16"
    if args.batch is not None:
        B = args.batch
    bf16 = args.dtype == "bf16"
    esize = 2 if bf16 else 4
    t0 = time.time()
    net = Network(ops, B, 224, nm.NM_BF16 if bf16 else nm.NM_F32, seed0)
    t1 = time.time()
    if not args.no_tune:
        net.autotune()
    torch.cuda.synchronize()
    t2 = time.time()
    gen = torch.Generator(device=net.dev)
    gen.manual_seed(1234)
    net.t[0].copy_(torch.rand(net.shapes[0], generator=gen, device=net.dev, dtype=torch.float32))
    log(f"set-up: prune+pack {t1 - t0:.2f}s, tune {t2 - t1:.2f}s, {len(ops)} operators")

    stream = torch.cuda.current_stream()
    net.forward(stream=stream)
    torch.cuda.synchronize()
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            net.forward(stream=torch.cuda.current_stream())
    run_step = graph.replay if graph is not None else (lambda: net.forward(stream=stream))
    for _ in range(args.warmup):
        run_step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(args.steps):
        run_step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms_step = e0.elapsed_time(e1) / args.steps

    convs = [op.layer for op in ops if op.kind == "conv"]
    dense = sum(l.dense_flops(B) for l in convs)
    eff = sum(l.effective_flops(B) for l in convs)
    # every tensor written once and read by its consumers, plus the packed weights
    byts = sum(l.algorithmic_bytes(B, esize, esize) for l in convs)
    for op in ops:
        if op.residual >= 0:
            byts += int(torch.tensor(net.shapes[op.residual]).prod()) * esize
        if op.kind != "conv":
            byts += (int(torch.tensor(net.shapes[op.src]).prod()) + int(torch.tensor(net.shapes[op.dst]).prod())) * esize
    if bf16:
        roofline = {"bound": "hbm", "achieved": byts / ms_step / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": byts / ms_step / 1e6 / PEAK_HBM_GBS, "traffic": None}
    else:
        roofline = {"bound": "mfma", "achieved": eff / ms_step / 1e9, "peak": PEAK_TFLOPS["f32"],
                    "unit": "TFLOP/s", "frac": eff / ms_step / 1e9 / PEAK_TFLOPS["f32"], "traffic": None}
    roofline["note"] = "whole step (all operators) against the convolutions' flops / all tensors' bytes"
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline([l for l in convs], B, bf16, seed0)
        cpu["sample"] += "; convolutions only"
    out = {
        "metric": f"images/s, {name} whole network @batch {B}", "value": B / ms_step * 1e3, "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "ms_per_img": ms_step / B, "dense_equiv_gflops": dense / ms_step / 1e6,
        "effective_gflops": eff / ms_step / 1e6, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{name}_whole_network_batch{B}_{args.dtype}", "batch": B,
                   "operators": len(ops), "tuned": not args.no_tune,
                   "launch": "hip_graph_replay" if graph is not None else "one_launch_per_operator"},
        "setup": {"prune_pack_s": t1 - t0, "autotune_s": t2 - t1},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


def fusion_ablation(args, n_, m_, t_):
    """Fused im2col + contraction against the unfused pipeline, on the k x k layers of ResNet-50."""
    import numpy as np
    import torch
    from paper_2507_17301_amd import binding as nm
    from paper_2507_17301_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    B = args.batch or 64
    bf16 = args.dtype == "bf16"
    tdt = torch.bfloat16 if bf16 else torch.float32
    ndt = nm.NM_BF16 if bf16 else nm.NM_F32
    esize = 2 if bf16 else 4
    layers = [l for l in wl.unique_shapes(wl.resnet50_stack(n_, m_, t_)) if l.Kh * l.Kw > 1]
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    items = []
    for i, l in enumerate(layers):
        _, w, bias = wl.make_tensors(l, B, 4000 + i, with_input=False)
        wp = nm.nm_prune(w, l.n, l.m, l.tile, ndt)
        wp1 = nm.nm_prune(np.ascontiguousarray(w.reshape(l.Cout, 1, 1, -1)), l.n, l.m, l.tile, ndt)
        x = torch.rand((B, l.H, l.W, l.Cin), generator=gen, device=dev, dtype=torch.float32).to(tdt)
        a = torch.empty((B, l.Ho, l.Wo, l.K), device=dev, dtype=tdt)
        y = torch.empty((B, l.Ho, l.Wo, l.Cout), device=dev, dtype=tdt)
        bd = torch.from_numpy(bias).to(dev)
        if not args.no_tune:
            nm.nm_autotune(ndt, B, l.H, l.W, l.Cin, wp, True, l.stride, l.pad, l.dil, True)
            nm.nm_autotune(ndt, B, l.Ho, l.Wo, l.K, wp1, True, 1, 0, 1, True)
        items.append((l, wp, wp1, x, a, y, bd))
    stream = torch.cuda.current_stream()
    reps = max(3, args.steps)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    t_f, t_i, t_c = [[] for _ in items], [[] for _ in items], [[] for _ in items]
    for r in range(args.warmup + reps):
        for k, (l, wp, wp1, x, a, y, bd) in enumerate(items):     # all layers in turn: no layer finds its data cached
            e = [ev() for _ in range(4)]
            e[0].record(stream)
            nm.nm_conv2d(x, wp, bd, l.stride, l.pad, l.dil, True, y=y, stream=stream)
            e[1].record(stream)
            nm.nm_im2col(x, l.Kh, l.Kw, l.stride, l.pad, l.dil, a=a, stream=stream)
            e[2].record(stream)
            nm.nm_conv2d(a, wp1, bd, 1, 0, 1, True, y=y, stream=stream)
            e[3].record(stream)
            torch.cuda.synchronize()
            if r >= args.warmup:
                t_f[k].append(e[0].elapsed_time(e[1]))
                t_i[k].append(e[1].elapsed_time(e[2]))
                t_c[k].append(e[2].elapsed_time(e[3]))
    med = lambda v: sorted(v)[len(v) // 2]
    rows, sf, su = [], 0.0, 0.0
    for k, (l, *_rest) in enumerate(items):
        f, i2c, c1 = med(t_f[k]), med(t_i[k]), med(t_c[k])
        abytes = l.P(B) * l.K * esize
        rows.append({"layer": l.name, "fused_ms": f, "im2col_ms": i2c, "conv_over_im2col_ms": c1,
                     "speedup": (i2c + c1) / f, "im2col_matrix_mb": abytes / 1e6,
                     "fused_algorithmic_mb": l.algorithmic_bytes(B, esize, esize) / 1e6})
        sf += f
        su += i2c + c1
        log(f"{l.name:>18s}  fused {f * 1e3:7.1f} us | im2col {i2c * 1e3:7.1f} us + contraction {c1 * 1e3:7.1f} us "
            f"= x{(i2c + c1) / f:.2f} | im2col matrix {abytes / 1e6:7.1f} MB written and read back, "
            f"fused moves {l.algorithmic_bytes(B, esize, esize) / 1e6:6.1f} MB")
    out = {"metric": f"fused-over-unfused speedup, k x k layers of ResNet-50 {n_}:{m_} T{t_} @batch {B}",
           "value": su / sf, "unit": "x", "n_gpus": 1, "steps": reps, "warmup": args.warmup,
           "ms_per_step": sf, "unfused_ms_per_step": su, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
           "config": {"workload": f"resnet50_kxk_layers_fused_vs_unfused_batch{B}_{args.dtype}", "batch": B,
                      "layers": len(items)},
           "roofline": None, "cpu_baseline": None, "layers": rows}
    if args.report:
        with open(args.report, "w") as f:
            json.dump(out, f, indent=1)
    print(json.dumps(out), flush=True)


def cpu_baseline(layers, B, bf16, seed0):
    """The CPU oracle, as it stands, on the first images of the same workload."""
    import numpy as np
    import oracle
    from paper_2507_17301_amd import workloads as wl

    cores = min(16, os.cpu_count() or 1)
    prepared = []
    for i, l in enumerate(layers):
        _, w, bias = wl.make_tensors(l, 1, seed0 + i, with_input=False)
        _, _, wz = oracle.prune(w, l.n, l.m, l.tile)
        if bf16:
            wz = oracle.round_bf16(wz)
        prepared.append((l, wz, bias))
    rng = np.random.default_rng(99)

    def run(nimg):
        total = 0.0
        for l, wz, bias in prepared:
            x = rng.random((nimg, l.H, l.W, l.Cin), dtype=np.float32)
            t = time.time()
            oracle.conv2d(x, wz, bias, l.stride, l.pad, l.dil, True, out_bf16=bf16, nthreads=cores)
            total += time.time() - t
        return total

    t1 = run(1)
    nimg = int(max(2, min(B, round(15.0 / max(t1, 1e-3)))))
    t = run(nimg)
    dense_per_img = sum(l.dense_flops(1) for l, _, _ in prepared)
    log(f"cpu oracle: {nimg} images in {t:.2f}s on {cores} threads")
    return {"value": dense_per_img * nimg / t / 1e9, "unit": "GFLOP/s", "cores": cores,
            "kind": "oracle", "ms_per_img": t * 1e3 / nimg,
            "sample": f"first {nimg} of {B} images through all {len(prepared)} layers "
                      f"(direct convolution on zero-filled weights, fp64 accumulate)"}


if __name__ == "__main__":
    main()

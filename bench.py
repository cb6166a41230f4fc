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

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0, "f8": 5000.0}   # dense MFMA peaks of MI355X
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Stack:
    """The resident state of one conv stack: pruned + packed weights, one synthetic input
    and one output tensor per layer, biases, and (after tune()) the chosen variants."""

    def __init__(self, layers, B, dtype, seed0, cand_tiles=None):
        import torch
        from paper_2507_17301_amd import binding as nm
        from paper_2507_17301_amd import workloads as wl
        self.nm, self.torch = nm, torch
        self.layers, self.B, self.dtype = list(layers), B, dtype
        self.bf16 = dtype == "bf16"
        self.f8 = dtype == "f8"        # E4M3 activations and weights, bf16 output
        self.tdt = torch.float8_e4m3fn if self.f8 else (torch.bfloat16 if self.bf16 else torch.float32)
        self.tdt_out = torch.bfloat16 if self.f8 else self.tdt
        self.ndt = nm.NM_F8E4M3 if self.f8 else (nm.NM_BF16 if self.bf16 else nm.NM_F32)
        self.esize = 1 if self.f8 else (2 if self.bf16 else 4)
        self.esize_out = 2 if self.f8 else self.esize
        dev = torch.device("cuda:0")
        gen = torch.Generator(device=dev)
        gen.manual_seed(1234)
        self.packed, self.xs, self.ys, self.biases = [], [], [], []
        self.prune_s = self.tune_s = 0.0
        for i, l in enumerate(self.layers):
            _, w, bias = wl.make_tensors(l, B, seed0 + i, with_input=False)
            tp = time.time()
            if cand_tiles and l.n < l.m:
                import dataclasses
                wp, best_t, t_ms = nm.nm_autotune_tile(w, l.n, l.m, cand_tiles, self.ndt, B, l.H, l.W, True,
                                                       l.stride, l.pad, l.dil, True)
                log(f"{l.name:>22s}  T -> {best_t:2d}   " +
                    "  ".join(f"T{t}: {v * 1e3:7.1f} us" for t, v in zip(cand_tiles, t_ms)))
                self.layers[i] = l = dataclasses.replace(l, tile=best_t)
            else:
                wp = nm.nm_prune(w, l.n, l.m, l.tile, self.ndt)
            self.prune_s += time.time() - tp
            self.packed.append(wp)
            self.xs.append(torch.rand((B, l.H, l.W, l.Cin), generator=gen, device=dev,
                                      dtype=torch.float32).to(self.tdt))
            self.ys.append(torch.empty((B, l.Ho, l.Wo, l.Cout), device=dev, dtype=self.tdt_out))
            self.biases.append(torch.from_numpy(bias).to(dev))
        self.launched = [None] * len(self.layers)
        self.graph = None

    def tune(self):
        tp = time.time()
        for i, l in enumerate(self.layers):
            self.nm.nm_autotune(self.ndt, self.B, l.H, l.W, l.Cin, self.packed[i], True, l.stride, l.pad,
                                l.dil, True)
        self.torch.cuda.synchronize()
        self.tune_s += time.time() - tp

    def enqueue(self, stream, marks=None):
        nm = self.nm
        for i, l in enumerate(self.layers):
            nm.nm_conv2d(self.xs[i], self.packed[i], self.biases[i], l.stride, l.pad, l.dil, True,
                         y=self.ys[i], stream=stream)
            self.launched[i] = nm.nm_last_variant()     # what actually ran (cache, or the default)
            if marks is not None:
                marks[i + 1].record(stream)

    def time_steps(self, steps, warmup, use_graph=True):
        """(ms per step from HIP events on the launch stream, ms per step on the host clock).
        The launch-bound sequence of a step is captured once into a HIP graph (the library
        only enqueues kernels, so it can be captured) and replayed per step."""
        torch = self.torch
        stream = torch.cuda.current_stream()
        self.enqueue(stream)
        torch.cuda.synchronize()
        self.graph = None
        if use_graph:
            self.graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(self.graph):
                self.enqueue(torch.cuda.current_stream())
        run_step = self.graph.replay if self.graph is not None else (lambda: self.enqueue(stream))
        for _ in range(warmup):
            run_step()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_host0 = time.time()
        e0.record(stream)
        for _ in range(steps):
            run_step()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps, (time.time() - t_host0) * 1e3 / steps

    def time_floor(self, steps, warmup, use_graph=True):
        """ms per step of the same launch sequence with every convolution replaced by a kernel
        that only reads the layer's input and writes its output (nm_stream_floor): what the
        stack's own traffic costs on this device, launch for launch."""
        torch, nm = self.torch, self.nm
        stream = torch.cuda.current_stream()

        def enqueue(s):
            for x, y in zip(self.xs, self.ys):
                nm.nm_stream_floor(x, y, stream=s)
        enqueue(stream)
        torch.cuda.synchronize()
        graph = None
        if use_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                enqueue(torch.cuda.current_stream())
        run = graph.replay if graph is not None else (lambda: enqueue(stream))
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            run()
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / steps
        # per layer, with an event after every launch of a few extra eager passes
        n = len(self.layers)
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(n + 1)] for _ in range(3)]
        for k in range(3):
            marks[k][0].record(stream)
            for i, (x, y) in enumerate(zip(self.xs, self.ys)):
                nm.nm_stream_floor(x, y, stream=stream)
                marks[k][i + 1].record(stream)
        torch.cuda.synchronize()
        self.floor_ms = [sorted(marks[k][i].elapsed_time(marks[k][i + 1]) for k in range(3))[1] for i in range(n)]
        return ms

    def per_layer(self, inst_steps=3):
        """Per-layer kernel durations in the stack (HIP events on the launch stream): an event
        after every layer of a few extra steps, so that each layer is timed with the caches in
        the state the stack leaves them in."""
        torch, nm = self.torch, self.nm
        stream = torch.cuda.current_stream()
        marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(self.layers) + 1)]
                 for _ in range(inst_steps)]
        for k in range(inst_steps):
            marks[k][0].record(stream)
            self.enqueue(stream, marks[k])
        torch.cuda.synchronize()
        rows = []
        for i, l in enumerate(self.layers):
            ms = sorted(marks[k][i].elapsed_time(marks[k][i + 1]) for k in range(inst_steps))[inst_steps // 2]
            eff = l.effective_flops(self.B)
            byts = l.algorithmic_bytes(self.B, self.esize, self.esize_out)
            t_flop = eff / (PEAK_TFLOPS[self.dtype] * 1e12) * 1e3
            t_mem = byts / (PEAK_HBM_GBS * 1e9) * 1e3
            rows.append({
                "layer": l.name, "variant": nm.nm_variant_name(self.launched[i]),
                "ms": ms, "dense_gflops": l.dense_flops(self.B) / ms / 1e6, "eff_gflops": eff / ms / 1e6,
                "alg_bytes": byts, "gbs": byts / ms / 1e6, "t_flop_ms": t_flop, "t_mem_ms": t_mem,
                "t_min_ms": max(t_flop, t_mem),
                "bound": "mfma" if t_flop >= t_mem else "hbm", "frac": max(t_flop, t_mem) / ms,
            })
        return rows

    def totals(self):
        B = self.B
        return (sum(l.dense_flops(B) for l in self.layers), sum(l.effective_flops(B) for l in self.layers),
                sum(l.algorithmic_bytes(B, self.esize, self.esize_out) for l in self.layers))

    def free(self):
        for wp in self.packed:
            wp.free()
        self.packed, self.xs, self.ys, self.biases, self.graph = [], [], [], [], None
        self.torch.cuda.empty_cache()


def profiled_traffic(dtype):
    """HBM bytes per launch of the headline workload as the rocprofv3 counter runs recorded them
    (FETCH_SIZE + WRITE_SIZE, each scaled by what it reads for a 1 GiB device copy): read from
    the tracked summary under profiles/, never measured by this process.  (value, source)."""
    import re
    name = {"f32": "nm_conv_kernel_resnet50_b64_f32.txt", "bf16": "nm_conv_sp16_kernel_resnet50_b64_bf16.txt"}.get(dtype)
    if name is None:
        return None, None
    path = os.path.join(ROOT, "profiles", name)
    try:
        m = re.search(r"HBM traffic per step\s+[\d.]+ GB \(([\d.]+) MB per launch\)", open(path).read())
    except OSError:
        m = None
    if not m:
        return None, None
    return float(m.group(1)) * 1e6, f"profiles/{name} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this command)"


def stack_roofline(st, ms_step, rows, headline, floor_ms=None):
    """The convolution kernel, all launches of a step taken together, against the roofline that
    binds the workload: each layer's lower bound is max(effective flops / matrix-core peak,
    algorithmic bytes / HBM peak); the workload is bound by whichever side has the larger sum.
    The average launch duration comes from the timed region itself: the launches of a step run
    back to back on one stream, so step time / launches is the kernel's duration plus whatever
    gap the launches leave (an upper bound on the duration; the kernel trace shows no gap)."""
    dense, eff, byts = st.totals()
    kern_ms = sum(r["ms"] for r in rows)
    tmin_ms = sum(r["t_min_ms"] for r in rows)
    hbm_bound = sum(r["t_mem_ms"] for r in rows) >= sum(r["t_flop_ms"] for r in rows)
    if hbm_bound:
        roofline = {"bound": "hbm", "achieved": byts / ms_step / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": byts / ms_step / 1e6 / PEAK_HBM_GBS}
    else:
        roofline = {"bound": "mfma", "achieved": eff / ms_step / 1e9, "peak": PEAK_TFLOPS[st.dtype],
                    "unit": "TFLOP/s", "frac": eff / ms_step / 1e9 / PEAK_TFLOPS[st.dtype]}
    traffic, source = profiled_traffic(st.dtype) if headline else (None, None)
    families = sorted({(r["variant"] or "?").split("_")[0] for r in rows})
    roofline.update({
        "traffic": traffic, "traffic_source": source,
        "kernel": "nm_conv_sp16_kernel<F8> (+ nm_conv_f8_kernel)" if st.f8 else ("nm_conv_sp16_kernel" if st.bf16 else "nm_conv_kernel"),
        "variant_families": families,
        "launches_per_step": len(rows), "avg_launch_ms": ms_step / len(rows),
        # with an event after every layer of three extra steps (adds the events' own cost)
        "avg_launch_ms_event_per_layer": kern_ms / len(rows),
        # sum of the per-layer lower bounds over the step time: the fraction of the roofline
        # that binds each layer
        "frac_of_binding_roofline_per_layer": tmin_ms / ms_step,
        "effective_tflops": eff / ms_step / 1e9,
        "algorithmic_gbytes_per_step": byts / 1e9, "achieved_gbs": byts / ms_step / 1e6,
    })
    if floor_ms:
        # the same launches moving only each layer's input and output (nm_stream_floor), timed in
        # this run: the step time a stack of perfect copy kernels reaches on this device
        roofline["traffic_only_ms_per_step"] = floor_ms
        roofline["traffic_only_over_step"] = floor_ms / ms_step
    return roofline


def log_rows(rows, ms_step, ms_host):
    kern_ms = sum(r["ms"] for r in rows)
    tmin_ms = sum(r["t_min_ms"] for r in rows)
    for r in rows:
        log(f"{r['layer']:>18s} {r['variant']:>34s} {r['ms'] * 1e3:9.1f} us  "
            f"{r['eff_gflops'] / 1e3:7.1f} eff TF/s {r['gbs']:8.0f} GB/s  {r['bound']:4s} {r['frac'] * 100:5.1f}%"
            + (f"   traffic only {r['traffic_only_ms'] * 1e3:6.1f} us" if "traffic_only_ms" in r else ""))
    log(f"sum of kernel times {kern_ms:.3f} ms, step {ms_step:.3f} ms (host {ms_host:.3f} ms), "
        f"sum of per-layer lower bounds {tmin_ms:.3f} ms -> {tmin_ms / ms_step * 100:.1f}% of binding roofline")


def sweep_speedups(steps, warmup):
    """Sparse over dense per N:M ratio and tile size on the ResNet-50 stage-3 3x3 layer
    (14x14x256 -> 256, batch 32, fp32): every cell and the dense (N = M) form of the same layer
    at the same T, each through its tuned variant, launched in turn inside one graph so that
    no cell finds its tensors warmer than another's; median over the replays."""
    import torch
    from paper_2507_17301_amd import workloads as wl
    cells = wl.sweep_config2()
    tiles = sorted({c.tile for c in cells})
    dense = [wl.dense_form(next(c for c in cells if c.tile == t), f"cfg2_dense_T{t}") for t in tiles]
    st = Stack(cells + dense, 32, "f32", 0)
    st.tune()
    stream = torch.cuda.current_stream()
    st.enqueue(stream)
    torch.cuda.synchronize()
    reps = max(5, steps)
    times = [[] for _ in st.layers]
    for r in range(warmup + reps):
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(len(st.layers) + 1)]
        marks[0].record(stream)
        st.enqueue(stream, marks)
        torch.cuda.synchronize()
        if r >= warmup:
            for i in range(len(st.layers)):
                times[i].append(marks[i].elapsed_time(marks[i + 1]))
    med = [sorted(t)[len(t) // 2] for t in times]
    t_dense = {l.tile: med[len(cells) + k] for k, l in enumerate(dense)}
    out, vs_best = {}, {}
    best_dense = min(t_dense.values())
    for i, c in enumerate(cells):
        out.setdefault(f"{c.n}:{c.m}", {})[f"T{c.tile}"] = round(t_dense[c.tile] / med[i], 3)
        vs_best.setdefault(f"{c.n}:{c.m}", {})[f"T{c.tile}"] = round(best_dense / med[i], 3)
    detail = {"layer": "3x3 14x14x256->256 batch 32 fp32", "baseline": "per_ratio divides by the dense form at the "
              "same T; over_fastest_dense by the fastest dense form of any T", "over_fastest_dense": vs_best,
              "dense_us": {f"T{t}": round(v * 1e3, 2) for t, v in t_dense.items()},
              "sparse_us": {c.name: round(med[i] * 1e3, 2) for i, c in enumerate(cells)}}
    for k, v in out.items():
        log(f"sparse over dense {k:>4s}: " + "  ".join(f"{t} x{s:.2f}" for t, s in v.items()))
    st.free()
    return out, detail


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--dtype", choices=["f32", "bf16", "f8"], default="f32",
                    help="f8: E4M3 activations and weights with bf16 output, the fp8 second workload; layers whose "
                         "input channels are not a multiple of 64 (the first layer) are left out of that stack")
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
    ap.add_argument("--no-extras", action="store_true",
                    help="headline run only: skip the bf16 stack, the dense stack and the N:M sweep that the "
                         "default run measures besides the fp32 headline")
    ap.add_argument("--no-tune", action="store_true",
                    help="time the untuned default variants, then tune and time again: reports how far the "
                         "cost-model default is from the tuned pick")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch the kernels of a step one by one instead of replaying a HIP graph")
    ap.add_argument("--cache", default=None, help="tuning cache file to load/save")
    ap.add_argument("--report", default=None, help="write the per-layer table (JSON) here")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

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
    if args.dtype == "f8":
        kept = [l for l in layers if l.Cin % 64 == 0]
        if len(kept) != len(layers):
            wname += f"_fp8_layers_only_{len(kept)}_of_{len(layers)}"
        layers = kept
    if args.batch is not None:
        B = args.batch
    cand_tiles = [int(t) for t in args.tune_tile.split(",")] if args.tune_tile else None
    if cand_tiles:
        wname += "_T_per_layer_of_" + "_".join(str(t) for t in cand_tiles)
    headline = (args.workload == "resnet50" and B == 64 and not args.group and (n_, m_, t_) == (2, 4, 16)
                and not cand_tiles and args.dtype != "f8")

    # ---- one-time set-up: weights, pruning, tuning, resident inputs ---------
    if args.cache and os.path.exists(args.cache):
        nm.nm_cache_load(args.cache)
    t0 = time.time()
    st = Stack(layers, B, args.dtype, seed0, cand_tiles)
    layers = st.layers

    # a plain device copy of known size (1 GiB read + 1 GiB written): the yardstick
    # for the FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc
    cal_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    untuned = None
    if args.no_tune:
        # the cost-model default first, on an empty cache, then the tuned pick of the same layers
        ms_def, _ = st.time_steps(args.steps, args.warmup, not args.no_graph)
        rows_def = st.per_layer()
        untuned = {"ms_per_step": ms_def, "variants": [r["variant"] for r in rows_def]}
    st.tune()
    if args.cache:
        nm.nm_cache_save(args.cache)
    log(f"set-up {time.time() - t0:.1f}s (prune+pack {st.prune_s:.2f}s, tune {st.tune_s:.2f}s), "
        f"{len(layers)} layers, {nm.nm_cache_size()} tuned shapes")

    ms_step, ms_step_host = st.time_steps(args.steps, args.warmup, not args.no_graph)
    per_layer = st.per_layer()
    floor_ms = st.time_floor(args.steps, args.warmup, not args.no_graph)
    for r, f in zip(per_layer, st.floor_ms):
        r["traffic_only_ms"] = f
    log_rows(per_layer, ms_step, ms_step_host)
    dense, eff, byts = st.totals()
    log(f"traffic only (every layer's input read and output written by a plain streaming kernel, same "
        f"launch sequence): {floor_ms:.3f} ms per step = {floor_ms / ms_step * 100:.0f}% of the step")
    roofline = stack_roofline(st, ms_step, per_layer, headline, floor_ms)
    launch = "hip_graph_replay" if st.graph is not None else "one_launch_per_layer"
    if untuned:
        same = sum(a == r["variant"] for a, r in zip(untuned["variants"], per_layer))
        untuned.update({"tuned_ms_per_step": ms_step, "default_over_tuned": untuned["ms_per_step"] / ms_step,
                        "layers_where_default_is_the_tuned_pick": same, "layers": len(per_layer)})
        del untuned["variants"]
        log(f"untuned default {untuned['ms_per_step']:.3f} ms per step = x{untuned['default_over_tuned']:.2f} "
            f"of the tuned {ms_step:.3f} ms; the default is the tuned pick on {same} of {len(per_layer)} layers")

    if args.workload == "sweep":
        # sparse-over-dense speedup per cell: the dense form of the same layer through the same kernel family
        t_dense = per_layer[-1]["ms"]
        for r in per_layer[:-1]:
            r["speedup_over_dense"] = t_dense / r["ms"]
            log(f"{r['layer']:>18s}  {r['ms'] * 1e3:7.1f} us   x{r['speedup_over_dense']:.2f} over dense ({t_dense * 1e3:.1f} us)")

    # ---- what the headline run reports besides the fp32 figure: the same stack with bf16
    # tensors, and sparse over dense -- for the stack (its N = M form through the same kernels)
    # and per N:M ratio and tile size on the stage-3 3x3 layer
    extras = {}
    if headline and args.dtype == "f32" and not args.no_extras and not args.no_tune:
        st.free()
        sb = Stack(wl.resnet50_stack(2, 4, 16), B, "bf16", seed0)
        sb.tune()
        ms_b, ms_b_host = sb.time_steps(args.steps, args.warmup, not args.no_graph)
        rows_b = sb.per_layer()
        floor_b = sb.time_floor(args.steps, args.warmup, not args.no_graph)
        for r, f in zip(rows_b, sb.floor_ms):
            r["traffic_only_ms"] = f
        log("--- bf16 tensors, same stack")
        log_rows(rows_b, ms_b, ms_b_host)
        d_b, e_b, by_b = sb.totals()
        log(f"traffic only, bf16: {floor_b:.3f} ms per step = {floor_b / ms_b * 100:.0f}% of the step")
        rf_b = stack_roofline(sb, ms_b, rows_b, True, floor_b)
        extras["bf16"] = {"ms_per_step": ms_b, "ms_per_img": ms_b / B, "dense_equiv_gflops": d_b / ms_b / 1e6,
                          "effective_gflops": e_b / ms_b / 1e6, "launches": len(rows_b),
                          "algorithmic_gbs": by_b / ms_b / 1e6, "setup": {"prune_pack_s": sb.prune_s, "autotune_s": sb.tune_s},
                          "roofline": rf_b}
        sb.free()
        s8 = Stack([l for l in wl.resnet50_stack(2, 4, 16) if l.Cin % 64 == 0], B, "f8", seed0 + 1)
        s8.tune()
        ms_8, ms_8_host = s8.time_steps(args.steps, args.warmup, not args.no_graph)
        rows_8 = s8.per_layer()
        floor_8 = s8.time_floor(args.steps, args.warmup, not args.no_graph)
        for r, f in zip(rows_8, s8.floor_ms):
            r["traffic_only_ms"] = f
        log("--- fp8 (E4M3 activations and weights, bf16 output), the 52 pruned layers of the stack")
        log_rows(rows_8, ms_8, ms_8_host)
        d_8, e_8, by_8 = s8.totals()
        extras["fp8"] = {"workload": "resnet50_conv_stack_52_pruned_layers_2of4_T16_batch64_e4m3_in_bf16_out",
                         "ms_per_step": ms_8, "ms_per_img": ms_8 / B, "dense_equiv_gflops": d_8 / ms_8 / 1e6,
                         "effective_gflops": e_8 / ms_8 / 1e6, "launches": len(rows_8),
                         "algorithmic_gbs": by_8 / ms_8 / 1e6,
                         "setup": {"prune_pack_s": s8.prune_s, "autotune_s": s8.tune_s},
                         "roofline": stack_roofline(s8, ms_8, rows_8, False, floor_8)}
        s8.free()
        sd = Stack(wl.resnet50_stack(1, 1, 16), B, "f32", seed0)
        sd.tune()
        ms_d, _ = sd.time_steps(args.steps, args.warmup, not args.no_graph)
        sd.free()
        log(f"--- dense (N = M) form of the stack, fp32: {ms_d:.3f} ms per step -> 2:4 is x{ms_d / ms_step:.2f} faster")
        sweep, detail = sweep_speedups(args.steps, args.warmup)
        extras["speedup_over_dense"] = {"resnet50_stack_2:4_T16_batch64_f32": round(ms_d / ms_step, 3),
                                        "dense_stack_ms_per_step": ms_d, "per_ratio": sweep, "per_ratio_detail": detail}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(layers, B, args.dtype == "bf16", seed0)

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
                   "batch": B, "layers": len(layers), "tuned": True, "launch": launch},
        "setup": {"prune_pack_s": st.prune_s, "autotune_s": st.tune_s},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    out.update(extras)
    if untuned:
        out["untuned_default"] = untuned
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


def host_cores():
    """Cores this process may use: the CPU affinity mask, cut down to the cgroup's CPU quota
    where one is set (a box may show every core of the host and still grant a share)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    try:
        quota, period = open("/sys/fs/cgroup/cpu.max").read().split()
        if quota != "max":
            n = max(1, min(n, int(int(quota) / int(period))))
    except (OSError, ValueError):
        pass
    return n


def cpu_baseline(layers, B, bf16, seed0):
    """The CPU oracle, as it stands, on the first images of the same workload, on every core
    this process may use; plus the single 3x3 layer of configuration 1 on one thread."""
    import numpy as np
    import oracle
    from paper_2507_17301_amd import workloads as wl

    cores = host_cores()
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
    nimg = int(max(2, min(B, round(12.0 / max(t1, 1e-3)))))
    t = run(nimg)
    dense_per_img = sum(l.dense_flops(1) for l, _, _ in prepared)
    log(f"cpu oracle: {nimg} images in {t:.2f}s on {cores} threads (host shows {os.cpu_count()} cores)")

    c1 = wl.single_conv_config1()
    x1, w1, b1 = wl.make_tensors(c1, 1, 0, weight_sigma=0.05)
    _, _, wz1 = oracle.prune(w1, c1.n, c1.m, c1.tile)
    ts = []
    for _ in range(3):
        tt = time.time()
        oracle.conv2d(x1, wz1, b1, c1.stride, c1.pad, c1.dil, True, nthreads=1)
        ts.append(time.time() - tt)
    t_c1 = sorted(ts)[1]
    log(f"cpu oracle, configuration 1 (one 3x3 layer, batch 1) on one thread: {t_c1 * 1e3:.1f} ms")
    return {"value": dense_per_img * nimg / t / 1e9, "unit": "GFLOP/s", "cores": cores,
            "host_cores": os.cpu_count(), "kind": "oracle", "ms_per_img": t * 1e3 / nimg,
            "sample": f"first {nimg} of {B} images through all {len(prepared)} layers "
                      f"(direct convolution on zero-filled weights, fp64 accumulate)",
            "config1_one_thread": {"value": c1.dense_flops(1) / t_c1 / 1e9, "unit": "GFLOP/s", "cores": 1,
                                   "ms": t_c1 * 1e3, "sample": "the single 3x3 layer 56x56x64->64, batch 1, whole output"}}


if __name__ == "__main__":
    main()

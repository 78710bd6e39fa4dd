#!/usr/bin/env python3
"""Benchmark of the Tucker-2 convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path over the ResNet-18-shaped sweep at batch 1
(four layers: C=N in {64,128,256,512} at 56/28/14/7 pixels, R1=R2=C/4, 3x3, stride 1, pad 1,
fp32), each layer one tdc_conv_tucker2 call on the current stream with inputs and re-laid-out
weights already resident in HBM.  Prints ONE JSON line.

  value        effective GFLOP/s of the sweep: algorithmic FLOPs of the four layers / step time
  layers       per layer: latency_us (event-timed over back-to-back launches on one stream, the
               primary figure), sync_latency_us (one launch + host synchronise, median),
               cold_latency_us (back-to-back launches that cycle through more than 512 MB of distinct
               x / y buffers, so no activation is found in a cache), GFLOP/s, the fraction of the
               layer's roofline max(bytes/8 TB/s, flops/157.3 TFLOP/s), dense_conv_us (this
               library's kernel for the undecomposed K x K layer, timed the same way) and oracle_us
               (the CPU oracle's three-stage and dense paths, all host threads and one thread)
  roofline     the same for the dominant (slowest) layer's kernel
  null_launch_us  an empty kernel timed the same way: the floor any batch-1 layer sits on
  throughput_regime  the batch-32 128->256 stride-2 layer (config 4) timed the same way, against the
               fp32 MFMA peak: a side figure, not part of value
  cpu_baseline the CPU oracle (three-stage, fp64) timed on the host cores on the same sweep
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

# HBM bytes per layer call (all its kernels) from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/cfg2.txt, each scaled by what the same counter reads for a plain 256 MiB
# device copy (FETCH_SIZE under-reads 2.0x on this machine, WRITE_SIZE is exact): (fetched, written) KiB,
# keyed by layer name and the variant that was profiled.
MEASURED_TRAFFIC = {
    ("b1_c64_n64_56x56_r16-16_k3_s1_p1", "fused-merged"): (5819.3, 784.0),
    ("b1_c128_n128_28x28_r32-32_k3_s1_p1", "fused-merged"): (4570.4, 784.0),
    ("b1_c256_n256_14x14_r64-64_k3_s1_p1", "merged"): (1082.9 + 1054.9, 49.0 + 196.0),
    ("b1_c512_n512_7x7_r128-128_k3_s1_p1", "merged"): (1110.9 + 2586.7, 24.5 + 98.0),
}


def _time_events(fn, iters, torch):
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) * 1e-3 / iters   # seconds per call


def _time_sync(fn, iters, torch):
    """Median wall time of one launch followed by a host synchronise."""
    ts = []
    for _ in range(iters):
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        ts.append(time.perf_counter() - t0)
    ts.sort()
    return ts[len(ts) // 2]


def _time_cold(conv, L, x, torch, min_bytes=512 << 20, max_sets=2048):
    """Seconds per call when every call reads and writes buffers no earlier call of the pass touched."""
    y_shape = conv.out_shape()
    per_set = 4 * (x.numel() + L.batch * L.N * conv.Ho * conv.Wo)
    n_sets = max(2, min(max_sets, -(-min_bytes // per_set)))
    xs = [x.clone() for _ in range(n_sets)]
    ys = [torch.empty(y_shape, device=x.device, dtype=torch.float32) for _ in range(n_sets)]
    launchers = [conv.bind(a, b) for a, b in zip(xs, ys)]
    for launch in launchers:                       # one untimed pass: page tables, code
        launch()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for launch in launchers:
        launch()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) * 1e-3 / n_sets, n_sets


def oracle_layer_times(L, inp, budget_s=1.5):
    """CPU oracle on one image of the layer: three-stage and dense paths, all threads and one thread (us)."""
    from oracle import tdc_oracle as orc
    orc.load()
    d = L.asdict()
    d["batch"] = 1
    sh = orc.Shape(**d)
    one = dict(inp, x=inp["x"][:1])
    Wd, _ = orc.reconstruct(sh, one["U_in"], one["core"], one["U_out"])
    out = {"images": 1}
    nmax = orc.max_threads()
    for label, nthr in (("all", nmax), ("1t", 1)):
        orc.set_threads(nthr)
        for name, fn in (("factored", lambda: orc.conv_factored(sh, **one)),
                         ("dense", lambda: orc.conv_dense_with(sh, one["x"], Wd))):
            fn()
            best, t_begin = 1e30, time.perf_counter()
            for _ in range(5):
                t0 = time.perf_counter()
                fn()
                best = min(best, time.perf_counter() - t0)
                if time.perf_counter() - t_begin > budget_s / 4:
                    break
            out["%s_%s" % (name, label)] = best * 1e6
    orc.set_threads(nmax)
    return out


def cpu_baseline(layers, inputs, budget_s=12.0, max_sweeps=100000):
    """The oracle as it stands (three-stage, Eqs. 2-4, fp64 accumulation, OpenMP over output channels)."""
    from oracle import tdc_oracle as orc
    from paper_2211_03715_amd import roofline as R
    orc.load()
    shapes = [orc.Shape(**L.asdict()) for L in layers]
    fl = sum(R.flops(L) for L in layers)
    for sh, inp in zip(shapes, inputs):          # warm caches / thread pool
        orc.conv_factored(sh, **inp)
    t0 = time.perf_counter()
    sweeps = 0
    while sweeps < max_sweeps and time.perf_counter() - t0 < budget_s:
        for sh, inp in zip(shapes, inputs):
            orc.conv_factored(sh, **inp)
        sweeps += 1
    dt = time.perf_counter() - t0
    return {"value": fl * sweeps / dt / 1e9, "unit": "GFLOP/s", "cores": orc.max_threads(), "kind": "oracle",
            "sample": "%d passes over the same %d layer(s), three-stage path, %.1f s wall" % (sweeps, len(layers), dt),
            "us_per_sweep": dt / sweeps * 1e6}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, help="workload id 1..5 (default: the ResNet-18-shaped sweep)")
    ap.add_argument("--variant", default="auto", choices=["auto", "naive", "split", "fused", "chain", "merged", "fused_merged"])
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"],
                    help="activation layout (default NCHW, the layout the metric's workload is stated in)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg and the per-layer oracle times")
    ap.add_argument("--brief", action="store_true",
                    help="only the queued latency per layer (no sync / cold-cache / dense-kernel columns)")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2211_03715_amd import binding as B
    from paper_2211_03715_amd import roofline as R
    from paper_2211_03715_amd.layer import DenseConv2d, TuckerConv2d
    from paper_2211_03715_amd.workloads import config_layers, layer_seed, make_dense_inputs, make_inputs

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.load()                                   # fails loudly if libtdc.so has not been built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    variant = {"auto": B.VARIANT_AUTO, "naive": B.VARIANT_NAIVE, "split": B.VARIANT_SPLIT,
               "fused": B.VARIANT_FUSED, "chain": B.VARIANT_CHAIN, "merged": B.VARIANT_MERGED,
               "fused_merged": B.VARIANT_FUSED_MERGED}[args.variant]

    layout = B.LAYOUT_NHWC if args.layout == "nhwc" else B.LAYOUT_NCHW
    layers = config_layers(args.config)
    host_inputs = [make_inputs(L, layer_seed(args.config, i)) for i, L in enumerate(layers)]
    convs, xs, ys = [], [], []
    for L, inp in zip(layers, host_inputs):
        t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
        conv = TuckerConv2d(L, 0, B.make_tuning(variant=variant) if variant else None, layout=layout)
        conv.pack(t["U_in"], t["core"], t["U_out"])         # one-off re-layout, untimed (as in the paper)
        convs.append(conv)
        xs.append(t["x"].permute(0, 2, 3, 1).contiguous() if layout == B.LAYOUT_NHWC else t["x"])
        ys.append(torch.empty(conv.out_shape(), device=dev, dtype=torch.float32))
    torch.cuda.synchronize()

    # arguments marshalled once; one foreign call per layer and step
    launchers = [conv.bind(x, y) for conv, x, y in zip(convs, xs, ys)]

    def step():
        for launch in launchers:
            launch()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    total_flops = sum(R.flops(L) for L in layers)

    # per-layer: events around back-to-back launches of that layer alone, on the launch stream
    iters = max(200, min(2000, args.steps))
    # (all layers first, before the slower side measurements below leave the GPU idle between launches)
    queued = []
    for launch in launchers:
        for _ in range(200):                      # clocks and caches settled before the timed launches
            launch()
        queued.append(_time_events(launch, iters, torch))
    per_layer = []
    for i, (L, conv, launch) in enumerate(zip(layers, convs, launchers)):
        sec = queued[i]
        bound, t_roof, t_hbm, t_mfma = R.roofline(L)
        row = {
            "layer": L.name(), "plan": conv.describe(), "kernels": conv.kernel_count(),
            "latency_us": sec * 1e6, "gflops": R.flops(L) / sec / 1e9,
            "dense_equiv_gflops": R.dense_flops(L) / sec / 1e9,
            "bound": bound, "roofline_us": t_roof * 1e6, "roofline_frac": t_roof / sec,
        }
        if not args.brief:
            row["sync_latency_us"] = _time_sync(launch, 200, torch) * 1e6
            cold, n_sets = _time_cold(conv, L, xs[i], torch)
            row["cold_latency_us"], row["cold_buffer_sets"] = cold * 1e6, n_sets
            # the undecomposed layer on this library's own dense kernel (the t2 of the paper's threshold test)
            dense = DenseConv2d(L, 0, layout=layout)
            W = torch.from_numpy(make_dense_inputs(L, layer_seed(args.config, i) + 500)["W"]).to(dev)
            dense.pack(W)
            dl = dense.bind(xs[i], ys[i])
            for _ in range(20):
                dl()
            row["dense_conv_us"] = _time_events(dl, max(50, iters // 4), torch) * 1e6
            row["dense_conv_plan"] = dense.describe()
            row["speedup_vs_dense_conv"] = row["dense_conv_us"] / row["latency_us"]
            torch.cuda.synchronize()
            dense.close()
            launch()                              # ys[i] holds the Tucker layer's output again
        per_layer.append(row)
    import ctypes
    null_fn, null_stream = B.load().tdc_launch_null, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    null_us = _time_events(lambda: null_fn(null_stream), 2000, torch) * 1e6
    null_sync_us = _time_sync(lambda: null_fn(null_stream), 200, torch) * 1e6

    for row in per_layer:
        row["null_launch_us"] = null_us          # the floor any launch pays, beside every latency
    dom = max(range(len(layers)), key=lambda i: per_layer[i]["latency_us"])
    Ld, pd = layers[dom], per_layer[dom]
    sec = pd["latency_us"] * 1e-6
    if pd["bound"] == "hbm":
        roof = {"bound": "hbm", "achieved": R.bytes_compulsory(Ld) / sec / 1e9, "peak": R.HBM_PEAK / 1e9, "unit": "GB/s"}
    else:
        roof = {"bound": "mfma", "achieved": R.flops(Ld) / sec / 1e12, "peak": R.FP32_MFMA_PEAK / 1e12, "unit": "TFLOP/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    traffic = MEASURED_TRAFFIC.get((Ld.name(), pd["plan"].split(" ")[0])) if layout == B.LAYOUT_NCHW else None
    roof["traffic"] = None if traffic is None else (traffic[0] + traffic[1]) * 1024.0      # bytes per layer call
    roof["traffic_fetch_write_kib"] = traffic
    roof["algorithmic_bytes"] = R.bytes_compulsory(Ld)
    roof["kernel"] = pd["plan"]
    roof["layer"] = Ld.name()
    roof["launch_us"] = pd["latency_us"]

    out = {
        "metric": "effective GFLOP/s (algorithmic FLOPs of the Tucker-2 layers / time), batch 1, per-layer latency in `layers`",
        "value": total_flops / (dt / args.steps) / 1e9, "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s" % (args.config, {
            1: "single Tucker-2 3x3 layer 64->16->16->64 at 56x56, batch 1",
            2: "ResNet-18-shaped sweep, batch 1, 3x3 s1 p1, (C=N,HxW) in (64,56) (128,28) (256,14) (512,7), R1=R2=C/4",
            3: "rank sweep at C=N=256, 14x14, (R1,R2) in {8,16,32,64,128}^2, batch 1",
            4: "stride/batch variants: 128->256 s2 56->28 r32/64 and 128->128 28x28 r32, batch 1/8/32",
            5: "ResNet-50-style chain of 16 Tucker-2 3x3 layers, ranks round(0.3C) to 8, batch 1"}[args.config]),
            "layers_per_step": len(layers), "variant": args.variant, "layout": args.layout},
        "roofline": roof,
        "layers": per_layer,
        "null_launch_us": null_us,
        "null_sync_us": null_sync_us,
        "sum_layer_latency_us": sum(p["latency_us"] for p in per_layer),
    }
    if not args.brief:
        # the same step replayed from a HIP graph (captured once; no memset nodes: the launch path records none)
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            cap = [conv.bind(x, y) for conv, x, y in zip(convs, xs, ys)]     # launchers carry their stream
            for launch in cap:
                launch()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for launch in cap:
                    launch()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(20):
            graph.replay()
        out["graph_replay_us_per_step"] = _time_events(graph.replay, max(200, min(2000, args.steps)), torch) * 1e6
        torch.cuda.synchronize()
        del graph
    if layout == B.LAYOUT_NCHW and not args.brief:
        # the same step with pixel-major activations (tdc_shape.layout = 1): reported beside the NCHW figure
        n_convs, n_x, n_y = [], [], []
        for L, conv, x in zip(layers, convs, xs):
            c2 = TuckerConv2d(L, 0, B.make_tuning(variant=variant) if variant else None, layout=B.LAYOUT_NHWC)
            c2.pack(*conv._weights)
            n_convs.append(c2)
            n_x.append(x.permute(0, 2, 3, 1).contiguous())
            n_y.append(torch.empty(c2.out_shape(), device=dev, dtype=torch.float32))
        n_launch = [c.bind(x, y) for c, x, y in zip(n_convs, n_x, n_y)]

        def n_step():
            for launch in n_launch:
                launch()

        for _ in range(args.warmup):
            n_step()
        n_sec = _time_events(n_step, args.steps, torch)
        out["nhwc"] = {"value": total_flops / n_sec / 1e9, "unit": "GFLOP/s", "ms_per_step": n_sec * 1e3,
                       "layers": [{"layer": L.name(), "plan": c.describe(), "latency_us": _time_events(l, iters, torch) * 1e6}
                                  for L, c, l in zip(layers, n_convs, n_launch)]}
        torch.cuda.synchronize()
        for c in n_convs:
            c.close()
    if args.config == 2 and variant == 0 and not args.brief:
        # beside the latency-bound headline: the one layer of config 4 whose batch fills the chip, against the
        # same fp32 MFMA peak (a reported side figure; `value` and `roofline` above are the batch-1 sweep's)
        Lt = config_layers(4)[2]
        inp = make_inputs(Lt, layer_seed(4, 2))
        t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
        ct = TuckerConv2d(Lt, 0, None, layout=layout)
        ct.pack(t["U_in"], t["core"], t["U_out"])
        xt = t["x"].permute(0, 2, 3, 1).contiguous() if layout == B.LAYOUT_NHWC else t["x"]
        yt = torch.empty(ct.out_shape(), device=dev, dtype=torch.float32)
        lt = ct.bind(xt, yt)
        for _ in range(200):
            lt()
        t_sec = _time_events(lt, 500, torch)
        out["throughput_regime"] = {
            "layer": Lt.name(), "plan": ct.describe(), "latency_us": t_sec * 1e6,
            "roofline": {"bound": "mfma", "achieved": R.flops(Lt) / t_sec / 1e12, "peak": R.FP32_MFMA_PEAK / 1e12,
                         "unit": "TFLOP/s", "frac": R.flops(Lt) / t_sec / R.FP32_MFMA_PEAK}}
        torch.cuda.synchronize()
        ct.close()
        del xt, yt, t
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(layers, host_inputs)
        if not args.brief:
            for row, L, inp in zip(per_layer, layers, host_inputs):
                row["oracle_us"] = oracle_layer_times(L, inp)
                # a reported baseline, not a target: the oracle on one image, all host threads, against the layer per image
                row["speedup_vs_oracle"] = row["oracle_us"]["factored_all"] * L.batch / row["latency_us"]
    if args.copy_mib > 0:
        src = torch.empty(args.copy_mib * 262144, device=dev, dtype=torch.float32).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_mib"] = args.copy_mib
    for conv in convs:
        conv.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()

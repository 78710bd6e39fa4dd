#!/usr/bin/env python3
"""Benchmark of the Tucker-2 convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path over the ResNet-18-shaped sweep at batch 1
(four layers: C=N in {64,128,256,512} at 56/28/14/7 pixels, R1=R2=C/4, 3x3, stride 1, pad 1,
fp32), each layer one tdc_conv_tucker2 call on the current stream with inputs and re-laid-out
weights already resident in HBM.  Prints ONE JSON line.

  value        effective GFLOP/s of the sweep: algorithmic FLOPs of the four layers / step time
  layers       per layer: latency_us (event-timed over back-to-back launches on one stream, the
               primary figure: median of 7 repeats, with min and max), sync_latency_us (one launch + host synchronise, median),
               cold_latency_us (back-to-back launches that cycle through more than 512 MB of distinct
               x / y buffers, so no activation is found in a cache), GFLOP/s, the fraction of the
               layer's roofline max(bytes/8 TB/s, flops/157.3 TFLOP/s), dense_conv_us (this
               library's kernel for the undecomposed K x K layer, timed the same way) and oracle_us
               (the CPU oracle's three-stage and dense paths, all host threads and one thread),
               achieved_hbm_gbs (compulsory bytes over the cold-cache latency), traffic_bytes (see roofline);
               one_launch, for a layer whose plan takes two launches (MERGED): the same work in ONE launch
               (MERGED_XCD, with a barrier among the workgroups of each XCD), timed like latency_us
  roofline     the same for the dominant (slowest) layer's kernel; traffic = HBM bytes per call measured with
               rocprofv3 for exactly this plan, looked up in profiles/traffic.txt (null for a plan not profiled)
  null_launch_us  an empty kernel timed the same way: the floor any batch-1 layer sits on
  throughput_regime  the batch-32 128->256 stride-2 layer (config 4) timed the same way, against the
               fp32 MFMA peak: a side figure, not part of value; throughput_layers lists it with the
               other batched layers (28x28 and 14x14 at batch 32, 128 and 256, the stride-2 layer at batch 64); each
               carries `concurrent`: time per call with 2 / 3 / 4 independent calls in flight on as many streams
  resnet50_body  the 16 bottleneck blocks (65 kernels) of a ResNet-50-shaped network at batch 1, eagerly and as
               one HIP graph, NCHW and NHWC; resnet18_body the same for the 8 basic blocks (16 Tucker-2 layers) of a
               ResNet-18-shaped one
  graph_replay_us_per_step  the step replayed from a HIP graph (--graph-study explains the difference to eager)
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

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "traffic.txt")


def measured_traffic(layer_name, layout, plan):
    """HBM bytes one call of `layer_name` moved when it was profiled with exactly this plan, from profiles/traffic.txt
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by what the counter reads for a plain device copy of known
    size; the file names its runs).  None when no profile of this plan exists: a changed tuning never carries the
    bytes of another one."""
    key = plan.split(" model=")[0].strip()
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                if line.startswith("#") or not line.strip():
                    continue
                cols = [c.strip() for c in line.rstrip("\n").split("|")]
                if len(cols) >= 5 and cols[0] == layer_name and cols[1] == layout and cols[2] == key:
                    return float(cols[3]), float(cols[4])
    except OSError:
        pass
    return None


def _time_repeats(fn, iters, repeats, torch):
    """`repeats` event-timed runs of `iters` back-to-back launches: (median, min, max) seconds per call.  The spread
    shows the two clock / power states a run of launches can land in."""
    ts = sorted(_time_events(fn, iters, torch) for _ in range(repeats))
    return ts[len(ts) // 2], ts[0], ts[-1]


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


def _in_flight(torch, Lt, t, xt, yt, layout, n_cus, n_str, share, rounds_timed=100, repeats=5):
    """`n_str` independent calls of layer Lt in flight: one plan, one set of buffers and one stream (default priority)
    per call, launched round-robin; plans made for 1/`share` of the chip.  Returns (sorted seconds per call, plan)."""
    from paper_2211_03715_amd import binding as B
    from paper_2211_03715_amd.layer import TuckerConv2d
    shape_t = B.make_shape(**Lt.asdict(), layout=layout)
    streams = [torch.cuda.Stream() for _ in range(n_str)]
    cs, ls, keep = [], [], []
    for st in streams:
        tun = B.tdc_select_tuning(shape_t, compute_units=n_cus // share) if share > 1 else None
        c = TuckerConv2d(Lt, 0, tun, layout=layout)
        c.pack(t["U_in"], t["core"], t["U_out"])
        xs_, ys_ = xt.clone(), torch.empty_like(yt)
        keep.append((xs_, ys_))
        torch.cuda.synchronize()
        ls.append(c.bind(xs_, ys_, stream=st.cuda_stream))
        cs.append(c)

    def rounds(n):
        for _ in range(n):
            for l in ls:
                l()

    rounds(30)
    torch.cuda.synchronize()
    per_call = []
    for _ in range(repeats):
        t0 = time.perf_counter()
        rounds(rounds_timed)
        torch.cuda.synchronize()
        per_call.append((time.perf_counter() - t0) / (rounds_timed * n_str))
    plan = cs[0].describe()
    for c in cs:
        c.close()
    per_call.sort()
    return per_call, plan


def in_flight_only(args):
    """--in-flight LAYER:STREAMS:SHARE -- only that measurement, for a kernel trace of calls in flight: layer LAYER of
    workload 6 with STREAMS calls in flight and plans made for 1/SHARE of the chip; then the same layer on one stream."""
    import torch
    from paper_2211_03715_amd import binding as B, roofline as R
    from paper_2211_03715_amd.layer import TuckerConv2d
    from paper_2211_03715_amd.workloads import config_layers, layer_seed, make_inputs
    idx, n_str, share = (int(v) for v in args.in_flight.split(":"))
    B.load()
    dev = torch.device("cuda:0")
    layout = B.LAYOUT_NHWC if args.layout == "nhwc" else B.LAYOUT_NCHW
    Lt = config_layers(6)[idx]
    t = {k: torch.from_numpy(v).to(dev) for k, v in make_inputs(Lt, layer_seed(6, idx)).items()}
    xt = t["x"].permute(0, 2, 3, 1).contiguous() if layout == B.LAYOUT_NHWC else t["x"]
    ct = TuckerConv2d(Lt, 0, None, layout=layout)
    yt = torch.empty(ct.out_shape(), device=dev, dtype=torch.float32)
    n_cus = torch.cuda.get_device_properties(dev).multi_processor_count
    pc, plan = _in_flight(torch, Lt, t, xt, yt, layout, n_cus, n_str, share, rounds_timed=200, repeats=3)
    ct.pack(t["U_in"], t["core"], t["U_out"])
    lt = ct.bind(xt, yt)
    for _ in range(100):
        lt()
    alone, _, _ = _time_repeats(lt, 200, 3, torch)
    torch.cuda.synchronize()
    print(json.dumps({"layer": Lt.name(), "layout": args.layout, "streams": n_str, "planned_for_chip_share": "1/%d" % share,
                      "plan_in_flight": plan, "us_per_call_in_flight": pc[len(pc) // 2] * 1e6,
                      "frac_of_fp32_mfma_peak_in_flight": R.flops(Lt) / pc[len(pc) // 2] / R.FP32_MFMA_PEAK,
                      "plan_alone": ct.describe(), "us_per_call_alone": alone * 1e6,
                      "frac_of_fp32_mfma_peak_alone": R.flops(Lt) / alone / R.FP32_MFMA_PEAK}))
    ct.close()
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--config", type=int, default=2, help="workload id 1..7 (default 2: the ResNet-18-shaped sweep)")
    ap.add_argument("--variant", default="auto", choices=["auto", "naive", "split", "fused", "chain", "merged", "fused_merged", "merged_xcd"])
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"],
                    help="activation layout (default NCHW, the layout the metric's workload is stated in)")
    ap.add_argument("--in-flight", default="", metavar="LAYER:STREAMS:SHARE",
                    help="only: layer LAYER of workload 6 with STREAMS calls in flight, plans for 1/SHARE of the chip (for a kernel trace)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg and the per-layer oracle times")
    ap.add_argument("--brief", action="store_true",
                    help="only the queued latency per layer (no sync / cold-cache / dense-kernel columns)")
    ap.add_argument("--copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by)")
    ap.add_argument("--graph-study", action="store_true",
                    help="only the step, --steps times eagerly, then (after a 50 ms pause that separates the two in a kernel "
                         "trace) --steps replays of its HIP graph; prints both per-step times and exits")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")
    if args.in_flight:
        import torch
        if not torch.cuda.is_available():
            sys.exit("bench.py needs a GPU")
        return in_flight_only(args)

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
               "fused_merged": B.VARIANT_FUSED_MERGED, "merged_xcd": B.VARIANT_MERGED_XCD}[args.variant]

    layout = B.LAYOUT_NHWC if args.layout == "nhwc" else B.LAYOUT_NCHW
    layers = config_layers(args.config)
    host_inputs = [make_inputs(L, layer_seed(args.config, i)) for i, L in enumerate(layers)]
    convs, xs, ys, ws = [], [], [], []
    for L, inp in zip(layers, host_inputs):
        t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
        conv = TuckerConv2d(L, 0, B.make_tuning(variant=variant) if variant else None, layout=layout)
        conv.pack(t["U_in"], t["core"], t["U_out"])         # one-off re-layout, untimed (as in the paper)
        convs.append(conv)
        ws.append(t)
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
    if args.graph_study:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            cap = [conv.bind(x, y) for conv, x, y in zip(convs, xs, ys)]     # launchers carry their stream
            for launch in cap:
                launch()
        graph8 = torch.cuda.CUDAGraph()                                       # eight steps in one graph
        with torch.cuda.graph(graph8):
            for _ in range(8):
                for launch in cap:
                    launch()
        for _ in range(args.warmup):
            graph.replay()
            graph8.replay()
        torch.cuda.synchronize()
        res = {"steps": args.steps, "kernels_per_step": sum(c.kernel_count() for c in convs)}
        for name, fn, per in (("eager", step, 1), ("graph", graph.replay, 1), ("graph_of_8_steps", graph8.replay, 8)):
            time.sleep(0.05)
            t0 = time.perf_counter()
            for _ in range(args.steps // per):
                fn()
            t_enq = time.perf_counter() - t0
            torch.cuda.synchronize()
            n = args.steps // per * per
            res[name + "_us_per_step"] = (time.perf_counter() - t0) / n * 1e6
            res[name + "_host_enqueue_us_per_step"] = t_enq / n * 1e6
        print(json.dumps(res))
        return
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
        queued.append(_time_repeats(launch, max(100, iters // 4), 7, torch))
    per_layer = []
    for i, (L, conv, launch) in enumerate(zip(layers, convs, launchers)):
        sec, sec_min, sec_max = queued[i]
        bound, t_roof, t_hbm, t_mfma = R.roofline(L)
        row = {
            "layer": L.name(), "plan": conv.describe(), "kernels": conv.kernel_count(),
            "latency_us": sec * 1e6, "latency_us_min": sec_min * 1e6, "latency_us_max": sec_max * 1e6,
            "latency_repeats": 7, "gflops": R.flops(L) / sec / 1e9,
            "dense_equiv_gflops": R.dense_flops(L) / sec / 1e9,
            "bound": bound, "roofline_us": t_roof * 1e6, "roofline_frac": t_roof / sec,
        }
        if not args.brief:
            row["sync_latency_us"] = _time_sync(launch, 200, torch) * 1e6
            cold, n_sets = _time_cold(conv, L, xs[i], torch)
            row["cold_latency_us"], row["cold_buffer_sets"] = cold * 1e6, n_sets
            # compulsory bytes over the cold-cache latency: what the layer pulls from HBM when nothing is cached
            row["achieved_hbm_gbs"] = R.bytes_compulsory(L) / cold / 1e9
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
            if conv.kernel_count() == 2:
                # the two-launch MERGED plan against the same work in ONE launch (MERGED_XCD, never the selector's choice)
                try:
                    one = TuckerConv2d(L, 0, B.make_tuning(variant=B.VARIANT_MERGED_XCD), layout=layout)
                except B.TdcError:
                    one = None
                if one is not None:
                    one.pack(ws[i]["U_in"], ws[i]["core"], ws[i]["U_out"])
                    ol = one.bind(xs[i], ys[i])
                    for _ in range(100):
                        ol()
                    o_sec, o_min, o_max = _time_repeats(ol, max(100, iters // 4), 7, torch)
                    torch.cuda.synchronize()
                    row["one_launch"] = {"plan": one.describe(), "latency_us": o_sec * 1e6, "latency_us_min": o_min * 1e6,
                                         "latency_us_max": o_max * 1e6, "status": B.tdc_plan_status(one.plan)}
                    one.close()
            launch()                              # ys[i] holds the Tucker layer's output again
        per_layer.append(row)
    import ctypes
    null_fn, null_stream = B.load().tdc_launch_null, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for _ in range(100):                          # the first launch of a kernel loads its code: ~13 ms, not a launch cost
        null_fn(null_stream)
    torch.cuda.synchronize()
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
    traffic = measured_traffic(Ld.name(), args.layout, pd["plan"])
    roof["traffic"] = None if traffic is None else (traffic[0] + traffic[1]) * 1024.0      # bytes per layer call
    roof["traffic_fetch_write_kib"] = traffic
    roof["traffic_source"] = "profiles/traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE of this plan, an earlier run)" if traffic else None
    for row in per_layer:
        tr = measured_traffic(row["layer"], args.layout, row["plan"])
        row["traffic_bytes"] = None if tr is None else (tr[0] + tr[1]) * 1024.0
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
            5: "ResNet-50-style chain of 16 Tucker-2 3x3 layers, ranks round(0.3C) to 8, batch 1",
            6: "throughput set: 128->256 s2 56->28 r32/64 at batch 32 and 64, 128->128 28x28 r32 at batch 32, 128 and 256, "
               "256->256 14x14 r64 at batch 32, 128 and 256",
            7: "large-image layers of a VGG-16-shaped network, batch 1: 64->64 224x224 r64/32, 128->128 112x112 r64/32, 128->256 and "
               "256->256 56x56, 512->512 28x28 and 14x14 at a quarter of the channels"}[args.config]),
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
        # beside the latency-bound headline: layers whose batch fills the chip, against the same fp32 MFMA peak
        # (reported side figures; `value` and `roofline` above are the batch-1 sweep's): workload 6, whose first
        # two layers are the batch-32 layers of config 4, then a 14x14 layer at batch 32 and 128, then larger batches.

        def throughput(Lt, seed):
            inp = make_inputs(Lt, seed)
            t = {k: torch.from_numpy(v).to(dev) for k, v in inp.items()}
            ct = TuckerConv2d(Lt, 0, None, layout=layout)
            ct.pack(t["U_in"], t["core"], t["U_out"])
            xt = t["x"].permute(0, 2, 3, 1).contiguous() if layout == B.LAYOUT_NHWC else t["x"]
            yt = torch.empty(ct.out_shape(), device=dev, dtype=torch.float32)
            lt = ct.bind(xt, yt)
            for _ in range(100):
                lt()
            t_sec, t_min, t_max = _time_repeats(lt, 100, 5, torch)
            torch.cuda.synchronize()
            entry = {"layer": Lt.name(), "plan": ct.describe(), "latency_us": t_sec * 1e6, "latency_us_min": t_min * 1e6,
                     "latency_us_max": t_max * 1e6,
                     "roofline": {"bound": "mfma", "achieved": R.flops(Lt) / t_sec / 1e12, "peak": R.FP32_MFMA_PEAK / 1e12,
                                  "unit": "TFLOP/s", "frac": R.flops(Lt) / t_sec / R.FP32_MFMA_PEAK}}
            ct.close()
            # the same layer with several independent calls in flight: one plan, one set of buffers and one stream
            # (default priority) per call, launched round-robin.  The next call's workgroups then start as those of
            # the previous one finish and share compute units with them in different phases, which back-to-back
            # launches on one stream (each waits for the last workgroup of the one before) cannot offer.  Timed with
            # 2, 3 and 4 calls in flight, each on fresh streams (which hardware queue, 4 per process, a stream lands on
            # depends on the streams the process made before, and two streams on one queue serialise), and with plans
            # chosen for the whole chip (the default) and for half of it (tdc_select_tuning with half the compute
            # units: a call that shares the GPU is better off with fewer, larger workgroups).  The best of the six is
            # reported with its settings, all six are listed.
            n_cus = torch.cuda.get_device_properties(dev).multi_processor_count

            def in_flight(n_str, share):
                return _in_flight(torch, Lt, t, xt, yt, layout, n_cus, n_str, share)

            tried = {(n, sh): in_flight(n, sh) for sh in (1, 2) for n in (2, 3, 4)}
            k_best = min(tried, key=lambda k: tried[k][0][2])
            (pc, plan_best), c_sec = tried[k_best], tried[k_best][0][2]
            entry["concurrent"] = {"streams": k_best[0], "planned_for_chip_share": "1/%d" % k_best[1], "plan": plan_best,
                                   "us_per_call": c_sec * 1e6, "us_per_call_min": pc[0] * 1e6, "us_per_call_max": pc[-1] * 1e6,
                                   "us_per_call_by_streams_and_share": {"%d streams, 1/%d" % k: v[0][2] * 1e6 for k, v in tried.items()},
                                   "roofline": {"bound": "mfma", "achieved": R.flops(Lt) / c_sec / 1e12,
                                                "peak": R.FP32_MFMA_PEAK / 1e12, "unit": "TFLOP/s",
                                                "frac": R.flops(Lt) / c_sec / R.FP32_MFMA_PEAK}}
            return entry

        regime = [throughput(Lt, layer_seed(6, j)) for j, Lt in enumerate(config_layers(6))]
        out["throughput_regime"] = regime[0]
        out["throughput_layers"] = regime
    if args.config == 2 and variant == 0 and not args.brief:
        # the paper's end-to-end setting in this library's terms: the 3 + 4 + 6 + 3 bottleneck blocks of a ResNet-50-shaped
        # network (dense 1x1s, Tucker-2 3x3s, projection shortcuts, epilogues fused), eagerly and as ONE HIP graph
        from paper_2211_03715_amd.bottleneck import TuckerResNetBody, time_network
        chains = []
        for lay_name, lay in (("nchw", B.LAYOUT_NCHW), ("nhwc", B.LAYOUT_NHWC)):
            net = TuckerResNetBody(1, layout=lay)
            entry = {"network": "ResNet-50 residual stages (16 bottleneck blocks), 64x56x56 in, 2048x7x7 out, batch 1",
                     "layout": lay_name, "kernels": net.kernels(), "gflop": net.flops() / 1e9}
            entry.update(time_network(net))
            entry["graph_gflops"] = net.flops() / entry["graph_us"] / 1e3
            chains.append(entry)
            net.close()
        out["resnet50_body"] = chains
        # and the ResNet-18-shaped one: 8 basic blocks whose 16 3x3 convolutions are all Tucker-2 layers (the shapes of
        # this sweep and their stride-2 neighbours, chained with shortcuts and epilogues)
        from paper_2211_03715_amd.bottleneck import TuckerResNet18Body
        chains18 = []
        for lay_name, lay in (("nchw", B.LAYOUT_NCHW), ("nhwc", B.LAYOUT_NHWC)):
            net = TuckerResNet18Body(1, layout=lay)
            entry = {"network": "ResNet-18 residual stages (8 basic blocks, 16 Tucker-2 3x3 layers), 64x56x56 in, 512x7x7 out, batch 1",
                     "layout": lay_name, "kernels": net.kernels(), "gflop": net.flops() / 1e9}
            entry.update(time_network(net))
            entry["graph_gflops"] = net.flops() / entry["graph_us"] / 1e3
            chains18.append(entry)
            net.close()
        out["resnet18_body"] = chains18
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

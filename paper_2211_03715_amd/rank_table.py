"""Latency table T over Tucker ranks, measured on the GPU, and the rank selection that reads it.

The paper's co-design step (section 6) runs every candidate decomposition (D1, D2) of a layer, in
steps of 32 channels, records its latency in a table T, measures the original convolution too, and
then picks ranks under a FLOPs budget with a threshold theta against the original layer.  This
module is that workflow on this library: tdc_conv_tucker2 for the candidates, tdc_conv_dense for
the original layer, tdc_select_ranks for the choice.  Latencies are queued latencies (events around
back-to-back launches on one stream), the same figure bench.py reports per layer.

    python -m paper_2211_03715_amd.rank_table --config 2 --step 32 --budget 0.6
    python -m paper_2211_03715_amd.rank_table --staircase
"""
from __future__ import annotations

import argparse
import json
import sys
from dataclasses import replace
from typing import Dict, List, Sequence, Tuple

from . import binding as B
from .layer import DenseConv2d, TuckerConv2d
from .workloads import Layer, config_layers, make_dense_inputs, make_inputs


def _queued_us(launch, iters: int, warmup: int = 20) -> float:
    import torch
    for _ in range(warmup):
        launch()
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    start.record()
    for _ in range(iters):
        launch()
    stop.record()
    stop.synchronize()
    return start.elapsed_time(stop) * 1e3 / iters


def measure_tucker(layer: Layer, iters: int = 300, device: int = 0, seed: int = 1) -> Tuple[float, str]:
    """Queued latency (us) of the Tucker-2 layer with the selector's tuning, and the plan's description."""
    import torch
    dev = torch.device("cuda", device)
    t = {k: torch.from_numpy(v).to(dev) for k, v in make_inputs(layer, seed).items()}
    conv = TuckerConv2d(layer, device)
    try:
        conv.pack(t["U_in"], t["core"], t["U_out"])
        y = torch.empty((layer.batch, layer.N, conv.Ho, conv.Wo), device=dev, dtype=torch.float32)
        us = _queued_us(conv.bind(t["x"], y), iters)
        torch.cuda.synchronize()
        return us, conv.describe()
    finally:
        conv.close()


def measure_dense(layer: Layer, iters: int = 300, device: int = 0, seed: int = 1) -> Tuple[float, str]:
    """Queued latency (us) of the undecomposed layer on the library's dense kernel."""
    import torch
    dev = torch.device("cuda", device)
    t = {k: torch.from_numpy(v).to(dev) for k, v in make_dense_inputs(layer, seed).items()}
    conv = DenseConv2d(layer, device)
    try:
        conv.pack(t["W"])
        y = torch.empty((layer.batch, layer.N, conv.Ho, conv.Wo), device=dev, dtype=torch.float32)
        us = _queued_us(conv.bind(t["x"], y), iters)
        torch.cuda.synchronize()
        return us, conv.describe()
    finally:
        conv.close()


def candidate_ranks(channels: int, step: int) -> List[int]:
    """step, 2*step, ... up to the channel count (the paper reduces 32 channels at a time)."""
    return list(range(step, channels + 1, step))


def latency_table(layer: Layer, step: int = 32, iters: int = 300, device: int = 0,
                  progress=None) -> List[Tuple[int, int, float]]:
    """T for one layer: (R1, R2, us) for R1 in steps up to C and R2 in steps up to N."""
    table = []
    for r1 in candidate_ranks(layer.C, step):
        for r2 in candidate_ranks(layer.N, step):
            us, desc = measure_tucker(replace(layer, R1=r1, R2=r2), iters, device)
            table.append((r1, r2, us))
            if progress:
                progress("T[%s](%d,%d) = %.2f us  %s" % (layer.name(), r1, r2, us, desc))
    return table


def select(layers: Sequence[Layer], tables, dense_us: Sequence[float], budget: float, theta: float = 0.15,
           tie_tol: float = 0.02) -> List[Dict]:
    """tdc_select_ranks on measured tables."""
    return B.tdc_select_ranks(list(layers), tables, list(dense_us), budget, theta, tie_tol)


def staircase(C: int, HW: int, Ns: Sequence[int], iters: int = 300, device: int = 0) -> List[Tuple[int, float]]:
    """Latency of a 3x3 convolution with C input channels on an HW x HW image as its output channels
    grow: the experiment behind the paper's staircase figure (section 6), on the dense kernel."""
    return [(n, measure_dense(Layer(1, C, n, HW, HW, 1, 1), iters, device)[0]) for n in Ns]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=2, help="workload whose layer shapes are tabulated (ranks are swept)")
    ap.add_argument("--step", type=int, default=32)
    ap.add_argument("--iters", type=int, default=300)
    ap.add_argument("--budget", type=float, nargs="*", default=[0.4, 0.6, 0.8], help="FLOPs reduction targets to select for")
    ap.add_argument("--theta", type=float, default=0.15)
    ap.add_argument("--tie-tol", type=float, default=0.02)
    ap.add_argument("--staircase", action="store_true", help="only the output-channel staircase of the dense kernel")
    ap.add_argument("--out", default=None, help="write everything as JSON to this file")
    args = ap.parse_args(argv)

    import torch
    if not torch.cuda.is_available():
        sys.exit("rank_table needs a GPU")
    B.load()
    say = lambda s: print(s, flush=True)
    result: Dict = {"step": args.step, "theta": args.theta, "tie_tol": args.tie_tol}
    if args.staircase:
        Ns = list(range(32, 257, 16))
        result["staircase"] = {}
        for hw in (28, 14):
            rows = staircase(64, hw, Ns, args.iters)
            result["staircase"]["C64_%dx%d" % (hw, hw)] = rows
            say("dense 3x3, C=64, %dx%d:  " % (hw, hw) + "  ".join("N=%d %.2fus" % r for r in rows))
    else:
        seen, layers = set(), []
        for L in config_layers(args.config):            # distinct geometries only
            key = (L.batch, L.C, L.N, L.H, L.W, L.K, L.stride, L.pad)
            if key not in seen:
                seen.add(key)
                layers.append(L)
        tables, dense_us = [], []
        for L in layers:
            t2, desc = measure_dense(L, args.iters)
            say("original layer %s: %.2f us  %s" % (L.name(), t2, desc))
            dense_us.append(t2)
            tables.append(latency_table(L, args.step, args.iters, progress=say))
        result["layers"] = [L.asdict() for L in layers]
        result["tables"], result["dense_us"] = tables, dense_us
        result["selection"] = {}
        for b in args.budget:
            choice = select(layers, tables, dense_us, b, args.theta, args.tie_tol)
            result["selection"]["%g" % b] = choice
            kept = sum(c["macs"] for c in choice)
            total = sum(B.tdc_select_ranks([L], [[]], [1.0], 0.0)[0]["macs"] for L in layers)
            say("budget %.2f: " % b + "; ".join(
                ("%s -> (%d,%d) %.2fus" % (L.name(), c["R1"], c["R2"], c["latency_us"])) if c["decomposed"]
                else ("%s -> dense %.2fus" % (L.name(), c["latency_us"])) for L, c in zip(layers, choice))
                + "   MACs kept %.1f%%, latency %.2f us (all dense %.2f us)"
                % (100.0 * kept / total, sum(c["latency_us"] for c in choice), sum(dense_us)))
    if args.out:
        with open(args.out, "w") as f:
            json.dump(result, f)
    return 0


if __name__ == "__main__":
    sys.exit(main())

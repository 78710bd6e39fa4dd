"""Exhaustive autotuner, and the "model against exhaustive search" experiment.

The paper chooses its tile with an analytical model and reports how far that lands from an
exhaustive search over tilings (section 5.5, about 25% on its hardware).  This module is the
exhaustive side for this library: it times every launchable tuning of a layer on the GPU
(tdc_plan_create_tuned accepts or refuses each candidate, so only what the library itself deems
launchable runs) and compares the best with what the selector's closed-form model picks.

    python -m paper_2211_03715_amd.autotune --config 2            # table: model pick vs best found
    best = autotune(layer)["best"]["tuning"]                      # a tuning to pass to TuckerConv2d
    python -m paper_2211_03715_amd.autotune --analyse sweep.json  # no GPU: the paper's two-step tile rule on a saved sweep

Stage tunings of the SPLIT and MERGED variants are independent of one another (their kernels run
back to back), so those are searched one stage at a time around the selector's choice; that is
exhaustive for a sum of independent terms.
"""
from __future__ import annotations

import argparse
import itertools
import json
import sys
from typing import Dict, Iterable, List

from . import binding as B
from .layer import TuckerConv2d
from .workloads import Layer, config_layers, make_inputs

FUSED_MENU = [(1, 1, 1, 1), (1, 1, 2, 1), (2, 2, 2, 1), (2, 2, 4, 1), (4, 4, 4, 1),
              (1, 1, 1, 2), (1, 1, 2, 2), (2, 2, 2, 2), (2, 2, 4, 2), (4, 4, 4, 2)]   # (mb1, mb2, mb3, pb)
TILE_H = (1, 2, 4, 7, 8, 14, 16)
TILE_W = (4, 7, 8, 14, 16, 28, 32)
STAGE_WAVES = (1, 2, 3, 4, 6, 8)


def _tiles(L: Layer):
    return sorted({(min(th, L.Ho), min(tw, L.Wo)) for th in TILE_H for tw in TILE_W if min(th, L.Ho) * min(tw, L.Wo) <= 512})


def candidates(L: Layer, variants: Iterable[str] = ("fused", "chain", "split", "merged", "fused_merged")) -> List[Dict]:
    """Keyword sets for binding.make_tuning; the library refuses those that do not fit the layer."""
    out: List[Dict] = []
    if "fused" in variants:
        for (th, tw), nw, m in itertools.product(_tiles(L), (2, 4, 8), FUSED_MENU):
            out.append(dict(variant=B.VARIANT_FUSED, tile_h=th, tile_w=tw, waves=(nw,) * 3, mb=m[:3], pb=(m[3],) * 3))
    if "chain" in variants:
        for (th, tw), nw, mb1, pb in itertools.product(_tiles(L), (1, 2, 4, 8), (1, 2, 4), (1, 2)):
            out.append(dict(variant=B.VARIANT_CHAIN, tile_h=th, tile_w=tw, waves=(nw,) * 3, mb=(mb1, 1, 1), pb=(pb,) * 3))
    if "fused_merged" in variants:
        small = sorted({(min(th, L.Ho), min(tw, L.Wo)) for th in (1, 2, 3, 4) for tw in (4, 7, 8, 14, 16, 28, 32)
                        if min(th, L.Ho) * min(tw, L.Wo) <= 64})
        for (th, tw), nbg, mb1 in itertools.product(small, (1, 2, 4, 8), (1, 2, 4)):
            for nw in range(nbg, 9, nbg):
                out.append(dict(variant=B.VARIANT_FUSED_MERGED, tile_h=th, tile_w=tw, waves=(nw, 0, 0), mb=(mb1, nbg, 0)))
    for name, var, stages in (("split", B.VARIANT_SPLIT, 3), ("merged", B.VARIANT_MERGED, 2)):
        if name not in variants:
            continue
        try:
            base = B.tdc_select_tuning(B.make_shape(**L.asdict()), tuning=B.make_tuning(variant=var))
        except B.TdcError:
            continue
        b = dict(waves=list(base.waves), mb=list(base.mb), pb=list(base.pb))
        out.append(dict(variant=var, waves=tuple(b["waves"]), mb=tuple(b["mb"]), pb=tuple(b["pb"])))
        for st in range(stages):
            for mb, pb, nw in itertools.product((1, 2, 4), (1, 2, 4), STAGE_WAVES):
                c = {k: list(v) for k, v in b.items()}
                c["mb"][st], c["pb"][st], c["waves"][st] = mb, pb, nw
                if name == "merged" and st == 1:
                    c["mb"][2], c["pb"][2], c["waves"][2] = mb, pb, nw
                out.append(dict(variant=var, waves=tuple(c["waves"]), mb=tuple(c["mb"]), pb=tuple(c["pb"])))
    return out


def _time(launch, iters: int) -> float:
    import torch
    for _ in range(10):
        launch()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(iters):
        launch()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) * 1e3 / iters


def autotune(L: Layer, device: int = 0, iters: int = 200, variants=("fused", "chain", "split", "merged", "fused_merged"),
             seed: int = 1, progress=None, layout: int = B.LAYOUT_NCHW) -> Dict:
    """Times the selector's pick and every candidate.  Returns {"auto": row, "best": row, "by_variant":
    {name: best row}, "rows": all rows sorted by latency}; a row is {us, plan, tuning}."""
    import torch
    dev = torch.device("cuda", device)
    t = {k: torch.from_numpy(v).to(dev) for k, v in make_inputs(L, seed).items()}
    if layout == B.LAYOUT_NHWC:
        t["x"] = t["x"].permute(0, 2, 3, 1).contiguous()
    y = torch.empty(L.batch * L.N * L.Ho * L.Wo, device=dev, dtype=torch.float32)

    def run(tuning):
        conv = TuckerConv2d(L, device, tuning, layout=layout)
        try:
            conv.pack(t["U_in"], t["core"], t["U_out"])
            us = _time(conv.bind(t["x"], y), iters)
            torch.cuda.synchronize()
            return {"us": us, "plan": conv.describe(), "tuning": conv.tuning()}
        finally:
            conv.close()

    auto = run(None)
    rows, seen = [], set()
    for c in candidates(L, variants):
        key = json.dumps(c, sort_keys=True)
        if key in seen:
            continue
        seen.add(key)
        try:
            rows.append(run(B.make_tuning(**c)))
        except B.TdcError as e:
            if e.status != B.TDC_ERR_BAD_TUNING:
                raise
    rows.sort(key=lambda r: r["us"])
    by_variant: Dict[str, Dict] = {}
    for r in rows:
        by_variant.setdefault(r["tuning"]["variant"], r)
    # SPLIT, MERGED: the candidates vary one stage at a time around the selector's tuning; put the best
    # setting of every stage together and time that too
    keys = ("waves", "mb", "pb")
    for name, var, stages in (("split", B.VARIANT_SPLIT, 3), ("merged", B.VARIANT_MERGED, 2)):
        mine = [r for r in rows if r["tuning"]["variant"] == name]
        if not mine:
            continue
        base = B.tdc_select_tuning(B.make_shape(**L.asdict()), tuning=B.make_tuning(variant=var)).as_dict()
        combo = {k: list(base[k]) for k in keys}
        for st in range(stages):
            around = [r for r in mine if all(r["tuning"][k][o] == base[k][o] for k in keys for o in range(stages) if o != st)]
            if around:
                best = min(around, key=lambda r: r["us"])
                for k in keys:
                    combo[k][st] = best["tuning"][k][st]
        if name == "merged":
            for k in keys:
                combo[k][2] = combo[k][1]
        try:
            r = run(B.make_tuning(variant=var, waves=tuple(combo["waves"]), mb=tuple(combo["mb"]), pb=tuple(combo["pb"])))
        except B.TdcError:
            continue
        rows.append(r)
        if r["us"] < by_variant[name]["us"]:
            by_variant[name] = r
    rows.sort(key=lambda r: r["us"])
    if progress:
        progress("%s: auto %.2f us [%s]; best %.2f us [%s]; %d tunings timed" % (
            L.name(), auto["us"], auto["plan"], rows[0]["us"], rows[0]["plan"], len(rows)))
    return {"layer": L.name(), "auto": auto, "best": rows[0], "by_variant": by_variant, "rows": rows}


def paper_tile_rule(L: Layer, rows: List[Dict], cus: int = 256, top: float = 0.05) -> Dict:
    """The paper's tile selection (sections 5.3-5.5) applied to the FUSED kernel's tilings of one layer.

    Step 1, computation latency: waves of thread blocks over the chip times the latency of one block,
    the block's FLOPs (halo positions included, as the paper counts them) over its share of the peak.
    Here a block is a workgroup, the chip holds `cus` x resident of them at once, and a workgroup of
    nw wavefronts can use min(nw, 4) / 4 of its CU's MFMA rate.  Step 2, data movement: among the
    tilings within the best `top` fraction of step 1, the one that moves the fewest global bytes
    (input tile with halo and all weights once per workgroup, the output once).
    `rows` are timed FUSED tunings ({us, tuning, plan}); returns the row the rule selects."""
    fused = [r for r in rows if r["tuning"]["variant"] == "fused"]
    if not fused:
        return {}
    scored = []
    for r in fused:
        t = r["tuning"]
        th, tw, nw = t["tile_h"], t["tile_w"], t["waves"][0]
        qh, qw = (th - 1) * L.stride + L.K, (tw - 1) * L.stride + L.K
        wgs = -(-L.Ho // th) * -(-L.Wo // tw) * L.batch
        lds = int(r["plan"].split("lds=")[1].split("B")[0])
        resident = max(1, min(160 * 1024 // max(lds, 1), 32 // nw, 8))
        flops_blk = 2.0 * (qh * qw * L.C * L.R1 + th * tw * (L.K * L.K * L.R1 * L.R2 + L.R2 * L.N))
        blk_peak = 157.3e12 / cus * min(nw, 4) / 4.0 / resident
        comp = -(-wgs // (cus * resident)) * flops_blk / blk_peak
        volume = 4.0 * (wgs * (qh * qw * L.C + L.C * L.R1 + L.R1 * L.R2 * L.K * L.K + L.R2 * L.N) + L.batch * L.N * L.Ho * L.Wo)
        scored.append((comp, volume, r))
    scored.sort(key=lambda x: x[0])
    keep = scored[:max(1, int(round(top * len(scored))))]
    # tilings that tie with the last one kept belong to the same class
    keep += [x for x in scored[len(keep):] if x[0] <= keep[-1][0] * (1 + 1e-9)]
    return min(keep, key=lambda x: x[1])[2]


def analyse(path: str) -> int:
    """Offline: on a sweep saved with --out, compare the paper's two-step rule and this library's
    closed-form model as selectors of FUSED tilings, each against the best FUSED tuning timed."""
    with open(path) as f:
        results = json.load(f)
    layers = {L.name(): L for cfg in range(1, 6) for L in config_layers(cfg)}
    print("%-44s %9s %22s %22s" % ("layer (FUSED tunings only)", "best us", "paper's rule: us (gap)", "this model: us (gap)"))
    gaps_p, gaps_m = [], []
    for res in results:
        L = layers[res["layer"]]
        fused = [r for r in res["rows"] if r["tuning"]["variant"] == "fused"]
        if not fused:
            continue
        best = min(r["us"] for r in fused)
        rule = paper_tile_rule(L, res["rows"])
        mine = B.tdc_select_tuning(B.make_shape(**L.asdict()), tuning=B.make_tuning(variant=B.VARIANT_FUSED)).as_dict()
        same = [r for r in fused if all(r["tuning"][k] == mine[k] for k in ("tile_h", "tile_w", "mb", "pb")) and
                r["tuning"]["waves"][0] == mine["waves"][0]]
        gp = rule["us"] / best - 1.0
        gaps_p.append(gp)
        cell = "not in the sweep"
        if same:
            gm = same[0]["us"] / best - 1.0
            gaps_m.append(gm)
            cell = "%6.2f (%4.1f%%)" % (same[0]["us"], 100 * gm)
        print("%-44s %9.2f %15.2f (%4.1f%%) %22s" % (L.name(), best, rule["us"], 100 * gp, cell))
    print("paper's rule behind the best FUSED tuning: mean %.1f%%, max %.1f%%" % (100 * sum(gaps_p) / len(gaps_p), 100 * max(gaps_p)))
    if gaps_m:
        print("this library's model (on the %d layers whose pick was timed): mean %.1f%%, max %.1f%%" % (
            len(gaps_m), 100 * sum(gaps_m) / len(gaps_m), 100 * max(gaps_m)))
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, nargs="*", default=[2])
    ap.add_argument("--shapes", nargs="*", default=[], metavar="B,C,N,H,W,R1,R2[,K,stride,pad]",
                    help="layers of one's own instead of --config, e.g. 1,96,96,28,28,24,24")
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--variants", nargs="*", default=["fused", "chain", "split", "merged", "fused_merged"])
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"])
    ap.add_argument("--out", default=None, help="JSON with every timed tuning")
    ap.add_argument("--analyse", default=None, metavar="JSON", help="no GPU: the paper's two-step tile rule on a sweep saved with --out")
    args = ap.parse_args(argv)
    if args.analyse:
        B.load()
        return analyse(args.analyse)
    import torch
    if not torch.cuda.is_available():
        sys.exit("autotune needs a GPU")
    B.load()
    results = []
    print("%-46s %9s %9s %7s  %s" % ("layer", "model us", "best us", "gap", "best plan"), flush=True)
    groups = [[Layer(*[int(v) for v in spec.split(",")]) for spec in args.shapes]] if args.shapes else \
             [config_layers(cfg) for cfg in args.config]
    for layers in groups:
        seen = set()
        for L in layers:
            if L.name() in seen:
                continue
            seen.add(L.name())
            r = autotune(L, 0, args.iters if L.batch == 1 else max(50, args.iters // 4), tuple(args.variants),
                         layout=B.LAYOUT_NHWC if args.layout == "nhwc" else B.LAYOUT_NCHW)
            results.append(r)
            print("%-46s %9.2f %9.2f %6.1f%%  %s   (model chose: %s)" % (
                L.name(), r["auto"]["us"], r["best"]["us"], 100.0 * (r["auto"]["us"] / r["best"]["us"] - 1.0), r["best"]["plan"],
                r["auto"]["plan"]), flush=True)
    gaps = [r["auto"]["us"] / r["best"]["us"] - 1.0 for r in results]
    print("model pick behind the best tuning found: mean %.1f%%, max %.1f%% over %d layers" % (
        100.0 * sum(gaps) / len(gaps), 100.0 * max(gaps), len(gaps)), flush=True)
    if args.out:
        with open(args.out, "w") as f:
            json.dump(results, f)
    return 0


if __name__ == "__main__":
    sys.exit(main())

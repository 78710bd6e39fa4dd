"""Exhaustive autotuner, and the "model against exhaustive search" experiment.

The paper chooses its tile with an analytical model and reports how far that lands from an
exhaustive search over tilings (section 5.5, about 25% on its hardware).  This module is the
exhaustive side for this library: it times every launchable tuning of a layer on the GPU
(tdc_plan_create_tuned accepts or refuses each candidate, so only what the library itself deems
launchable runs) and compares the best with what the selector's closed-form model picks.

    python -m paper_2211_03715_amd.autotune --config 2            # table: model pick vs best found
    best = autotune(layer)["best"]["tuning"]                      # a tuning to pass to TuckerConv2d

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


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, nargs="*", default=[2])
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--variants", nargs="*", default=["fused", "chain", "split", "merged", "fused_merged"])
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"])
    ap.add_argument("--out", default=None, help="JSON with every timed tuning")
    args = ap.parse_args(argv)
    import torch
    if not torch.cuda.is_available():
        sys.exit("autotune needs a GPU")
    B.load()
    results = []
    print("%-46s %9s %9s %7s  %s" % ("layer", "model us", "best us", "gap", "best plan"), flush=True)
    for cfg in args.config:
        seen = set()
        for L in config_layers(cfg):
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

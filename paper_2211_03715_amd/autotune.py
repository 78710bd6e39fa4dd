"""Exhaustive autotuner, and the "model against exhaustive search" experiment.

The paper chooses its tile with an analytical model and reports how far that lands from an
exhaustive search over tilings (section 5.5, about 25% on its hardware).  This module is the
exhaustive side for this library: it times every launchable tuning of a layer on the GPU
(tdc_plan_create_tuned accepts or refuses each candidate, so only what the library itself deems
launchable runs) and compares the best with what the selector's closed-form model picks.

    python -m paper_2211_03715_amd.autotune --config 2            # table: model pick vs best found
    best = autotune(layer)["best"]["tuning"]                      # a tuning to pass to TuckerConv2d
    python -m paper_2211_03715_amd.autotune --analyse sweep.json  # no GPU: the paper's two-step tile rule on a saved sweep
    python -m paper_2211_03715_amd.autotune --fit a.json b.json   # no GPU: refit the selector's coefficients to saved sweeps

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
    # The selector's pick once more, now that clocks and caches are where they were for the candidates: the first
    # measurement of a process reads 5-10% high on the longer kernels, which would be booked as the model's error.
    first, auto = auto, run(None)
    auto["first_us"] = first["us"]
    if progress:
        progress("%s: auto %.2f us [%s]; best %.2f us [%s]; %d tunings timed" % (
            L.name(), auto["us"], auto["plan"], rows[0]["us"], rows[0]["plan"], len(rows)))
    return {"layer": L.name(), "layout": "nhwc" if layout == B.LAYOUT_NHWC else "nchw", "auto": auto, "best": rows[0],
            "by_variant": by_variant, "rows": rows}


EPILOGUES = {"none": (False, False, False), "bias": (True, False, False), "bias_relu": (True, False, True),
             "bias_residual_relu": (True, True, True)}


def autotune_dense(L: Layer, device: int = 0, iters: int = 200, epilogue: str = "bias_residual_relu", progress=None,
                   layout: int = B.LAYOUT_NCHW) -> Dict:
    """The dense K x K layer of L's shape (tdc_conv_dense; R1, R2 are ignored) with every register-tile / wavefront
    combination of its one GEMM launch, timed with the given epilogue.  Same result format as autotune()."""
    import torch
    from .layer import DenseConv2d
    dev = torch.device("cuda", device)
    bias, residual, relu = EPILOGUES[epilogue]
    x = torch.randn((L.batch, L.H, L.W, L.C) if layout == B.LAYOUT_NHWC else (L.batch, L.C, L.H, L.W), device=dev)
    W = torch.randn((L.C, L.N, L.K, L.K), device=dev) * float(L.C * L.K * L.K) ** -0.5

    def run(tuning):
        conv = DenseConv2d(L, device, tuning, layout=layout)
        try:
            conv.pack(W)
            y = torch.empty(conv.out_shape(), device=dev)
            us = _time(conv.bind(x, y, bias=torch.zeros(L.N, device=dev) if bias else None,
                                 residual=torch.zeros_like(y) if residual else None, relu=relu), iters)
            torch.cuda.synchronize()
            return {"us": us, "plan": conv.describe(), "tuning": conv.tuning()}
        finally:
            conv.close()

    auto = run(None)
    rows = []
    for mb, pb, nw in itertools.product((1, 2, 4), (1, 2, 4), STAGE_WAVES):
        try:
            rows.append(run(B.make_tuning(mb=(0, mb, 0), pb=(0, pb, 0), waves=(0, nw, 0))))
        except B.TdcError as e:
            if e.status != B.TDC_ERR_BAD_TUNING:
                raise
    rows.sort(key=lambda r: r["us"])
    first, auto = auto, run(None)
    auto["first_us"] = first["us"]
    if progress:
        progress("%s dense: auto %.2f us [%s]; best %.2f us [%s]; %d tunings timed" % (
            L.name(), auto["us"], auto["plan"], rows[0]["us"], rows[0]["plan"], len(rows)))
    return {"layer": L.name(), "layout": "nhwc" if layout == B.LAYOUT_NHWC else "nchw", "epilogue": epilogue, "auto": auto,
            "best": rows[0], "by_variant": {"dense": rows[0]}, "rows": rows}


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


COEF_HEADER = __import__("os").path.join(__import__("os").path.dirname(__import__("os").path.abspath(__file__)), "csrc", "tdc_select_coef.h")
COEF_TABLES = {"fused_latency": "kFusedLatencyCoef", "fused_throughput": "kFusedThroughputCoef", "chain": "kChainCoef",
               "fused_merged": "kFmCoef", "stage": "kStageCoef", "dense": "kDenseCoef"}
_VARIANT_IDS = {v: k for k, v in B.VARIANT_NAMES.items()}
_LAYER_RE = __import__("re").compile(r"b(\d+)_c(\d+)_n(\d+)_(\d+)x(\d+)_r(\d+)-(\d+)_k(\d+)_s(\d+)_p(\d+)$")


def _layer_from_name(name: str) -> Layer:
    m = _LAYER_RE.match(name)
    if not m:
        raise ValueError("not a layer name: %r" % name)
    return Layer(*[int(v) for v in m.groups()])


def _load_sweep(path: str) -> List[Dict]:
    """The per-layer results of a sweep file: the list --out writes, or that list under "results" beside a note."""
    with open(path) as f:
        d = json.load(f)
    return d["results"] if isinstance(d, dict) else d


def read_coefficients(path: str = COEF_HEADER) -> Dict[str, List[float]]:
    """The coefficient tables the library is built with, by model name."""
    import re
    text = open(path).read()
    out = {}
    for model, sym in COEF_TABLES.items():
        m = re.search(r"%s\[\d+\] = \{([^}]*)\}" % sym, text)
        out[model] = [float(v) for v in m.group(1).split(",")]
    return out


def sweep_rows(paths: Iterable[str], default_layout: str = "nchw") -> Dict[str, List[Dict]]:
    """Rows of saved sweeps (--out files) grouped by the coefficient table that prices them: each row gets the layer, the
    measured latency and the model's terms for its tuning (tdc_model_terms: the one copy of the model, in the library)."""
    by_model: Dict[str, List[Dict]] = {}
    for path in paths:
        for res in _load_sweep(path):
            L = _layer_from_name(res["layer"])
            layout = B.LAYOUT_NHWC if res.get("layout", default_layout) == "nhwc" else B.LAYOUT_NCHW
            shape = B.make_shape(**L.asdict(), layout=layout)
            for r in res["rows"]:
                t = r["tuning"]
                tuning = B.make_tuning(variant=_VARIANT_IDS[t["variant"]], tile_h=t["tile_h"], tile_w=t["tile_w"],
                                       waves=tuple(t["waves"]), mb=tuple(t["mb"]), pb=tuple(t["pb"]))
                try:
                    model, names, terms = B.tdc_model_terms(shape, tuning)
                except B.TdcError:
                    continue
                # CHAIN is only ever chosen where every CU gets two pixel blocks or more; its table is fitted there
                if model == "chain" and L.batch * L.Ho * L.Wo < 32 * 256:
                    continue
                by_model.setdefault(model, []).append({"layer": res["layer"], "layout": res.get("layout", default_layout),
                                                       "us": r["us"], "terms": terms, "names": names, "plan": r["plan"]})
    return by_model


def fit(paths: Iterable[str], default_layout: str = "nchw", models: Iterable[str] = (), near_best: float = 0.0) -> Dict[str, Dict]:
    """Non-negative least squares of the measured latencies against the model's terms, in relative error (each row
    weighted by 1 / latency) times (best latency of its layer / its latency) ** near_best: the model has to rank the
    fast tunings of a layer right, how wrong it is about the slow ones matters less.  Returns {model: {names, coef, rows, median_err, p90_err, regret: {(layer, layout): ...}}};
    regret = how far the tuning the fitted model ranks first lies behind the best one timed, per layer."""
    import numpy as np
    from scipy.optimize import nnls
    out = {}
    for model, rows in sweep_rows(paths, default_layout).items():
        if models and model not in models:
            continue
        X = np.array([r["terms"] for r in rows], dtype=float)
        y = np.array([r["us"] for r in rows], dtype=float)
        best_of: Dict = {}
        for r in rows:
            key = (r["layer"], r["layout"])
            best_of[key] = min(best_of.get(key, r["us"]), r["us"])
        w = np.array([(best_of[(r["layer"], r["layout"])] / r["us"]) ** near_best / r["us"] for r in rows])
        coef, _ = nnls(X * w[:, None], y * w)
        pred = X @ coef
        err = np.abs(pred - y) / y
        groups: Dict = {}
        for r, p in zip(rows, pred):
            groups.setdefault((r["layer"], r["layout"]), []).append((p, r["us"], r["plan"]))
        regret = {}
        for key, v in groups.items():
            best = min(x[1] for x in v)
            pick = min(v, key=lambda x: x[0])
            regret[key] = {"best_us": best, "pick_us": pick[1], "pick_plan": pick[2], "regret": pick[1] / best - 1.0, "n": len(v)}
        out[model] = {"names": rows[0]["names"], "coef": [float(c) for c in coef], "rows": len(rows),
                      "median_err": float(np.median(err)), "p90_err": float(np.percentile(err, 90)), "regret": regret}
    return out


def evaluate(paths: Iterable[str], coefficients: Dict[str, List[float]], default_layout: str = "nchw") -> Dict:
    """How a set of coefficient tables ranks the tunings of saved sweeps: per (layer, layout), the measured latency of
    the tuning with the lowest estimate over ALL models (what AUTO compares) against the best one timed."""
    import numpy as np
    groups: Dict = {}
    for model, rows in sweep_rows(paths, default_layout).items():
        if model not in coefficients:
            continue
        c = np.array(coefficients[model])
        for r in rows:
            groups.setdefault((r["layer"], r["layout"]), []).append((float(np.dot(c, r["terms"])), r["us"], r["plan"]))
    out = {}
    for key, v in groups.items():
        best = min(x[1] for x in v)
        pick = min(v, key=lambda x: x[0])
        out[key] = {"best_us": best, "pick_us": pick[1], "pick_plan": pick[2], "estimate_us": pick[0], "regret": pick[1] / best - 1.0, "n": len(v)}
    return out


def selector_gap(paths: Iterable[str], default_layout: str = "nchw") -> List[Dict]:
    """The library's own choice (tdc_select_tuning with everything left open, all its rules applied) looked up in saved
    sweeps: per (layer, layout) the latency timed for exactly that tuning against the best tuning timed.  A choice the
    sweep did not time (a tile outside its menu) is listed with gap None."""
    def key(t):
        return (t["variant"], t["tile_h"], t["tile_w"], tuple(t["waves"]), tuple(t["mb"]), tuple(t["pb"]))
    out = []
    for path in paths:
        for res in _load_sweep(path):
            L = _layer_from_name(res["layer"])
            lay = res.get("layout", default_layout)
            shape = B.make_shape(**L.asdict(), layout=B.LAYOUT_NHWC if lay == "nhwc" else B.LAYOUT_NCHW)
            dense = bool(res["rows"]) and res["rows"][0]["tuning"]["variant"] == "dense"     # a sweep made with --dense
            pick = B.tdc_select_tuning(shape, tuning=B.make_tuning(variant=B.VARIANT_DENSE) if dense else None).as_dict()
            same = [r for r in res["rows"] if key(r["tuning"]) == key(pick)]
            best = min(r["us"] for r in res["rows"])
            out.append({"layer": res["layer"], "layout": lay, "best_us": best, "pick": pick,
                        "pick_us": same[0]["us"] if same else None, "gap": same[0]["us"] / best - 1.0 if same else None})
    return out


def selector_gap_main(paths: List[str], default_layout: str) -> int:
    B.load()
    rows = selector_gap(paths, default_layout)
    print("%-46s %-5s %9s %9s %7s  %s" % ("layer", "", "best us", "chosen us", "gap", "chosen tuning"))
    for r in rows:
        t = r["pick"]
        what = "%s tile=%dx%d waves=%s mb=%s pb=%s" % (t["variant"], t["tile_h"], t["tile_w"], t["waves"], t["mb"], t["pb"])
        if r["gap"] is None:
            print("%-46s %-5s %9.2f %9s %7s  %s" % (r["layer"], r["layout"], r["best_us"], "-", "-", what + "  (not timed in the sweep)"))
        else:
            print("%-46s %-5s %9.2f %9.2f %6.1f%%  %s" % (r["layer"], r["layout"], r["best_us"], r["pick_us"], 100 * r["gap"], what))
    gaps = [r["gap"] for r in rows if r["gap"] is not None]
    if gaps:
        print("the selector's choice behind the best tuning timed: mean %.1f%%, max %.1f%% over %d layers (%d more not timed)" % (
            100 * sum(gaps) / len(gaps), 100 * max(gaps), len(gaps), len(rows) - len(gaps)))
    return 0


def write_coefficients(fitted: Dict[str, Dict], path: str = COEF_HEADER) -> None:
    """Replace the tables of the fitted models in the coefficient header; the other tables stay as they are."""
    import re
    text = open(path).read()
    for model, res in fitted.items():
        sym = COEF_TABLES[model]
        body = ", ".join("%.4f" % c if c else "0" for c in res["coef"])
        text, n = re.subn(r"(%s\[\d+\] = \{)[^}]*(\})" % sym, lambda m: m.group(1) + body + m.group(2), text)
        if n != 1:
            raise RuntimeError("table %s not found in %s" % (sym, path))
    with open(path, "w") as f:
        f.write(text)


def fit_main(paths: List[str], default_layout: str, models: List[str], write: bool, held_out: List[str] = (),
             near_best: float = 0.0) -> int:
    B.load()
    fitted = fit(paths, default_layout, models, near_best)
    current = read_coefficients()
    for model, res in fitted.items():
        print("model %s: %d tunings, median relative error %.1f%%, 90th percentile %.1f%%" % (
            model, res["rows"], 100 * res["median_err"], 100 * res["p90_err"]))
        print("  %-12s %10s %10s" % ("term", "fitted", "built with"))
        for n, c, old in zip(res["names"], res["coef"], current[model]):
            print("  %-12s %10.4f %10.4f" % (n, c, old))
        regs = [v["regret"] for v in res["regret"].values()]
        for (layer, layout), v in sorted(res["regret"].items()):
            print("  %-46s %-4s best %8.2f us  model's first %8.2f us (%4.1f%% behind) of %d" % (
                layer, layout, v["best_us"], v["pick_us"], 100 * v["regret"], v["n"]))
        print("  the model's first choice behind the best tuning timed: mean %.1f%%, max %.1f%% over %d layers" % (
            100 * sum(regs) / len(regs), 100 * max(regs), len(regs)))
        print("  static const double %s[%d] = {%s};" % (COEF_TABLES[model], len(res["coef"]),
                                                       ", ".join("%.4f" % c if c else "0" for c in res["coef"])))
    merged = dict(current)
    merged.update({m: r["coef"] for m, r in fitted.items()})
    cases = [("fitted sweeps", paths, "built-in tables", current), ("fitted sweeps", paths, "fitted tables", merged)]
    if held_out:
        cases += [("held-out sweeps", held_out, "built-in tables", current), ("held-out sweeps", held_out, "fitted tables", merged)]
    for which, files, label, table in cases:
        ev = evaluate(files, table, default_layout)
        regs = [v["regret"] for v in ev.values()]
        print("%s, across models, %s: lowest estimate behind the best tuning timed: mean %.1f%%, max %.1f%% over %d layers" % (
            which, label, 100 * sum(regs) / len(regs), 100 * max(regs), len(regs)))
        if label == "fitted tables":
            for (layer, layout), v in sorted(ev.items()):
                print("  %-46s %-4s best %8.2f  picked %8.2f (%4.1f%%)  %s" % (layer, layout, v["best_us"], v["pick_us"], 100 * v["regret"],
                                                                            v["pick_plan"].split(" model=")[0]))
    if write:
        write_coefficients(fitted)
        print("wrote %s -- rebuild the library (python -m paper_2211_03715_amd.build)" % COEF_HEADER)
    return 0


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, nargs="*", default=[2])
    ap.add_argument("--shapes", nargs="*", default=[], metavar="B,C,N,H,W,R1,R2[,K,stride,pad]",
                    help="layers of one's own instead of --config, e.g. 1,96,96,28,28,24,24")
    ap.add_argument("--iters", type=int, default=200)
    ap.add_argument("--variants", nargs="*", default=["fused", "chain", "split", "merged", "fused_merged"])
    ap.add_argument("--layout", default="nchw", choices=["nchw", "nhwc"])
    ap.add_argument("--dense", action="store_true", help="sweep the dense K x K layer of each shape (tdc_conv_dense; R1, R2 ignored) "
                    "instead of the Tucker layer: the data of the `dense` coefficient table")
    ap.add_argument("--epilogue", default="bias_residual_relu", choices=sorted(EPILOGUES), help="with --dense: what the timed calls carry")
    ap.add_argument("--out", default=None, help="JSON with every timed tuning")
    ap.add_argument("--analyse", default=None, metavar="JSON", help="no GPU: the paper's two-step tile rule on a sweep saved with --out")
    ap.add_argument("--fit", nargs="+", default=None, metavar="JSON",
                    help="no GPU: refit the selector's coefficients to sweeps saved with --out (the library supplies the "
                         "model's terms per tuning, tdc_model_terms) and print the tables of csrc/tdc_select_coef.h")
    ap.add_argument("--selector-gap", nargs="+", default=None, metavar="JSON",
                    help="no GPU: look the built library's own choice up in sweeps saved with --out and print how far it "
                         "lies behind the best tuning timed")
    ap.add_argument("--models", nargs="*", default=[], help="with --fit: only these coefficient tables "
                    "(fused_latency fused_throughput chain fused_merged stage)")
    ap.add_argument("--held-out", nargs="*", default=[], metavar="JSON", help="with --fit: sweeps the fit does not see, "
                    "ranked with the fitted tables as a check")
    ap.add_argument("--near-best", type=float, default=0.0, help="with --fit: exponent of (layer's best / row's latency) "
                    "in a row's weight; 0 weighs every tuning of a layer alike")
    ap.add_argument("--write-coef", action="store_true", help="with --fit: write the fitted tables into csrc/tdc_select_coef.h")
    args = ap.parse_args(argv)
    if args.selector_gap:
        return selector_gap_main(args.selector_gap, args.layout)
    if args.fit:
        return fit_main(args.fit, args.layout, args.models, args.write_coef, args.held_out, args.near_best)
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
            lay = B.LAYOUT_NHWC if args.layout == "nhwc" else B.LAYOUT_NCHW
            if args.dense:
                r = autotune_dense(L, 0, args.iters, args.epilogue, layout=lay)
            else:
                r = autotune(L, 0, args.iters if L.batch == 1 else max(50, args.iters // 4), tuple(args.variants), layout=lay)
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

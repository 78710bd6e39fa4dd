"""The selector's calibration tool on the CPU: the library exports the terms of its latency estimate per tuning
(tdc_model_terms), autotune.fit refits the coefficient tables to saved sweeps.  Runs on a small sample of a sweep timed
on MI355X (tests/golden/sweep_sample.json); no GPU, no kernels."""
import json
import os
import shutil

import numpy as np
import pytest

from paper_2211_03715_amd import autotune as A
from paper_2211_03715_amd import binding as B

SAMPLE = os.path.join(os.path.dirname(__file__), "golden", "sweep_sample.json")


@pytest.fixture(scope="module")
def lib():
    B.load()
    return B


def test_tables_match_the_terms_the_library_exports(lib):
    tables = A.read_coefficients()
    assert set(tables) == set(A.COEF_TABLES)
    rows = A.sweep_rows([SAMPLE])
    assert {"chain", "fused_throughput"} <= set(rows)
    for model, rs in rows.items():
        for r in rs:
            assert len(r["terms"]) == len(r["names"]) == len(tables[model])
            assert all(t >= 0.0 for t in r["terms"])
            assert r["terms"][0] >= 1.0          # every model starts with its launches


def test_estimate_is_the_dot_product_the_selector_ranks_by(lib):
    """A tuning the selector prefers has the lower dot product: force two CHAIN tunings of one layer and compare the
    selector's choice between them with the estimates rebuilt from the exported terms and the tracked tables.  (A layer
    below 64 output pixels per compute unit in NCHW: above that the selector widens the stage-1 unit after ranking.)"""
    tables = A.read_coefficients()
    shape = B.make_shape(batch=16, C=128, N=128, H=28, W=28, R1=32, R2=32, K=3, stride=1, pad=1)
    pick = B.tdc_select_tuning(shape, tuning=B.make_tuning(variant=B.VARIANT_CHAIN))
    model, names, terms = B.tdc_model_terms(shape, pick)
    assert model == "chain"
    est_pick = float(np.dot(tables[model], terms))
    d = pick.as_dict()
    for mb1 in (1, 2):
        for pb in (1, 2):
            other = B.make_tuning(variant=B.VARIANT_CHAIN, tile_h=d["tile_h"], tile_w=d["tile_w"], waves=tuple(d["waves"]),
                                  mb=(mb1, 1, 1), pb=(pb, pb, pb))
            try:
                _, _, t2 = B.tdc_model_terms(shape, other)
            except B.TdcError:
                continue
            assert est_pick <= float(np.dot(tables[model], t2)) + 1e-9


def test_fit_recovers_latencies_made_from_known_coefficients(lib, tmp_path):
    """Latencies synthesised as (tracked table) . terms are fitted back to zero error and zero regret."""
    tables = A.read_coefficients()
    with open(SAMPLE) as f:
        sample = json.load(f)
    for res in sample["results"]:
        L = A._layer_from_name(res["layer"])
        shape = B.make_shape(**L.asdict(), layout=B.LAYOUT_NHWC if res["layout"] == "nhwc" else B.LAYOUT_NCHW)
        keep = []
        for r in res["rows"]:
            t = r["tuning"]
            tuning = B.make_tuning(variant=A._VARIANT_IDS[t["variant"]], tile_h=t["tile_h"], tile_w=t["tile_w"],
                                   waves=tuple(t["waves"]), mb=tuple(t["mb"]), pb=tuple(t["pb"]))
            try:
                model, _, terms = B.tdc_model_terms(shape, tuning)
            except B.TdcError:
                continue
            r["us"] = float(np.dot(tables[model], terms))
            keep.append(r)
        res["rows"] = keep
    path = tmp_path / "synthetic.json"
    path.write_text(json.dumps(sample))
    fitted = A.fit([str(path)])
    assert fitted
    for model, res in fitted.items():
        assert res["median_err"] < 1e-6 and res["p90_err"] < 1e-5, model
        assert max(v["regret"] for v in res["regret"].values()) < 1e-9


def test_fit_on_the_measured_sample(lib):
    fitted = A.fit([SAMPLE], models=("chain", "fused_throughput"))
    for model in ("chain", "fused_throughput"):
        res = fitted[model]
        assert all(c >= 0.0 for c in res["coef"])
        assert res["median_err"] < 0.15, (model, res["median_err"])
        assert max(v["regret"] for v in res["regret"].values()) < 0.15
    ev = A.evaluate([SAMPLE], A.read_coefficients())
    assert len(ev) == 4 and all(v["regret"] < 0.25 for v in ev.values())


def test_selector_choice_looked_up_in_the_sample(lib):
    rows = A.selector_gap([SAMPLE])
    assert len(rows) == 4
    for r in rows:
        assert r["gap"] is None or 0.0 <= r["gap"] < 0.25


def test_coefficient_header_round_trip(lib, tmp_path):
    copy = tmp_path / "coef.h"
    shutil.copy(A.COEF_HEADER, copy)
    before = A.read_coefficients(str(copy))
    fake = {"chain": {"coef": [0.5 * i for i in range(len(before["chain"]))]}}
    A.write_coefficients(fake, str(copy))
    after = A.read_coefficients(str(copy))
    assert after["chain"] == pytest.approx(fake["chain"]["coef"])
    assert after["stage"] == before["stage"] and after["fused_latency"] == before["fused_latency"]


def test_model_terms_error_paths(lib):
    import ctypes
    raw = B.load()
    shape = B.make_shape(batch=32, C=128, N=128, H=28, W=28, R1=32, R2=32, K=3, stride=1, pad=1)
    pick = B.tdc_select_tuning(shape)
    terms = (ctypes.c_double * 64)()
    names = (ctypes.c_char_p * 64)()
    n, model = ctypes.c_int(0), ctypes.c_char_p()
    ok = raw.tdc_model_terms(ctypes.byref(shape), ctypes.byref(pick), 256, 160 * 1024, terms, names, 64, ctypes.byref(n), ctypes.byref(model))
    assert ok == B.TDC_OK and n.value > 0 and model.value in (b"chain", b"fused_throughput")
    assert [names[i] for i in range(n.value)][0] == b"launch"
    # names and model are optional
    assert raw.tdc_model_terms(ctypes.byref(shape), ctypes.byref(pick), 256, 160 * 1024, terms, None, 64, ctypes.byref(n), None) == B.TDC_OK
    # too few slots, missing pointers, a tuning that names no kernel, a device that cannot exist
    assert raw.tdc_model_terms(ctypes.byref(shape), ctypes.byref(pick), 256, 160 * 1024, terms, names, 3, ctypes.byref(n), None) == B.TDC_ERR_BAD_SHAPE
    assert raw.tdc_model_terms(None, ctypes.byref(pick), 256, 160 * 1024, terms, names, 64, ctypes.byref(n), None) == B.TDC_ERR_NULL
    assert raw.tdc_model_terms(ctypes.byref(shape), ctypes.byref(pick), 256, 160 * 1024, None, names, 64, ctypes.byref(n), None) == B.TDC_ERR_NULL
    auto = B.make_tuning(variant=B.VARIANT_AUTO)
    assert raw.tdc_model_terms(ctypes.byref(shape), ctypes.byref(auto), 256, 160 * 1024, terms, names, 64, ctypes.byref(n), None) == B.TDC_ERR_BAD_TUNING
    assert raw.tdc_model_terms(ctypes.byref(shape), ctypes.byref(pick), 0, 160 * 1024, terms, names, 64, ctypes.byref(n), None) == B.TDC_ERR_BAD_TUNING
    # a tile the LDS cannot hold is refused like in tdc_plan_create
    big = B.make_tuning(variant=B.VARIANT_CHAIN, tile_h=16, tile_w=32, waves=(8, 8, 8), mb=(1, 1, 1), pb=(1, 1, 1))
    wide = B.make_shape(batch=1, C=512, N=512, H=64, W=64, R1=256, R2=128, K=3, stride=1, pad=1)
    assert raw.tdc_model_terms(ctypes.byref(wide), ctypes.byref(big), 256, 64 * 1024, terms, names, 64, ctypes.byref(n), None) == B.TDC_ERR_BAD_TUNING


def test_dense_layer_has_its_own_table_with_output_terms():
    """The dense layer is priced by the `dense` table: the eight terms of a GEMM stage and the outputs a thread owns,
    booked under the layout the launch writes."""
    coef = A.read_coefficients()
    assert len(coef["dense"]) == 10 and len(coef["stage"]) == 8
    for layout, live, dead in ((B.LAYOUT_NCHW, "y_nchw", "y_nhwc"), (B.LAYOUT_NHWC, "y_nhwc", "y_nchw")):
        shape = B.make_shape(1, 64, 256, 56, 56, 1, 1, 1, 1, 0, layout)
        for mb, pb, nw, want in ((4, 1, 1, 16.0), (2, 1, 4, 2.0), (1, 2, 8, 1.0)):
            t = B.make_tuning(variant=B.VARIANT_DENSE, waves=(nw,) * 3, mb=(mb,) * 3, pb=(pb,) * 3)
            model, names, terms = B.tdc_model_terms(shape, t)
            assert model == "dense" and names[:8] == ["launch", "wave", "kg", "mfma", "conv_b", "reduce", "act_1x1", "act_conv"]
            by = dict(zip(names, terms))
            assert by[live] == want and by[dead] == 0.0
        # the selector's own choice is the lowest estimate among the tunings it offers (no 3 or 6 wavefronts)
        pick = B.tdc_select_tuning(shape, tuning=B.make_tuning(variant=B.VARIANT_DENSE)).as_dict()
        est = {}
        for mb in (1, 2, 4):
            for pb in (1, 2, 4):
                for nw in (1, 2, 4):          # 64 input channels are 4 k-groups: no more wavefronts than that
                    t = B.make_tuning(variant=B.VARIANT_DENSE, waves=(nw,) * 3, mb=(mb,) * 3, pb=(pb,) * 3)
                    _, _, terms = B.tdc_model_terms(shape, t)
                    est[(mb, pb, nw)] = sum(c * f for c, f in zip(coef["dense"], terms))
        assert (pick["mb"][1], pick["pb"][1], pick["waves"][1]) == min(est, key=est.get)

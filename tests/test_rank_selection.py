"""Rank selection (paper section 6, Algorithm 1 step 1): the oracle against hand-worked cases and
against the rules themselves, planted mistakes in the oracle, and the library's tdc_select_ranks
against the oracle.  Host logic only: no GPU."""
import json
import os
import random

import pytest

from oracle import rank_oracle as RO
from paper_2211_03715_amd import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = json.load(open(os.path.join(HERE, "golden", "rank_selection_handworked.json")))


def _tables(g):
    return [[tuple(e) for e in tab] for tab in g["tables"]]


def _run_golden(select):
    for case in GOLDEN["cases"]:
        got = select(GOLDEN["layers"], _tables(GOLDEN), case["dense_latency"], case["budget"], case["theta"],
                     case["tie_tol"])
        assert len(got) == len(case["expect"])
        for g, e in zip(got, case["expect"]):
            assert (g["decomposed"], g["D1"], g["D2"]) == (e["decomposed"], e["D1"], e["D2"]), case["_why"]
            assert g["latency"] == e["latency"] and g["macs"] == e["macs"], case["_why"]


def test_macs_of_the_golden_fixture_follow_the_complexity_formula():
    """Section 3: P = HWC*D1 + H'W'K^2*D1*D2 + H'W'N*D2, F = H'W'K^2*C*N -- the fixture's hand-computed counts."""
    A, Bl = GOLDEN["layers"]
    m = GOLDEN["_macs"]
    assert RO.dense_macs(A) == m["F_A"] and RO.dense_macs(Bl) == m["F_B"]
    for key, want in m["P_A"].items():
        d1, d2 = map(int, key.split(","))
        assert RO.tucker_macs(A, d1, d2) == want
    for key, want in m["P_B"].items():
        d1, d2 = map(int, key.split(","))
        assert RO.tucker_macs(Bl, d1, d2) == want
    # stride 2, no padding, batch 3, non-square image, worked by hand: H'=3, W'=4
    L = {"batch": 3, "C": 5, "N": 7, "H": 8, "W": 10, "K": 3, "stride": 2, "pad": 0}
    assert RO.dense_macs(L) == 3 * 12 * 9 * 5 * 7
    assert RO.tucker_macs(L, 2, 4) == 3 * (80 * 5 * 2 + 12 * 9 * 2 * 4 + 12 * 7 * 4)


def test_oracle_reproduces_the_handworked_cases():
    _run_golden(RO.select_ranks)


def _random_instance(rng, n_layers):
    layers, tables, dense = [], [], []
    for _ in range(n_layers):
        C, N = rng.choice([32, 64, 96, 128]), rng.choice([32, 64, 96, 128])
        H = rng.choice([4, 7, 8, 14])
        stride = rng.choice([1, 1, 2])
        layers.append({"batch": rng.choice([1, 2]), "C": C, "N": N, "H": H, "W": H + rng.choice([0, 1]), "K": 3,
                       "stride": stride, "pad": 1})
        step = rng.choice([8, 16, 32])
        tab = []
        for d1 in range(step, C + 1, step):
            for d2 in range(step, N + 1, step):
                # staircase-like latencies: few distinct values so that ties and near-ties occur
                tab.append((d1, d2, round(3.0 + 0.5 * ((d1 * d2) // 2048) + rng.choice([0.0, 0.0, 0.01, 0.05]), 4)))
        rng.shuffle(tab)
        tables.append(tab)
        dense.append(round(rng.uniform(3.0, 9.0), 3))
    return layers, tables, dense


def _check_against_the_rules(layers, tables, dense, budget, theta, tol, result):
    """A verifier written from the rules, not a second selector: replays the budget bookkeeping with
    the reported choices and checks each choice's defining properties."""
    F = [RO.dense_macs(l) for l in layers]
    need, removed = budget * sum(F), 0.0
    for l, (layer, res) in enumerate(zip(layers, result)):
        b = max(0.0, (need - removed) / sum(F[l:]))
        cap = (1.0 - b) * F[l]
        adm = [c for c in tables[l] if RO.tucker_macs(layer, c[0], c[1]) <= cap]
        if res["decomposed"]:
            c = (res["D1"], res["D2"], res["latency"])
            assert c in adm                                               # within the budget, from the table
            t_min = min(t for _, _, t in adm)
            assert c[2] <= (1.0 + tol) * t_min                            # minimal latency
            for o in adm:                                                 # largest ranks among the minimal
                if o[2] <= (1.0 + tol) * t_min:
                    assert (o[0] * o[1], o[0] + o[1], o[0]) <= (c[0] * c[1], c[0] + c[1], c[0])
            assert c[2] < (1.0 - theta) * dense[l]                        # beats the original layer by theta
            assert res["macs"] == RO.tucker_macs(layer, c[0], c[1])
            removed += F[l] - res["macs"]
        else:
            assert res["D1"] == 0 and res["D2"] == 0 and res["latency"] == dense[l] and res["macs"] == F[l]
            if adm:                                                       # only the threshold can have refused it
                t_min = min(t for _, _, t in adm)
                best = max((o for o in adm if o[2] <= (1.0 + tol) * t_min), key=lambda o: (o[0] * o[1], o[0] + o[1], o[0]))
                assert best[2] >= (1.0 - theta) * dense[l]


def test_oracle_obeys_the_rules_on_random_tables():
    rng = random.Random(20221103)
    for trial in range(300):
        layers, tables, dense = _random_instance(rng, rng.randint(1, 6))
        budget, theta, tol = rng.choice([0.0, 0.1, 0.3, 0.5, 0.7]), rng.choice([0.0, 0.15, 0.3]), rng.choice([0.0, 0.02])
        res = RO.select_ranks(layers, tables, dense, budget, theta, tol)
        _check_against_the_rules(layers, tables, dense, budget, theta, tol, res)


def test_special_cases():
    layer = {"batch": 1, "C": 64, "N": 64, "H": 8, "W": 8, "K": 3, "stride": 1, "pad": 1}
    flat = [(d1, d2, 4.0) for d1 in (16, 32, 48, 64) for d2 in (16, 32, 48, 64)]
    # flat table, no threshold, no budget: every candidate ties, so the largest ranks win
    r = RO.select_ranks([layer], [flat], [10.0], 0.0, 0.0, 0.0)[0]
    # (64,64) costs more MACs than the dense layer and is out; (48,64) and (64,48) tie on product and
    # sum, and the larger D1 wins
    assert (r["D1"], r["D2"]) == (64, 48)
    # a strictly increasing table picks the smallest ranks
    inc = [(d1, d2, 1.0 + d1 * d2 * 1e-3) for d1 in (16, 32) for d2 in (16, 32)]
    r = RO.select_ranks([layer], [inc], [10.0], 0.0, 0.15, 0.0)[0]
    assert (r["D1"], r["D2"]) == (16, 16)
    # theta: equality refuses (t1 >= (1 - theta) t2)
    one = [(16, 16, 8.5)]
    assert not RO.select_ranks([layer], [one], [10.0], 0.0, 0.15, 0.0)[0]["decomposed"]
    assert RO.select_ranks([layer], [one], [10.0], 0.0, 0.14, 0.0)[0]["decomposed"]
    # an empty table leaves the layer dense
    assert not RO.select_ranks([layer], [[]], [10.0], 0.2, 0.15, 0.0)[0]["decomposed"]
    # a tighter budget never raises the MACs kept by a single layer
    tab = [(d1, d2, 5.0 - 0.001 * d1 - 0.0005 * d2) for d1 in range(8, 65, 8) for d2 in range(8, 65, 8)]
    kept = [RO.select_ranks([layer], [tab], [100.0], b, 0.15, 0.0)[0]["macs"] for b in (0.0, 0.2, 0.4, 0.6, 0.8)]
    assert all(a >= b for a, b in zip(kept, kept[1:]))


MUTATIONS = [
    ("need = budget * sum(F)", "need = budget * F[0]"),
    ("b = (need - removed) / remaining", "b = budget"),                                  # no carry-over
    ("cap = (1.0 - b) * F[l]", "cap = b * F[l]"),
    ("<= cap]", "<= cap or True]"),
    ("t_min = min(t for (_, _, t) in admissible)", "t_min = max(t for (_, _, t) in admissible)"),
    ("c[2] <= (1.0 + tie_tol) * t_min", "c[2] <= t_min"),                                 # tolerance ignored
    ("choice = max(minimal, key=", "choice = min(minimal, key="),
    ("(c[0] * c[1], c[0] + c[1], c[0])", "(c[0] + c[1], c[0] * c[1], c[0])"),
    ("(c[0] * c[1], c[0] + c[1], c[0])", "(c[0] * c[1], c[0] + c[1], c[1])"),
    (">= (1.0 - theta) * dense_latency[l]", "> (1.0 - theta) * dense_latency[l]"),
    (">= (1.0 - theta) * dense_latency[l]", ">= (1.0 + theta) * dense_latency[l]"),
    ("removed += F[l] - P", "removed += P"),
    ("layer[\"H\"] * layer[\"W\"] * layer[\"C\"] * D1", "Ho * Wo * layer[\"C\"] * D1"),   # stage 1 on output pixels
    ("+ Ho * Wo * layer[\"N\"] * D2))", "+ Ho * Wo * layer[\"N\"] * D1))"),
    ("layer[\"K\"] * layer[\"K\"] * D1 * D2", "layer[\"K\"] * D1 * D2"),
    ("return (n + 2 * pad - K) // stride + 1", "return (n + 2 * pad - K) // stride"),
]


def _all_pins(mod):
    """The pins above, run against a module object."""
    saved = {k: getattr(RO, k) for k in ("select_ranks", "tucker_macs", "dense_macs", "out_size")}
    try:
        for k in saved:
            setattr(RO, k, getattr(mod, k))
        test_macs_of_the_golden_fixture_follow_the_complexity_formula()
        test_oracle_reproduces_the_handworked_cases()
        test_special_cases()
        test_oracle_obeys_the_rules_on_random_tables()
    finally:
        for k, v in saved.items():
            setattr(RO, k, v)


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_planted_mistakes_in_the_oracle_are_caught(idx):
    import types
    old, new = MUTATIONS[idx]
    src = open(RO.__file__).read()
    assert src.count(old) >= 1, "mutation target vanished: %r" % old
    mod = types.ModuleType("rank_oracle_mutant")
    exec(compile(src.replace(old, new, 1), "rank_oracle_mutant", "exec"), mod.__dict__)
    with pytest.raises(AssertionError):
        _all_pins(mod)


# ---------------------------------------------------------------- the library against the oracle

def _lib_select(layers, tables, dense, budget, theta, tol):
    got = B.tdc_select_ranks(layers, tables, dense, budget, theta, tol)
    return [{"decomposed": g["decomposed"], "D1": g["R1"], "D2": g["R2"], "latency": g["latency_us"], "macs": g["macs"]}
            for g in got]


def test_library_reproduces_the_handworked_cases():
    _run_golden(_lib_select)


def test_library_equals_oracle_on_random_tables():
    rng = random.Random(7)
    for trial in range(400):
        layers, tables, dense = _random_instance(rng, rng.randint(1, 8))
        budget, theta, tol = rng.choice([0.0, 0.1, 0.3, 0.5, 0.7, 0.9]), rng.choice([0.0, 0.15, 0.3]), rng.choice([0.0, 0.02, 0.1])
        assert _lib_select(layers, tables, dense, budget, theta, tol) == RO.select_ranks(layers, tables, dense, budget, theta, tol)


def test_library_rejects_bad_arguments():
    import ctypes
    lib = B.load()
    layer = {"batch": 1, "C": 64, "N": 64, "H": 8, "W": 8, "K": 3, "stride": 1, "pad": 1}
    tab = [(16, 16, 3.0)]
    assert lib.tdc_select_ranks(None, 1, 0.5, 0.15, 0.0, None) == B.TDC_ERR_NULL
    for kw in (dict(budget=1.0), dict(budget=-0.1), dict(theta=1.0), dict(theta=-0.5), dict(tie_tol=-1.0)):
        args = dict(budget=0.5, theta=0.15, tie_tol=0.0)
        args.update(kw)
        with pytest.raises(B.TdcError):
            B.tdc_select_ranks([layer], [tab], [5.0], **args)
    with pytest.raises(B.TdcError):
        B.tdc_select_ranks([layer], [[(0, 16, 3.0)]], [5.0], 0.5)
    with pytest.raises(B.TdcError):
        B.tdc_select_ranks([layer], [tab], [0.0], 0.5)
    with pytest.raises(B.TdcError):
        B.tdc_select_ranks([dict(layer, H=1, pad=0)], [tab], [5.0], 0.5)
    assert ctypes.sizeof(B.tdc_rank_entry) == 16 and ctypes.sizeof(B.tdc_rank_choice) == 32

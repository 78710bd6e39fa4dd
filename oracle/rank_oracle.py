"""CPU oracle of the hardware-aware rank selection (paper section 6 and the first step of Algorithm 1).

TEST INFRASTRUCTURE ONLY: tests/ may import this; the product (libtdc.so's tdc_select_ranks) shares
no code with it.

What the paper fixes
  * every layer has a measured table T of latencies over candidate ranks (D1, D2) and the latency
    t2 of its original, undecomposed convolution;
  * under a FLOPs budget B (a target reduction ratio) only candidates with P(D1, D2) within the
    budget are admissible, P being the complexity of the Tucker layer (section 3):
        P = H*W*C*D1 + H'*W'*K*K*D1*D2 + H'*W'*N*D2      against      F = H'*W'*K*K*C*N ;
  * among the admissible candidates take those of minimal latency, and among these the largest
    ranks (Algorithm 1: max{ argmin_{P <= B} T });
  * do not decompose the layer if the chosen latency t1 >= (1 - theta) * t2;
  * a layer left undecomposed hands its share of the reduction to the layers after it.

Readings where the paper leaves room (the product takes the same ones)
  R1  "P <= B" with B a ratio: layer l may keep at most (1 - b_l) * F_l, where
      b_l = (B * sum_k F_k - reduction achieved by layers before l) / sum_{k >= l} F_k, floored at 0.
      With b_l recomputed at every layer an undecomposed layer raises the ratio demanded of the
      rest (the paper's carry-over) and an over-achieving one lowers it.
  R2  measured latencies never tie exactly: candidates within a relative tolerance `tie_tol` of the
      minimum count as minimal (tie_tol = 0 is the paper's rule read literally).
  R3  "largest ranks" = largest D1*D2, then largest D1+D2, then largest D1.
  R4  batch multiplies P and F alike and is included; MACs are counted (a factor 2 cancels).
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple


def out_size(n: int, K: int, stride: int, pad: int) -> int:
    return (n + 2 * pad - K) // stride + 1


def dense_macs(layer: Dict) -> float:
    Ho = out_size(layer["H"], layer["K"], layer["stride"], layer["pad"])
    Wo = out_size(layer["W"], layer["K"], layer["stride"], layer["pad"])
    return float(layer["batch"] * Ho * Wo * layer["K"] * layer["K"] * layer["C"] * layer["N"])


def tucker_macs(layer: Dict, D1: int, D2: int) -> float:
    Ho = out_size(layer["H"], layer["K"], layer["stride"], layer["pad"])
    Wo = out_size(layer["W"], layer["K"], layer["stride"], layer["pad"])
    return float(layer["batch"] * (layer["H"] * layer["W"] * layer["C"] * D1
                                   + Ho * Wo * layer["K"] * layer["K"] * D1 * D2
                                   + Ho * Wo * layer["N"] * D2))


def select_ranks(layers: Sequence[Dict], tables: Sequence[Sequence[Tuple[int, int, float]]],
                 dense_latency: Sequence[float], budget: float, theta: float, tie_tol: float) -> List[Dict]:
    """One dict per layer: decomposed (bool), D1, D2 (0 when not decomposed), latency, macs."""
    F = [dense_macs(l) for l in layers]
    need = budget * sum(F)
    removed = 0.0
    out = []
    for l, layer in enumerate(layers):
        remaining = sum(F[l:])
        b = (need - removed) / remaining
        if b < 0.0:
            b = 0.0
        cap = (1.0 - b) * F[l]
        admissible = [(D1, D2, t) for (D1, D2, t) in tables[l] if tucker_macs(layer, D1, D2) <= cap]
        choice = None
        if admissible:
            t_min = min(t for (_, _, t) in admissible)
            minimal = [c for c in admissible if c[2] <= (1.0 + tie_tol) * t_min]
            choice = max(minimal, key=lambda c: (c[0] * c[1], c[0] + c[1], c[0]))
            if choice[2] >= (1.0 - theta) * dense_latency[l]:
                choice = None
        if choice is None:
            out.append({"decomposed": False, "D1": 0, "D2": 0, "latency": float(dense_latency[l]), "macs": F[l]})
        else:
            P = tucker_macs(layer, choice[0], choice[1])
            removed += F[l] - P
            out.append({"decomposed": True, "D1": choice[0], "D2": choice[1], "latency": float(choice[2]), "macs": P})
    return out

"""Algorithmic work of a Tucker-2 layer and the MI355X roofline it is priced against.

FLOPs follow the paper's complexity formula (section 3): 2*(H*W*C*R1 + Ho*Wo*K*K*R1*R2 + Ho*Wo*N*R2)
per image.  Bytes are the compulsory traffic of the fused layer: x read once, y written once,
the three weight tensors once; the intermediates z1, z2 are not compulsory and are not counted,
whichever variant runs.
"""
from __future__ import annotations

HBM_PEAK = 8.0e12            # bytes/s, MI355X HBM3E
FP32_MFMA_PEAK = 157.3e12    # flop/s, dense fp32 MFMA (same figure as packed fp32 VALU)


def flops(L) -> int:
    return 2 * L.batch * (L.H * L.W * L.C * L.R1 + L.Ho * L.Wo * L.K * L.K * L.R1 * L.R2 + L.Ho * L.Wo * L.N * L.R2)


def dense_flops(L) -> int:
    return 2 * L.batch * L.Ho * L.Wo * L.K * L.K * L.C * L.N


def bytes_compulsory(L) -> int:
    return 4 * (L.batch * L.C * L.H * L.W + L.batch * L.N * L.Ho * L.Wo
                + L.C * L.R1 + L.R1 * L.R2 * L.K * L.K + L.R2 * L.N)


def roofline(L):
    """Returns (bound, seconds, t_hbm, t_mfma): the larger of the two terms bounds the layer."""
    t_hbm = bytes_compulsory(L) / HBM_PEAK
    t_mfma = flops(L) / FP32_MFMA_PEAK
    return ("hbm" if t_hbm >= t_mfma else "mfma"), max(t_hbm, t_mfma), t_hbm, t_mfma

"""Pins for the CPU oracle: checks against what the paper and the mathematics fix.

Each ``pin_*`` function takes the oracle's Python front end (``orc``) and a loaded
oracle library (``lib``) and raises AssertionError when the oracle disagrees with
something that does not depend on the oracle itself: a hand-worked example, a
closed form, an independently written brute-force loop, a library routine
(numpy matmul / torch conv2d in fp64), or an invariant of the layer.

``test_oracle_pins.py`` runs them on the real oracle; ``test_oracle_mutants.py``
runs them on deliberately broken copies and requires each copy to be caught.
"""
from __future__ import annotations

import ctypes
import json
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

TIGHT = 1e-12      # fp64 agreement, normalised by the largest |value|


def _rand(sh, seed, integer=False):
    rng = np.random.default_rng(seed)
    if integer:
        f = lambda *s: rng.integers(-3, 4, size=s).astype(np.float32)
    else:
        f = lambda *s: rng.standard_normal(s).astype(np.float32)
    return dict(x=f(sh.batch, sh.C, sh.H, sh.W), U_in=f(sh.C, sh.R1),
                core=f(sh.R1, sh.R2, sh.K, sh.K), U_out=f(sh.R2, sh.N))


def _close(a, b, tol=TIGHT, what=""):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    assert a.shape == b.shape, "%s: shape %s vs %s" % (what, a.shape, b.shape)
    scale = max(np.abs(b).max(), 1e-300)
    err = np.abs(a - b).max() / scale
    assert err <= tol, "%s: normalised max error %.3e > %.1e" % (what, err, tol)


# --------------------------------------------------------------------------- shapes
def _shapes(orc):
    S = orc.Shape
    return [
        S(1, 5, 7, 6, 9, 3, 4, 3, 1, 1),      # everything different, asymmetric ranks
        S(2, 4, 3, 8, 5, 2, 5, 3, 2, 1),      # stride 2, batch 2, R2 > N
        S(1, 3, 6, 7, 7, 4, 2, 3, 1, 0),      # no padding ("valid"), R1 > C
        S(1, 6, 2, 5, 4, 3, 3, 1, 1, 0),      # 1x1 core
        S(3, 2, 2, 9, 6, 1, 1, 3, 2, 0),      # rank 1, stride 2 without padding
        S(1, 8, 8, 4, 4, 8, 8, 3, 1, 1),
    ]


# --------------------------------------------------------------------------- pins
def pin_handworked_golden(orc, lib):
    """The integer example worked by hand from Eqs. 2-4 (tests/golden)."""
    g = json.load(open(os.path.join(GOLDEN, "handworked_tucker2_3x3.json")))
    sh = orc.Shape(**g["shape"])
    args = [np.array(g[k], dtype=np.float32) for k in ("x", "U_in", "core", "U_out")]
    y, _, z1, z2 = orc.conv_factored(sh, *args, lib=lib, return_intermediates=True)
    assert np.array_equal(z1, np.array(g["z1"], dtype=np.float64)), "z1 (Eq. 2)"
    assert np.array_equal(z2, np.array(g["z2"], dtype=np.float64)), "z2 (Eq. 3)"
    assert np.array_equal(y, np.array(g["y"], dtype=np.float64)), "y (Eq. 4)"
    yd, _ = orc.conv_dense(sh, *args, lib=lib)
    assert np.array_equal(yd, np.array(g["y"], dtype=np.float64)), "y (Eq. 1 + definition)"


def pin_dense_equals_factored(orc, lib):
    """The paper's equivalence claim (after Eq. 4): three stages == dense conv with the kernel of Eq. 1."""
    for i, sh in enumerate(_shapes(orc)):
        t = _rand(sh, 100 + i)
        yf, _ = orc.conv_factored(sh, lib=lib, **t)
        yd, _ = orc.conv_dense(sh, lib=lib, **t)
        _close(yf, yd, what="dense vs factored %r" % (sh,))


def _brute(sh, x, U_in, core, U_out):
    """Eq. 1 substituted into the definition: one 9-deep loop, no intermediates.  Tiny shapes only."""
    y = np.zeros((sh.batch, sh.N, sh.Ho, sh.Wo), dtype=np.float64)
    x = x.astype(np.float64); U_in = U_in.astype(np.float64)
    core = core.astype(np.float64); U_out = U_out.astype(np.float64)
    for b in range(sh.batch):
        for n in range(sh.N):
            for i in range(sh.Ho):
                for j in range(sh.Wo):
                    acc = 0.0
                    for c in range(sh.C):
                        for r in range(sh.K):
                            for s in range(sh.K):
                                h = i * sh.stride + r - sh.pad
                                w = j * sh.stride + s - sh.pad
                                if not (0 <= h < sh.H and 0 <= w < sh.W):
                                    continue
                                for d1 in range(sh.R1):
                                    for d2 in range(sh.R2):
                                        acc += (x[b, c, h, w] * U_in[c, d1] * core[d1, d2, r, s]
                                                * U_out[d2, n])
                    y[b, n, i, j] = acc
    return y


def pin_bruteforce_tiny(orc, lib):
    """Small-integer tensors: the brute-force loop is exact, so equality is exact."""
    S = orc.Shape
    for i, sh in enumerate([S(1, 2, 3, 4, 4, 2, 2, 3, 1, 1), S(2, 3, 2, 5, 4, 2, 3, 3, 2, 1),
                            S(1, 2, 2, 4, 5, 3, 2, 3, 1, 0)]):
        t = _rand(sh, 200 + i, integer=True)
        want = _brute(sh, **t)
        yf, _ = orc.conv_factored(sh, lib=lib, **t)
        yd, _ = orc.conv_dense(sh, lib=lib, **t)
        assert np.array_equal(yf, want), "factored vs brute force %r" % (sh,)
        assert np.array_equal(yd, want), "dense vs brute force %r" % (sh,)


def pin_torch_conv2d(orc, lib):
    """Third opinion from a library routine: torch conv2d (fp64, CPU) with the kernel of Eq. 1 built by einsum."""
    import torch
    import torch.nn.functional as F
    for i, sh in enumerate(_shapes(orc)):
        t = _rand(sh, 300 + i)
        Wd = np.einsum("abrs,ca,bn->cnrs", t["core"].astype(np.float64),
                       t["U_in"].astype(np.float64), t["U_out"].astype(np.float64))
        w_oihw = torch.from_numpy(np.ascontiguousarray(Wd.transpose(1, 0, 2, 3)))
        want = F.conv2d(torch.from_numpy(t["x"].astype(np.float64)), w_oihw,
                        stride=sh.stride, padding=sh.pad).numpy()
        yf, _ = orc.conv_factored(sh, lib=lib, **t)
        yd, _ = orc.conv_dense(sh, lib=lib, **t)
        _close(yf, want, what="factored vs torch %r" % (sh,))
        _close(yd, want, what="dense vs torch %r" % (sh,))
        Wo, _ = orc.reconstruct(sh, t["U_in"], t["core"], t["U_out"], lib=lib)
        _close(Wo, Wd, what="Eq. 1 vs einsum %r" % (sh,))


def pin_intermediates(orc, lib):
    """Eq. 2 is a matrix product per pixel; Eq. 3 is a plain conv of z1 with core (in,out,r,s)."""
    import torch
    import torch.nn.functional as F
    sh = orc.Shape(2, 5, 4, 7, 6, 3, 2, 3, 2, 1)
    t = _rand(sh, 400)
    _, _, z1, z2 = orc.conv_factored(sh, lib=lib, return_intermediates=True, **t)
    z1_want = np.einsum("bchw,cd->bdhw", t["x"].astype(np.float64), t["U_in"].astype(np.float64))
    _close(z1, z1_want, what="z1")
    w = torch.from_numpy(np.ascontiguousarray(t["core"].astype(np.float64).transpose(1, 0, 2, 3)))
    z2_want = F.conv2d(torch.from_numpy(z1_want), w, stride=sh.stride, padding=sh.pad).numpy()
    _close(z2, z2_want, what="z2")


def pin_identity_factors(orc, lib):
    """C = R1, N = R2, U_in = I, U_out = I: the layer is a plain K x K conv with Wd[c][n] = core[c][n]."""
    import torch
    import torch.nn.functional as F
    sh = orc.Shape(1, 4, 3, 6, 5, 4, 3, 3, 1, 1)
    t = _rand(sh, 500)
    t["U_in"] = np.eye(4, dtype=np.float32)
    t["U_out"] = np.eye(3, dtype=np.float32)
    Wd, _ = orc.reconstruct(sh, t["U_in"], t["core"], t["U_out"], lib=lib)
    assert np.array_equal(Wd, t["core"].astype(np.float64)), "Eq. 1 with identity factors"
    w = torch.from_numpy(np.ascontiguousarray(t["core"].astype(np.float64).transpose(1, 0, 2, 3)))
    want = F.conv2d(torch.from_numpy(t["x"].astype(np.float64)), w, stride=1, padding=1).numpy()
    yf, _ = orc.conv_factored(sh, lib=lib, **t)
    _close(yf, want, what="identity factors")


def pin_delta_input(orc, lib):
    """x = delta(c0,h0,w0)  =>  y[n][i][j] = Wd[c0][n][h0 - i*st + pad][w0 - j*st + pad] (0 outside the filter)."""
    for st, pad in ((1, 1), (2, 1), (1, 0), (2, 0)):
        sh = orc.Shape(1, 3, 4, 7, 6, 2, 3, 3, st, pad)
        t = _rand(sh, 600 + st * 10 + pad)
        Wd = np.einsum("abrs,ca,bn->cnrs", t["core"].astype(np.float64),
                       t["U_in"].astype(np.float64), t["U_out"].astype(np.float64))
        for (c0, h0, w0) in ((1, 3, 2), (0, 0, 0), (2, 6, 5), (1, 0, 4)):
            x = np.zeros((1, sh.C, sh.H, sh.W), dtype=np.float32)
            x[0, c0, h0, w0] = 1.0
            want = np.zeros((1, sh.N, sh.Ho, sh.Wo))
            for i in range(sh.Ho):
                for j in range(sh.Wo):
                    r, s = h0 - i * st + pad, w0 - j * st + pad
                    if 0 <= r < sh.K and 0 <= s < sh.K:
                        want[0, :, i, j] = Wd[c0, :, r, s]
            tt = dict(t, x=x)
            yf, _ = orc.conv_factored(sh, lib=lib, **tt)
            yd, _ = orc.conv_dense(sh, lib=lib, **tt)
            _close(yf, want, what="delta factored st%d pad%d" % (st, pad))
            _close(yd, want, what="delta dense st%d pad%d" % (st, pad))


def pin_all_ones(orc, lib):
    """All-ones tensors: y = C*R1*R2 * (number of in-bounds taps): 9 inside, 6 on edges, 4 in corners (3x3, pad 1)."""
    sh = orc.Shape(1, 3, 2, 5, 6, 2, 4, 3, 1, 1)
    t = dict(x=np.ones((1, 3, 5, 6), np.float32), U_in=np.ones((3, 2), np.float32),
             core=np.ones((2, 4, 3, 3), np.float32), U_out=np.ones((4, 2), np.float32))
    taps = np.full((5, 6), 9.0)
    taps[0, :] = taps[-1, :] = 6.0
    taps[:, 0] = taps[:, -1] = 6.0
    taps[0, 0] = taps[0, -1] = taps[-1, 0] = taps[-1, -1] = 4.0
    want = np.broadcast_to(3 * 2 * 4 * taps, (1, 2, 5, 6))
    yf, _ = orc.conv_factored(sh, lib=lib, **t)
    yd, _ = orc.conv_dense(sh, lib=lib, **t)
    assert np.array_equal(yf, want) and np.array_equal(yd, want), "all-ones tap count"
    # output size rule: floor((H + 2*pad - K)/stride) + 1
    for (H, K, st, pad, Ho) in ((7, 3, 2, 1, 4), (8, 3, 2, 1, 4), (56, 3, 2, 1, 28), (5, 3, 1, 0, 3), (6, 1, 2, 0, 3)):
        s2 = orc.Shape(1, 1, 1, H, H, 1, 1, K, st, pad)
        cs = s2.c_struct()
        assert lib.orc_out_h(ctypes.byref(cs)) == Ho == s2.Ho, "Ho for H=%d K=%d st=%d pad=%d" % (H, K, st, pad)
        t2 = dict(x=np.ones((1, 1, H, H), np.float32), U_in=np.ones((1, 1), np.float32),
                  core=np.ones((1, 1, K, K), np.float32), U_out=np.ones((1, 1), np.float32))
        y2, _ = orc.conv_factored(s2, lib=lib, **t2)
        assert y2.shape == (1, 1, Ho, Ho)
        # last output row/column: taps that fall inside the image, counted directly
        last = (Ho - 1) * st - pad
        inside = sum(1 for r in range(K) if 0 <= last + r < H)
        assert y2[0, 0, Ho - 1, Ho - 1] == inside * inside, "tap count in the last row/column"


def pin_k1_matmul(orc, lib):
    """K = 1, pad 0: y = U_out^T (core00^T (U_in^T x)) -- three numpy matmuls."""
    sh = orc.Shape(2, 6, 5, 4, 3, 3, 4, 1, 1, 0)
    t = _rand(sh, 700)
    X = t["x"].astype(np.float64).reshape(2, 6, 12)
    A = t["U_in"].astype(np.float64).T            # R1 x C
    Bm = t["core"].astype(np.float64)[:, :, 0, 0].T  # R2 x R1
    Cm = t["U_out"].astype(np.float64).T           # N x R2
    want = np.matmul(Cm, np.matmul(Bm, np.matmul(A, X))).reshape(2, 5, 4, 3)
    yf, _ = orc.conv_factored(sh, lib=lib, **t)
    yd, _ = orc.conv_dense(sh, lib=lib, **t)
    _close(yf, want, what="K=1 factored")
    _close(yd, want, what="K=1 dense")


def pin_linearity(orc, lib):
    """y(a*x1 + b*x2) = a*y(x1) + b*y(x2); inputs chosen so that a*x1 + b*x2 is exact in fp32."""
    sh = orc.Shape(1, 4, 5, 6, 7, 3, 2, 3, 1, 1)
    t = _rand(sh, 800)
    rng = np.random.default_rng(801)
    x1 = rng.integers(-8, 9, size=(1, 4, 6, 7)).astype(np.float32)
    x2 = rng.integers(-8, 9, size=(1, 4, 6, 7)).astype(np.float32)
    a, b = 3.0, -0.5
    for f in (orc.conv_factored, orc.conv_dense):
        y1, _ = f(sh, lib=lib, **dict(t, x=x1))
        y2, _ = f(sh, lib=lib, **dict(t, x=x2))
        y12, _ = f(sh, lib=lib, **dict(t, x=(a * x1 + b * x2).astype(np.float32)))
        _close(y12, a * y1 + b * y2, what="linearity %s" % f.__name__)


def pin_translation(orc, lib):
    """Stride 1: shifting x by (dh,dw) shifts y by the same amount away from the borders."""
    sh = orc.Shape(1, 3, 2, 9, 10, 2, 3, 3, 1, 1)
    t = _rand(sh, 900)
    x = t["x"]
    xs = np.zeros_like(x)
    xs[:, :, 2:, 1:] = x[:, :, :-2, :-1]
    y, _ = orc.conv_factored(sh, lib=lib, **t)
    ys, _ = orc.conv_factored(sh, lib=lib, **dict(t, x=xs))
    _close(ys[:, :, 4:-1, 3:-1], y[:, :, 2:-3, 2:-2], what="translation")


def pin_batch_independence(orc, lib):
    sh = orc.Shape(3, 4, 3, 5, 6, 2, 2, 3, 2, 1)
    t = _rand(sh, 1000)
    y, _ = orc.conv_factored(sh, lib=lib, **t)
    yd, _ = orc.conv_dense(sh, lib=lib, **t)
    s1 = orc.Shape(1, 4, 3, 5, 6, 2, 2, 3, 2, 1)
    for b in range(3):
        yb, _ = orc.conv_factored(s1, lib=lib, **dict(t, x=t["x"][b:b + 1]))
        assert np.array_equal(yb[0], y[b]), "batch image %d (factored)" % b
        ydb, _ = orc.conv_dense(s1, lib=lib, **dict(t, x=t["x"][b:b + 1]))
        assert np.array_equal(ydb[0], yd[b]), "batch image %d (dense)" % b


def pin_gauge(orc, lib):
    """Tucker non-uniqueness: U_in -> U_in A, core -> A^-1 x_1 core leaves y unchanged (and likewise on mode 2).

    A is a signed permutation times powers of two, so the transformed weights are exact in fp32."""
    sh = orc.Shape(1, 5, 4, 6, 6, 3, 4, 3, 1, 1)
    t = _rand(sh, 1100)
    A = np.array([[0, 2, 0], [0, 0, -0.5], [4, 0, 0]], dtype=np.float64)
    Ainv = np.linalg.inv(A)
    Bm = np.array([[0, 0, 0, 2], [0.25, 0, 0, 0], [0, 0, -1, 0], [0, 8, 0, 0]], dtype=np.float64)
    Binv = np.linalg.inv(Bm)
    U_in2 = (t["U_in"].astype(np.float64) @ A).astype(np.float32)
    core2 = np.einsum("ad,dbrs->abrs", Ainv, t["core"].astype(np.float64))
    core2 = np.einsum("abrs,bq->aqrs", core2, Bm).astype(np.float32)
    U_out2 = (Binv @ t["U_out"].astype(np.float64)).astype(np.float32)
    y, _ = orc.conv_factored(sh, lib=lib, **t)
    y2, _ = orc.conv_factored(sh, lib=lib, x=t["x"], U_in=U_in2, core=core2, U_out=U_out2)
    _close(y2, y, what="gauge transform (factored)")
    yd2, _ = orc.conv_dense(sh, lib=lib, x=t["x"], U_in=U_in2, core=core2, U_out=U_out2)
    _close(yd2, y, what="gauge transform (dense)")


def pin_mac_counts(orc, lib):
    """Loop bounds against the paper's complexity formula (section 3): H*W*C*D1 + H'W'*R*S*D1*D2 + H'W'*N*D2."""
    for sh in _shapes(orc) + [orc.Shape(1, 64, 64, 56, 56, 16, 16, 3, 1, 1)]:
        t = _rand(sh, 1200)
        _, m = orc.conv_factored(sh, lib=lib, **t)
        B, Ho, Wo = sh.batch, sh.Ho, sh.Wo
        assert m == [B * sh.H * sh.W * sh.C * sh.R1,
                     B * Ho * Wo * sh.K * sh.K * sh.R1 * sh.R2,
                     B * Ho * Wo * sh.N * sh.R2], "stage MACs %r: %r" % (sh, m)
        _, md = orc.conv_dense(sh, lib=lib, **t)
        assert md == B * Ho * Wo * sh.K * sh.K * sh.C * sh.N
        _, mr = orc.reconstruct(sh, t["U_in"], t["core"], t["U_out"], lib=lib)
        assert mr == sh.C * sh.N * sh.K * sh.K * sh.R1 * sh.R2
    # FLOPs reduction ratio gamma_F of section 3 for C=N=64, 56x56, D1=D2=16: 115605504 / 13647872 = 8.47
    sh = orc.Shape(1, 64, 64, 56, 56, 16, 16, 3, 1, 1)
    t = _rand(sh, 1201)
    _, m = orc.conv_factored(sh, lib=lib, **t)
    _, md = orc.conv_dense(sh, lib=lib, **t)
    assert abs(md / sum(m) - 8.4706) < 1e-3


ALL_PINS = [pin_handworked_golden, pin_dense_equals_factored, pin_bruteforce_tiny, pin_torch_conv2d,
            pin_intermediates, pin_identity_factors, pin_delta_input, pin_all_ones, pin_k1_matmul,
            pin_linearity, pin_translation, pin_batch_independence, pin_gauge, pin_mac_counts]

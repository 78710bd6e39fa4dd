"""Truncated-HOSVD projection and ADMM auxiliary updates (paper section 4): the oracle against
hand-worked cases and properties, planted mistakes, and the library's host routines against the
oracle.  Host arithmetic only: no GPU (one round-trip test through the GPU layer is marked gpu)."""
import json
import os
import types

import numpy as np
import pytest

from oracle import hosvd_oracle as HO
from paper_2211_03715_amd import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))
GOLDEN = json.load(open(os.path.join(HERE, "golden", "hosvd_handworked.json")))


def _t(mat):
    a = np.asarray(mat, dtype=np.float64)
    return a.reshape(a.shape[0], a.shape[1], 1, 1)


def _random_w(rng, C, N, K):
    return rng.standard_normal((C, N, K, K))


def _low_rank_w(rng, C, N, K, r1, r2):
    return HO.reconstruct(rng.standard_normal((C, r1)), rng.standard_normal((r1, r2, K, K)), rng.standard_normal((r2, N)))


def check_handworked(mod):
    for c in GOLDEN["cases"]:
        U_in, core, U_out = mod.hosvd_tucker2(_t(c["W"]), c["R1"], c["R2"])
        assert np.allclose(np.abs(U_in), np.asarray(c["abs_U_in"]), atol=1e-12), c["_why"]
        assert np.allclose(np.abs(core).ravel(), [c["abs_core"]], atol=1e-12), c["_why"]
        assert np.allclose(np.abs(U_out), np.asarray(c["abs_U_out"]), atol=1e-12), c["_why"]
        assert np.allclose(mod.project(_t(c["W"]), c["R1"], c["R2"]), _t(c["K_hat"]), atol=1e-12), c["_why"]
    for c in GOLDEN["admm"]:
        K_hat, M_new = mod.admm_aux_updates(_t(c["K"]), _t(c["M"]), c["R1"], c["R2"])
        assert np.allclose(K_hat, _t(c["K_hat"]), atol=1e-12), c["_why"]
        assert np.allclose(M_new, _t(c["M_new"]), atol=1e-12), c["_why"]


def check_properties(mod):
    rng = np.random.default_rng(2211)
    # an exactly low-rank tensor is reproduced, and its factors feed Eq. 1 in the library's layouts
    W = _low_rank_w(rng, 9, 7, 3, 3, 2)
    U_in, core, U_out = mod.hosvd_tucker2(W, 3, 2)
    assert U_in.shape == (9, 3) and core.shape == (3, 2, 3, 3) and U_out.shape == (2, 7)
    assert np.allclose(mod.reconstruct(U_in, core, U_out), W, atol=1e-10)
    # full ranks are exact for any tensor; factors are orthonormal
    W = _random_w(rng, 6, 5, 3)
    U_in, core, U_out = mod.hosvd_tucker2(W, 6, 5)
    assert np.allclose(mod.reconstruct(U_in, core, U_out), W, atol=1e-10)
    U_in, core, U_out = mod.hosvd_tucker2(W, 4, 2)
    assert np.allclose(U_in.T @ U_in, np.eye(4), atol=1e-12) and np.allclose(U_out @ U_out.T, np.eye(2), atol=1e-12)
    # HOSVD error bounds: max(tail_1, tail_2) <= ||W - proj W||^2 <= tail_1 + tail_2, tails of squared singular values
    # (singular values recomputed here from the Gram matrices' eigenvalues, not through the oracle's SVD call)
    for (C, N, K, r1, r2) in ((8, 6, 3, 3, 4), (5, 9, 1, 2, 2), (12, 10, 3, 11, 3)):
        W = _random_w(rng, C, N, K)
        e1 = np.sort(np.linalg.eigvalsh(W.reshape(C, -1) @ W.reshape(C, -1).T))[::-1]
        W2 = np.transpose(W, (1, 0, 2, 3)).reshape(N, -1)
        e2 = np.sort(np.linalg.eigvalsh(W2 @ W2.T))[::-1]
        t1, t2 = e1[r1:].sum(), e2[r2:].sum()
        err = ((W - mod.project(W, r1, r2)) ** 2).sum()
        assert max(t1, t2) * (1 - 1e-9) <= err <= (t1 + t2) * (1 + 1e-9)
        # the projection is idempotent and never increases the norm
        P = mod.project(W, r1, r2)
        assert np.allclose(mod.project(P, r1, r2), P, atol=1e-9)
        assert (P ** 2).sum() <= (W ** 2).sum() * (1 + 1e-12)
        # the kept directions are the leading ones: the projector captures the top eigen-energy of the Gram matrix
        U_in, _, U_out = mod.hosvd_tucker2(W, r1, r2)
        assert np.isclose(np.trace(U_in.T @ (W.reshape(C, -1) @ W.reshape(C, -1).T) @ U_in), e1[:r1].sum(), rtol=1e-10)
        assert np.isclose(np.trace(U_out @ (W2 @ W2.T) @ U_out.T), e2[:r2].sum(), rtol=1e-10)
    # ADMM: at a fixed point (K already of the target ranks, M = 0) nothing moves; and K-hat + M_new = K + M always
    K = _low_rank_w(rng, 7, 6, 3, 2, 3)
    K_hat, M_new = mod.admm_aux_updates(K, np.zeros_like(K), 2, 3)
    assert np.allclose(K_hat, K, atol=1e-10) and np.allclose(M_new, 0.0, atol=1e-10)
    K, M = _random_w(rng, 6, 6, 3), 0.1 * _random_w(rng, 6, 6, 3)
    K_hat, M_new = mod.admm_aux_updates(K, M, 3, 3)
    assert np.allclose(K_hat + M_new, K + M, atol=1e-12)
    assert np.allclose(K_hat, mod.project(K + M, 3, 3), atol=1e-12)


def test_oracle_handworked():
    check_handworked(HO)


def test_oracle_properties():
    check_properties(HO)


MUTATIONS = [
    ("U1 = U1[:, :R1]", "U1 = U1[:, -R1:]"),                                    # smallest instead of largest
    ("U2 = U2[:, :R2]", "U2 = U2[:, -R2:]"),
    ('np.einsum("cnrs,cd,ne->ders"', 'np.einsum("cnrs,cd,ne->edrs"'),                 # core modes swapped
    ("np.transpose(W, (1, 0, 2, 3)).reshape(N, -1), full_matrices=False)", "W.reshape(N, -1), full_matrices=False)"),   # no transposition before unfolding mode 2
    ("return U1, core, np.ascontiguousarray(U2.T)", "return U1, core, np.ascontiguousarray(U2.T[::-1])"),
    ('np.einsum("ders,cd,en->cnrs"', 'np.einsum("ders,cd,en->cnsr"'),
    ("return K_hat, M + K - K_hat", "return K_hat, M - K + K_hat"),
    ("K_hat = project(K + M, R1, R2)", "K_hat = project(K, R1, R2)"),
]


@pytest.mark.parametrize("idx", range(len(MUTATIONS)))
def test_planted_mistakes_in_the_oracle_are_caught(idx):
    old, new = MUTATIONS[idx]
    src = open(HO.__file__).read()
    assert src.count(old) == 1, "mutation target vanished: %r" % old
    mod = types.ModuleType("hosvd_oracle_mutant")
    exec(compile(src.replace(old, new, 1), "hosvd_oracle_mutant", "exec"), mod.__dict__)
    with pytest.raises(Exception):
        check_handworked(mod)
        check_properties(mod)


# ---------------------------------------------------------------- the library against the oracle

class _Lib:
    """The library's host routines behind the oracle's function names (float32 in and out)."""

    @staticmethod
    def hosvd_tucker2(W, R1, R2):
        return tuple(a.astype(np.float64) for a in B.tdc_hosvd_tucker2(np.asarray(W, np.float32), R1, R2))

    reconstruct = staticmethod(HO.reconstruct)

    @staticmethod
    def project(W, R1, R2):
        return HO.reconstruct(*_Lib.hosvd_tucker2(W, R1, R2))

    @staticmethod
    def admm_aux_updates(K, M, R1, R2):
        K_hat, M_new = B.tdc_admm_project(np.asarray(K, np.float32), np.asarray(M, np.float32), R1, R2)
        return K_hat.astype(np.float64), M_new.astype(np.float64)


def test_library_handworked():
    for c in GOLDEN["cases"]:
        U_in, core, U_out = _Lib.hosvd_tucker2(_t(c["W"]), c["R1"], c["R2"])
        assert np.allclose(np.abs(U_in), np.asarray(c["abs_U_in"]), atol=1e-6), c["_why"]
        assert np.allclose(np.abs(core).ravel(), [c["abs_core"]], atol=1e-5), c["_why"]
        assert np.allclose(np.abs(U_out), np.asarray(c["abs_U_out"]), atol=1e-6), c["_why"]
        assert np.allclose(_Lib.project(_t(c["W"]), c["R1"], c["R2"]), _t(c["K_hat"]), atol=1e-5), c["_why"]
        assert U_in[np.argmax(np.abs(U_in[:, 0])), 0] > 0          # the documented sign convention
    for c in GOLDEN["admm"]:
        K_hat, M_new = _Lib.admm_aux_updates(_t(c["K"]), _t(c["M"]), c["R1"], c["R2"])
        assert np.allclose(K_hat, _t(c["K_hat"]), atol=1e-6) and np.allclose(M_new, _t(c["M_new"]), atol=1e-6), c["_why"]


@pytest.mark.parametrize("shape", [(8, 6, 3, 3, 4), (16, 24, 3, 5, 7), (33, 20, 1, 8, 8), (64, 48, 3, 16, 12), (5, 5, 5, 5, 5)],
                         ids=lambda s: "c%d_n%d_k%d_r%d-%d" % s)
def test_library_equals_oracle(shape):
    C, N, K, r1, r2 = shape
    rng = np.random.default_rng(C * 1000 + N)
    W = _random_w(rng, C, N, K).astype(np.float32)
    want = HO.project(W, r1, r2)
    U_in, core, U_out = _Lib.hosvd_tucker2(W, r1, r2)
    got = HO.reconstruct(U_in, core, U_out)
    scale = np.abs(want).max()
    assert np.abs(got - want).max() <= 2e-5 * scale                     # fp32 rounding of the three factors
    oU_in, _, oU_out = HO.hosvd_tucker2(W, r1, r2)
    assert np.abs(U_in @ U_in.T - oU_in @ oU_in.T).max() <= 1e-5        # same subspaces (vectors differ by sign)
    assert np.abs(U_out.T @ U_out - oU_out.T @ oU_out).max() <= 1e-5
    M = (0.05 * _random_w(rng, C, N, K)).astype(np.float32)
    K_hat, M_new = _Lib.admm_aux_updates(W, M, r1, r2)
    oK_hat, oM_new = HO.admm_aux_updates(W, M, r1, r2)
    assert np.abs(K_hat - oK_hat).max() <= 2e-5 * scale and np.abs(M_new - oM_new).max() <= 2e-5 * scale


def test_library_rejects_bad_arguments():
    W = np.zeros((4, 3, 3, 3), dtype=np.float32)
    for r1, r2 in ((0, 1), (1, 0), (5, 1), (1, 4)):
        with pytest.raises(B.TdcError) as e:
            B.tdc_hosvd_tucker2(W, r1, r2)
        assert e.value.status == B.TDC_ERR_BAD_SHAPE
    lib = B.load()
    assert lib.tdc_hosvd_tucker2(None, 4, 3, 3, 1, 1, None, None, None) == B.TDC_ERR_NULL
    assert lib.tdc_admm_project(None, None, 4, 3, 3, 1, 1, None) == B.TDC_ERR_NULL


@pytest.mark.gpu
def test_decomposed_layer_runs_on_the_gpu_and_matches_the_dense_layer(orc):
    """Round trip: a dense kernel of exact Tucker ranks is decomposed on the host and evaluated by the GPU
    Tucker layer; the result is the dense convolution with the original kernel."""
    import torch
    from paper_2211_03715_amd.layer import TuckerConv2d
    from paper_2211_03715_amd.workloads import Layer
    from parity_util import assert_parity
    print("[case] hosvd round trip", flush=True)
    rng = np.random.default_rng(3)
    L = Layer(2, 24, 40, 13, 11, 8, 12)
    W = (_low_rank_w(rng, L.C, L.N, 3, L.R1, L.R2) * 0.05).astype(np.float32)
    x = rng.standard_normal((L.batch, L.C, L.H, L.W), dtype=np.float32)
    want, _ = orc.conv_dense_with(orc.Shape(**L.asdict()), x, W.astype(np.float64))
    U_in, core, U_out = B.tdc_hosvd_tucker2(W, L.R1, L.R2)
    dev = torch.device("cuda:0")
    conv = TuckerConv2d(L, 0)
    try:
        t = [torch.from_numpy(a).to(dev) for a in (U_in, core, U_out)]
        conv.pack(*t)
        y = conv(torch.from_numpy(x).to(dev))
        torch.cuda.synchronize()
        assert_parity(y.cpu().numpy(), want, "hosvd -> tucker layer")
    finally:
        conv.close()

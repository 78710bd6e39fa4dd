"""CPU oracle of the projection onto Tucker-2 format and of the ADMM auxiliary updates (paper section 4).

TEST INFRASTRUCTURE ONLY: tests/ may import this; the product (libtdc.so's tdc_hosvd_tucker2 and
tdc_admm_project) shares no code with it.

proj (the paper's K-hat update): for T in R^{C x N x R x S}, take the SVDs of the mode-1 matricization
T_(1) (C x NRS) and of the mode-2 matricization T_(2) (N x CRS), keep the D1 (resp. D2) left singular
vectors of the largest singular values as U1 (C x D1) and U2 (N x D2), form the core
C = T x_1 U1^T x_2 U2^T (D1 x D2 x R x S), and recover K-hat = C x_1 U1 x_2 U2 (Eq. 1).
M update: M <- M + K - K-hat.

numpy.linalg.svd (LAPACK) is the library primitive for the SVD step; everything else is written out
with einsum in float64, in the order the section states it.

Layouts are the library's: W[C][N][K][K], U_in[C][R1] = U1, core[R1][R2][K][K], U_out[R2][N] = U2^T.
Singular vectors are only defined up to sign (and up to rotation inside a repeated singular value),
so tests compare what is unique: the projected tensor K-hat, the projectors U U^T, the singular values.
"""
from __future__ import annotations

import numpy as np


def mode_singular_values(W):
    """Singular values of the mode-1 and mode-2 matricizations, descending."""
    W = np.asarray(W, dtype=np.float64)
    C, N = W.shape[0], W.shape[1]
    s1 = np.linalg.svd(W.reshape(C, -1), compute_uv=False)
    s2 = np.linalg.svd(np.transpose(W, (1, 0, 2, 3)).reshape(N, -1), compute_uv=False)
    return s1, s2


def hosvd_tucker2(W, R1: int, R2: int):
    """Truncated HOSVD.  Returns (U_in [C][R1], core [R1][R2][K][K], U_out [R2][N]) in float64."""
    W = np.asarray(W, dtype=np.float64)
    C, N = W.shape[0], W.shape[1]
    U1, _, _ = np.linalg.svd(W.reshape(C, -1), full_matrices=False)                                  # T_(1) = U1 S1 V1
    U2, _, _ = np.linalg.svd(np.transpose(W, (1, 0, 2, 3)).reshape(N, -1), full_matrices=False)      # T_(2) = U2 S2 V2
    U1 = U1[:, :R1]
    U2 = U2[:, :R2]
    core = np.einsum("cnrs,cd,ne->ders", W, U1, U2)          # T x_1 U1^T x_2 U2^T
    return U1, core, np.ascontiguousarray(U2.T)


def reconstruct(U_in, core, U_out):
    """Eq. 1: K(c,n,r,s) = sum_{d1,d2} core(d1,d2,r,s) U1(c,d1) U2(n,d2)."""
    return np.einsum("ders,cd,en->cnrs", np.asarray(core, np.float64), np.asarray(U_in, np.float64), np.asarray(U_out, np.float64))


def project(T, R1: int, R2: int):
    """proj(T): the tensor of Tucker ranks (R1, R2) the truncated HOSVD yields."""
    return reconstruct(*hosvd_tucker2(T, R1, R2))


def admm_aux_updates(K, M, R1: int, R2: int):
    """K-hat <- proj(K + M);  M <- M + K - K-hat.  Returns (K_hat, M_new)."""
    K = np.asarray(K, dtype=np.float64)
    M = np.asarray(M, dtype=np.float64)
    K_hat = project(K + M, R1, R2)
    return K_hat, M + K - K_hat

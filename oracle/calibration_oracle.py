"""fp64 oracle of the offline calibration (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this
module.  It imports nothing from the HIP package.

Sec. 4.2 of the paper (arXiv 2510.24273): the pre-RoPE keys of the calibration tokens, all heads of a token
merged into one row of width n*d, are stacked into K [s x nd]; the covariance is C = K^T K; its eigenvalue
decomposition C = U Sigma U^T is taken and the r leading eigenvectors U_r are the projection into the latent
space.  The functions below are those definitions written out with numpy's fp64 matrix product and its
symmetric eigensolver as library steps; nothing is blocked, fused or reordered.

Eigenvectors are unique up to sign only (and up to a rotation inside an eigenspace of a repeated eigenvalue), so
comparisons against this oracle are made up to sign, or through quantities that are unique: the eigenvalues, the
projector U_r U_r^T when lambda_r > lambda_{r+1}, and the captured energy tr(U_r^T C U_r) (Lemma 1).

Pins: ``tests/test_oracle_calibration_pins.py``.
"""
from __future__ import annotations

import numpy as np


def covariance(K):
    """C = K^T K for K [s, nd] (Sec. 4.2): C[i, j] = sum_t K[t, i] K[t, j].  No centring, no 1/s factor."""
    K = np.asarray(K, dtype=np.float64)
    return K.T @ K


def eigen_decomposition(C):
    """C = U diag(lam) U^T with lam in descending order (Sec. 4.2).  Returns (lam [nd], U [nd, nd])."""
    C = np.asarray(C, dtype=np.float64)
    lam, U = np.linalg.eigh(C)          # ascending
    return lam[::-1].copy(), U[:, ::-1].copy()


def leading_eigenvectors(C, r):
    """The r leading eigenvectors U_r [nd, r] (columns, eigenvalue descending) and all eigenvalues."""
    lam, U = eigen_decomposition(C)
    return lam, U[:, :r].copy()


def captured_energy(C, U):
    """E(U) = tr(U^T C U): the variance of the calibration keys captured by the columns of U (Lemma 1)."""
    C = np.asarray(C, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    return float(np.trace(U.T @ C @ U))


def calibrate(K, r):
    """Keys -> (C, lam, U_r): the whole offline step of Sec. 4.2."""
    C = covariance(K)
    lam, U = leading_eigenvectors(C, r)
    return C, lam, U

"""Pins of the calibration oracle (Sec. 4.2, Lemma 1; CPU only): the covariance and the leading eigenvectors are
checked against loops and closed forms written out here, a constructed spectrum, the Eckart-Young identity, the
optimality of the captured energy and the lemma's joint-versus-per-head inequality."""
import math

import numpy as np
import pytest

from oracle import calibration_oracle as cal


def _same_up_to_sign(a, b, tol):
    """columns of a and b agree up to the sign of each column"""
    for i in range(a.shape[1]):
        d = min(np.max(np.abs(a[:, i] - b[:, i])), np.max(np.abs(a[:, i] + b[:, i])))
        assert d <= tol, (i, d)


def test_covariance_is_the_sum_of_outer_products_of_the_rows():
    rng = np.random.default_rng(1)
    K = rng.standard_normal((7, 5))
    C = np.zeros((5, 5))
    for t in range(7):           # sum over calibration tokens
        for i in range(5):
            for j in range(5):
                C[i, j] += K[t, i] * K[t, j]
    got = cal.covariance(K)
    assert got.shape == (5, 5)   # (K K^T would be 7 x 7)
    np.testing.assert_allclose(got, C, rtol=0, atol=1e-13)
    # not centred, not divided by the number of rows
    np.testing.assert_allclose(np.trace(got), np.sum(K * K), rtol=1e-14)


def test_two_by_two_closed_form():
    a, b, d = 3.0, 1.25, 0.5
    C = np.array([[a, b], [b, d]])
    lam, U = cal.eigen_decomposition(C)
    mid, rad = 0.5 * (a + d), math.sqrt((0.5 * (a - d)) ** 2 + b * b)
    np.testing.assert_allclose(lam, [mid + rad, mid - rad], rtol=1e-14)      # descending
    v = np.array([b, lam[0] - a]); v /= np.linalg.norm(v)                     # (C - lam I) v = 0
    _same_up_to_sign(U[:, :1], v[:, None], 1e-14)
    lam1, U1 = cal.leading_eigenvectors(C, 1)
    assert U1.shape == (2, 1)
    _same_up_to_sign(U1, v[:, None], 1e-14)


def test_constructed_spectrum_is_recovered_in_descending_order():
    rng = np.random.default_rng(2)
    D, s = 24, 60
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    G, _ = np.linalg.qr(rng.standard_normal((s, D)))       # orthonormal columns: G^T G = I
    sig = np.sort(rng.uniform(0.5, 4.0, D))[::-1] * (1.0 + 0.05 * np.arange(D)[::-1])  # distinct, descending
    K = (G * sig) @ Q.T                                      # so that K^T K = Q diag(sig^2) Q^T
    C, lam, U = cal.calibrate(K, 6)
    np.testing.assert_allclose(lam, sig ** 2, rtol=1e-11)
    _same_up_to_sign(U, Q[:, :6], 1e-10)
    np.testing.assert_allclose(U.T @ U, np.eye(6), atol=1e-13)
    np.testing.assert_allclose(C @ U, U * lam[:6], atol=1e-11)


def test_eckart_young_and_optimality_of_the_captured_energy():
    rng = np.random.default_rng(3)
    K = rng.standard_normal((40, 12)) * (np.arange(12, 0, -1) ** 0.7)
    r = 4
    C, lam, U = cal.calibrate(K, r)
    # what the projection loses is the tail of the spectrum
    resid = K - (K @ U) @ U.T
    np.testing.assert_allclose(np.sum(resid * resid), np.sum(lam[r:]), rtol=1e-11)
    np.testing.assert_allclose(cal.captured_energy(C, U), np.sum(lam[:r]), rtol=1e-12)
    # no other orthonormal basis of the same rank captures more
    for _ in range(50):
        W, _ = np.linalg.qr(rng.standard_normal((12, r)))
        assert cal.captured_energy(C, W) <= cal.captured_energy(C, U) * (1 + 1e-12)


@pytest.mark.parametrize("n_heads,d,r", [(4, 8, 8), (2, 16, 4), (8, 4, 16)])
def test_lemma_joint_projection_captures_at_least_the_per_head_one(n_heads, d, r):
    rng = np.random.default_rng(10 * n_heads + r)
    D = n_heads * d
    mix = rng.standard_normal((D, D))                      # heads are correlated
    K = rng.standard_normal((200, D)) @ mix
    C, lam, U = cal.calibrate(K, r)
    rp = r // n_heads
    B = np.zeros((D, r))
    for h in range(n_heads):                               # best block-diagonal basis: each head on its own
        blk = C[h * d:(h + 1) * d, h * d:(h + 1) * d]
        w, V = np.linalg.eigh(blk)
        B[h * d:(h + 1) * d, h * rp:(h + 1) * rp] = V[:, ::-1][:, :rp]
    np.testing.assert_allclose(B.T @ B, np.eye(r), atol=1e-12)
    assert cal.captured_energy(C, U) >= cal.captured_energy(C, B) * (1 - 1e-12)
    assert cal.captured_energy(C, U) > cal.captured_energy(C, B) * 1.01   # strictly more once heads are correlated


def test_generator_plants_the_spectrum_it_claims():
    from paper_2510_24273_amd import synth
    X = synth.widen(synth.make_calibration_keys(5, 4000, 32, "f32", decay=0.8))
    lam, _ = cal.eigen_decomposition(cal.covariance(X) / 4000.0)
    want = 0.8 ** np.arange(32)
    assert np.all(np.abs(lam[:8] / want[:8] - 1.0) < 0.2)   # sample eigenvalues of 4000 rows: within 20 %

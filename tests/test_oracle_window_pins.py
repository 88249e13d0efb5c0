"""Pins of the oracle's overlap score (Sec. 3.2) and recent-window attention (Sec. 5.1), CPU only.
Everything is checked against arithmetic written out in this file (loops, its own RoPE and
softmax), against hand-worked values, and against special cases that collapse to functions
pinned elsewhere."""
import math

import numpy as np
import pytest


def _rope(x, pos, theta, style=0):
    """One vector: pair i turns by pos * theta^(-2i/d); pairs (i, i+d/2) or (2i, 2i+1)."""
    d = x.shape[0]
    out = np.array(x, dtype=np.float64)
    for i in range(d // 2):
        ang = pos * theta ** (-2.0 * i / d)
        a, b = (i, i + d // 2) if style == 0 else (2 * i, 2 * i + 1)
        out[a] = x[a] * math.cos(ang) - x[b] * math.sin(ang)
        out[b] = x[b] * math.cos(ang) + x[a] * math.sin(ang)
    return out


def _softmax_attend(qR, keys, vals, H_kv):
    """qR [H,d]; keys, vals: lists of [H_kv*d] vectors (keys already rotated)."""
    H, d = qR.shape
    G = H // H_kv
    y = np.zeros((H, d))
    for h in range(H):
        g = h // G
        x = np.array([qR[h] @ k[g * d:(g + 1) * d] / math.sqrt(d) for k in keys])
        p = np.exp(x - x.max())
        p /= p.sum()
        for pj, v in zip(p, vals):
            y[h] += pj * v[g * d:(g + 1) * d]
    return y


# ---- overlap score ---------------------------------------------------------------------

def test_overlap_hand_worked(oracle):
    # query at position 0 (no rotation) along the first axis; key j has logit ln(a_j), so p_j = a_j / 10
    d = 4
    a = np.array([1.0, 2.0, 3.0, 4.0])
    q = np.zeros((1, d)); q[0, 0] = math.sqrt(d)
    KR = np.zeros((4, 1, d)); KR[:, 0, 0] = np.log(a)
    os_ = oracle.overlap_score(q, 0, KR, [1, 3], 1e4)
    np.testing.assert_allclose(os_, [0.6], rtol=0, atol=1e-14)
    np.testing.assert_allclose(oracle.overlap_score(q, 0, KR, [0], 1e4), [0.1], rtol=0, atol=1e-14)


@pytest.mark.parametrize("style", [0, 1])
def test_overlap_brute_force_and_complement(oracle, style):
    rng = np.random.default_rng(3 + style)
    H, H_kv, d, S, theta = 4, 2, 8, 23, 100.0
    q = rng.standard_normal((H, d))
    KR = rng.standard_normal((S, H_kv, d)) * 1.5
    idx = rng.choice(S, 7, replace=False)
    rest = np.setdiff1d(np.arange(S), idx)
    got = oracle.overlap_score(q, S, KR, idx, theta, style)
    want = np.zeros(H)
    for h in range(H):
        qr = _rope(q[h], S, theta, style)
        x = np.array([qr @ KR[j, h // 2] / math.sqrt(d) for j in range(S)])
        p = np.exp(x - x.max())
        want[h] = p[idx].sum() / p.sum()
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
    np.testing.assert_allclose(got + oracle.overlap_score(q, S, KR, rest, theta, style), np.ones(H), atol=1e-13)
    np.testing.assert_allclose(oracle.overlap_score(q, S, KR, np.arange(S), theta, style), np.ones(H), atol=1e-13)
    assert np.all(oracle.overlap_score(q, S, KR, [], theta, style) == 0)


# ---- recent window ---------------------------------------------------------------------

def _ortho(rng, D, r):
    qm, _ = np.linalg.qr(rng.standard_normal((D, r)))
    return qm


@pytest.mark.parametrize("style", [0, 1])
def test_window_brute_force_with_ring_wrap(oracle, style):
    """Tokens are appended one by one (the ring wraps twice); the expected output is written out
    with loops: every selected token takes its key and value from the cache that holds it."""
    rng = np.random.default_rng(17 + style)
    H, H_kv, d, r, r_hi, S, w, theta = 4, 2, 4, 3, 6, 19, 7, 50.0
    D = H_kv * d
    Uk, Uv, Uk_hi, Uv_hi = (_ortho(rng, D, n) for n in (r, r, r_hi, r_hi))
    k_tok, v_tok = rng.standard_normal((S, D)), rng.standard_normal((S, D))
    Kc, Vc = k_tok @ Uk, v_tok @ Uv
    Kw, Vw = np.full((w, r_hi), np.nan), np.full((w, r_hi), np.nan)
    for t in range(S):
        oracle.window_append(Kw, Vw, k_tok[t], v_tok[t], Uk_hi, Uv_hi, t)
    q = rng.standard_normal((H, d))
    # both sides of the window boundary S - w = 12, the newest token, sinks
    idx = np.array([0, 1, 5, 11, 12, 13, 18, 9, 16], dtype=np.int32)
    got = oracle.sparse_attend_window(q, S, Kc, Vc, Uk, Uv, Kw, Vw, Uk_hi, Uv_hi, idx, S, H_kv, theta, style)
    keys, vals = [], []
    for t in idx:
        if t >= S - w:
            kt, vt = Uk_hi @ (Uk_hi.T @ k_tok[t]), Uv_hi @ (Uv_hi.T @ v_tok[t])
        else:
            kt, vt = Uk @ (Uk.T @ k_tok[t]), Uv @ (Uv.T @ v_tok[t])
        keys.append(np.concatenate([_rope(kt[g * d:(g + 1) * d], int(t), theta, style) for g in range(H_kv)]))
        vals.append(vt)
    qR = np.stack([_rope(q[h], S, theta, style) for h in range(H)])
    np.testing.assert_allclose(got, _softmax_attend(qR, keys, vals, H_kv), rtol=0, atol=1e-12)


def test_window_reads_each_token_from_one_cache_only(oracle):
    rng = np.random.default_rng(23)
    H, H_kv, d, r, r_hi, S, w = 2, 1, 8, 4, 6, 12, 4
    D = H_kv * d
    Uk, Uv, Uk_hi, Uv_hi = (_ortho(rng, D, n) for n in (r, r, r_hi, r_hi))
    Kc, Vc = rng.standard_normal((S, r)), rng.standard_normal((S, r))
    Kw, Vw = rng.standard_normal((w, r_hi)), rng.standard_normal((w, r_hi))
    q = rng.standard_normal((H, d))
    idx = np.array([2, 7, 8, 10, 11], dtype=np.int32)   # window = tokens 8..11
    run = lambda: oracle.sparse_attend_window(q, S, Kc, Vc, Uk, Uv, Kw, Vw, Uk_hi, Uv_hi, idx, S, H_kv, 1e4)
    base = run()
    Kc[8:] += 5.0; Vc[8:] -= 3.0           # low-rank rows of window tokens: never read
    np.testing.assert_array_equal(run(), base)
    Kw[9 % w] += 5.0                       # ring row of a token that is not selected
    np.testing.assert_array_equal(run(), base)
    Vw[10 % w] += 1.0                      # ring row of a selected window token
    assert np.abs(run() - base).max() > 1e-3
    Vw[10 % w] -= 1.0
    Kc[7] += 1.0                           # last token outside the window
    assert np.abs(run() - base).max() > 1e-6


def test_window_with_zero_extra_coordinates_is_plain_sparse_attention(oracle):
    """If the window's projectors extend the low-rank ones and the extra coordinates are zero,
    both caches describe the same keys and values."""
    rng = np.random.default_rng(29)
    H, H_kv, d, r, r_hi, S, w = 4, 2, 8, 5, 9, 20, 6
    D = H_kv * d
    Uk_hi, Uv_hi = _ortho(rng, D, r_hi), _ortho(rng, D, r_hi)
    Uk, Uv = Uk_hi[:, :r].copy(), Uv_hi[:, :r].copy()
    Kc, Vc = rng.standard_normal((S, r)), rng.standard_normal((S, r))
    Kw, Vw = np.zeros((w, r_hi)), np.zeros((w, r_hi))
    for t in range(S - w, S):
        Kw[t % w, :r], Vw[t % w, :r] = Kc[t], Vc[t]
    q = rng.standard_normal((H, d))
    idx = np.array([0, 3, 13, 14, 15, 19, 17], dtype=np.int32)
    got = oracle.sparse_attend_window(q, S, Kc, Vc, Uk, Uv, Kw, Vw, Uk_hi, Uv_hi, idx, S, H_kv, 1e4)
    want = oracle.sparse_attend(q, S, Kc, Vc, Uk, Uv, idx, H_kv, 1e4)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_full_rank_window_over_everything_is_dense_attention(oracle):
    """r_hi = D_kv with an orthogonal projector loses nothing: a window that covers the whole
    cache, with every token selected, is dense attention over the original keys and values."""
    rng = np.random.default_rng(31)
    H, H_kv, d, r, S, w, theta = 4, 2, 4, 2, 9, 16, 1e4
    D = H_kv * d
    Uk, Uv = _ortho(rng, D, r), _ortho(rng, D, r)
    Qk, Qv = _ortho(rng, D, D), _ortho(rng, D, D)
    k_tok, v_tok = rng.standard_normal((S, D)), rng.standard_normal((S, D))
    Kw, Vw = np.zeros((w, D)), np.zeros((w, D))
    for t in range(S):
        oracle.window_append(Kw, Vw, k_tok[t], v_tok[t], Qk, Qv, t)
    q = rng.standard_normal((H, d))
    got = oracle.sparse_attend_window(q, S, np.zeros((S, r)), np.zeros((S, r)), Uk, Uv, Kw, Vw, Qk, Qv,
                                      np.arange(S, dtype=np.int32), S, H_kv, theta)
    keys = [np.concatenate([_rope(k_tok[t, g * d:(g + 1) * d], t, theta) for g in range(H_kv)]) for t in range(S)]
    qR = np.stack([_rope(q[h], S, theta) for h in range(H)])
    np.testing.assert_allclose(got, _softmax_attend(qR, keys, list(v_tok), H_kv), rtol=0, atol=1e-12)

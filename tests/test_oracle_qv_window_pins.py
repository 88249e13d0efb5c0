"""Pins of the oracle's recent window over the paper's own cache formats (Sec. 5.1; CPU only): latent keys with a
rank-r_hi ring for the recent tokens, group-quantised values with an 8-bit ring for them.  Everything is
checked against arithmetic written out here (its own RoPE, de-quantisation, softmax and loops), hand-worked
8-bit groups, and special cases that collapse to functions pinned elsewhere."""
import math

import numpy as np
import pytest


def _rope(x, pos, theta, style=0):
    d = x.shape[0]
    out = np.array(x, dtype=np.float64)
    for i in range(d // 2):
        ang = pos * theta ** (-2.0 * i / d)
        a, b = (i, i + d // 2) if style == 0 else (2 * i, 2 * i + 1)
        out[a] = x[a] * math.cos(ang) - x[b] * math.sin(ang)
        out[b] = x[b] * math.cos(ang) + x[a] * math.sin(ang)
    return out


def _ortho(rng, D, n):
    qm, _ = np.linalg.qr(rng.standard_normal((D, n)))
    return qm


def _dequant_row(codes, scale, zero):
    """zero + scale * code, group of 32 channels by group, with plain loops."""
    out = np.zeros(codes.shape[0])
    for c in range(codes.shape[0]):
        out[c] = zero[c // 32] + scale[c // 32] * float(codes[c])
    return out


def _attend(qR, keys, vals, H_kv):
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


def test_eight_bit_groups_hand_worked_and_nearest(oracle):
    # a group already on a 256-point grid: min -4, step 1/32
    k = (np.arange(32) * 37) % 256
    k[0], k[1] = 0, 255                      # the group spans the whole grid
    v = (-4.0 + k / 32.0)[None, :]
    codes, scale, zero = oracle.quantize_values(v, 8, "f32")
    assert scale.tolist() == [[1.0 / 32.0]] and zero.tolist() == [[-4.0]]
    assert codes[0].tolist() == k.tolist()
    np.testing.assert_array_equal(oracle.dequantize_values(codes, scale, zero), v)
    # random rows: the chosen code is a nearest grid point (brute force over all 256), error at most half a step
    rng = np.random.default_rng(3)
    v = rng.standard_normal((20, 64)).astype(np.float32).astype(np.float64)
    codes, scale, zero = oracle.quantize_values(v, 8, "f32")
    g = v.reshape(20, 2, 32)
    grid = zero[..., None, None] + scale[..., None, None] * np.arange(256)[None, None, None, :]
    err = np.abs(g[..., None] - grid)
    chosen = np.take_along_axis(err, codes.reshape(20, 2, 32)[..., None].astype(np.int64), -1)[..., 0]
    assert np.all(chosen <= err.min(axis=-1) + 1e-6 * scale[..., None])
    assert np.all(chosen <= 0.5 * scale[..., None] * (1 + 1e-5))
    assert codes.max() == 255 and codes.min() == 0
    # ties go to the even code: min 0, max 255 -> step 1
    t = np.zeros((1, 32)); t[0, :5] = [0.0, 255.0, 0.5, 1.5, 2.5]
    assert oracle.quantize_values(t, 8, "f32")[0][0, :5].tolist() == [0, 255, 0, 2, 2]


@pytest.mark.parametrize("style", [0, 1])
def test_qv_window_brute_force(oracle, style):
    """Every selected token takes its key and value from the cache that holds it: tokens of the last w positions from
    the ring rows t mod w (rank r_hi keys, 8-bit values), all others from the main caches (rank r keys, 4-bit values)."""
    rng = np.random.default_rng(29 + style)
    H, H_kv, d, r, r_hi, S, w, theta = 4, 2, 32, 5, 11, 23, 6, 100.0
    D = H_kv * d
    Uk, Uk_hi = _ortho(rng, D, r), _ortho(rng, D, r_hi)
    Kc = rng.standard_normal((S, r))
    Kw = rng.standard_normal((w, r_hi))
    codes = rng.integers(0, 16, size=(S, D)).astype(np.uint8)
    scale, zero = 0.1 + rng.random((S, D // 32)), rng.standard_normal((S, D // 32))
    codes_w = rng.integers(0, 256, size=(w, D)).astype(np.uint8)
    scale_w, zero_w = 0.01 + 0.02 * rng.random((w, D // 32)), rng.standard_normal((w, D // 32))
    q = rng.standard_normal((H, d))
    idx = np.array([0, 3, 16, 17, 18, 22, 9, 20], dtype=np.int32)     # window = tokens 17..22
    got = oracle.sparse_attend_qv_window(q, S, Kc, Uk, codes, scale, zero, Kw, Uk_hi, codes_w, scale_w, zero_w, idx, S,
                                         H_kv, theta, style)
    keys, vals = [], []
    for t in idx:
        if t >= S - w:
            kt, vt = Uk_hi @ Kw[t % w], _dequant_row(codes_w[t % w], scale_w[t % w], zero_w[t % w])
        else:
            kt, vt = Uk @ Kc[t], _dequant_row(codes[t], scale[t], zero[t])
        keys.append(np.concatenate([_rope(kt[g * d:(g + 1) * d], int(t), theta, style) for g in range(H_kv)]))
        vals.append(vt)
    qR = np.stack([_rope(q[h], S, theta, style) for h in range(H)])
    np.testing.assert_allclose(got, _attend(qR, keys, vals, H_kv), rtol=0, atol=1e-12)


def test_qv_window_reads_each_token_from_one_cache_only(oracle):
    rng = np.random.default_rng(31)
    H, H_kv, d, r, r_hi, S, w = 2, 1, 32, 4, 6, 12, 4
    D = H_kv * d
    Uk, Uk_hi = _ortho(rng, D, r), _ortho(rng, D, r_hi)
    Kc, Kw = rng.standard_normal((S, r)), rng.standard_normal((w, r_hi))
    codes = rng.integers(0, 4, size=(S, D)).astype(np.uint8)
    scale, zero = np.full((S, 1), 0.5), np.full((S, 1), -1.0)
    codes_w = rng.integers(0, 256, size=(w, D)).astype(np.uint8)
    scale_w, zero_w = np.full((w, 1), 0.01), np.full((w, 1), -1.0)
    q = rng.standard_normal((H, d))
    idx = np.array([2, 7, 8, 10, 11], dtype=np.int32)   # window = tokens 8..11
    run = lambda: oracle.sparse_attend_qv_window(q, S, Kc, Uk, codes, scale, zero, Kw, Uk_hi, codes_w, scale_w, zero_w,
                                                 idx, S, H_kv, 1e4)
    base = run()
    Kc[8:] += 5.0; codes[8:] = 3 - codes[8:]; zero[8:] += 2.0     # main-cache rows of window tokens: never read
    np.testing.assert_array_equal(run(), base)
    codes_w[9 % w] = 255 - codes_w[9 % w]                        # ring row of a token that is not selected
    np.testing.assert_array_equal(run(), base)
    zero_w[10 % w] += 1.0                                        # ring row of a selected window token
    assert np.abs(run() - base).max() > 1e-3
    zero_w[10 % w] -= 1.0
    codes[7] = 3 - codes[7]                                      # last token outside the window
    assert np.abs(run() - base).max() > 1e-6


def test_qv_window_of_width_zero_tokens_is_the_plain_quantised_path(oracle):
    """No selected token inside the window: the result is sparse_attend_qv (pinned on its own) whatever the ring holds."""
    rng = np.random.default_rng(37)
    H, H_kv, d, r, r_hi, S, w = 4, 2, 32, 6, 9, 30, 5
    D = H_kv * d
    Uk, Uk_hi = _ortho(rng, D, r), _ortho(rng, D, r_hi)
    Kc, Kw = rng.standard_normal((S, r)), rng.standard_normal((w, r_hi))
    codes = rng.integers(0, 16, size=(S, D)).astype(np.uint8)
    scale, zero = 0.1 + rng.random((S, D // 32)), rng.standard_normal((S, D // 32))
    codes_w = rng.integers(0, 256, size=(w, D)).astype(np.uint8)
    scale_w, zero_w = rng.random((w, D // 32)), rng.standard_normal((w, D // 32))
    q = rng.standard_normal((H, d))
    idx = np.array([1, 4, 24, 13], dtype=np.int32)      # window = tokens 25..29
    a = oracle.sparse_attend_qv_window(q, S + 2, Kc, Uk, codes, scale, zero, Kw, Uk_hi, codes_w, scale_w, zero_w, idx, S,
                                       H_kv, 1e4, 1)
    b = oracle.sparse_attend_qv(q, S + 2, Kc, Uk, codes, scale, zero, idx, H_kv, 1e4, 1)
    np.testing.assert_array_equal(a, b)

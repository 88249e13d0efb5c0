"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test ties one oracle function to what the paper (arXiv 2510.24273) and
the mathematics fix: hand-worked values, closed forms, invariants, special
cases that reduce to a textbook definition, and brute force on tiny inputs.
The dense-attention brute force below is written independently of the oracle
(complex-number RoPE, explicit loops over tokens) on purpose.
"""
import itertools
import math
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------------------
# independent brute force: dense RoPE attention over ALL tokens
# ---------------------------------------------------------------------------

def _rope_complex(x, pos, theta):
    """Half-split RoPE written with complex numbers: (x_i + i x_{i+d/2}) e^{i pos f_i}."""
    d = x.shape[-1]
    f = theta ** (-2.0 * np.arange(d // 2) / d)
    z = (x[..., : d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * pos * f)
    return np.concatenate([z.real, z.imag], axis=-1)


def dense_rope_attention(q, K, V, q_pos, theta):
    """q [H,d]; K,V [S,H_kv,d] full-rank pre-RoPE keys/values -> y [H,d]."""
    H, d = q.shape
    S, H_kv, _ = K.shape
    G = H // H_kv
    y = np.zeros((H, d))
    for h in range(H):
        g = h // G
        qr = _rope_complex(q[h], q_pos, theta)
        logit = np.array([qr @ _rope_complex(K[t, g], t, theta) for t in range(S)]) / math.sqrt(d)
        w = np.exp(logit - logit.max())
        w /= w.sum()
        for t in range(S):
            y[h] += w[t] * V[t, g]
    return y


def _orthogonal(rng, n):
    qm, _ = np.linalg.qr(rng.standard_normal((n, n)))
    return qm


# ---------------------------------------------------------------------------
# (i) whole path: k = S with a full-rank orthogonal projector is dense attention
#     (Eq. 2 with U U^T = I, and Eq. 5 with C = all tokens)
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("H,H_kv", [(4, 4), (4, 2), (6, 1)])
def test_full_rank_all_tokens_equals_dense_attention(oracle, H, H_kv):
    rng = np.random.default_rng(7)
    d, S = 8, 13
    D = H_kv * d
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((S, H_kv, d))
    V = rng.standard_normal((S, H_kv, d))
    Uk, Uv = _orthogonal(rng, D), _orthogonal(rng, D)
    Kc = K.reshape(S, D) @ Uk            # Eq. 1: K~ = K U
    Vc = V.reshape(S, D) @ Uv
    out = oracle.decode_step(q, S, Kc, Vc, Uk, Uv, H_kv, top_k=S, theta=10000.0)
    want = dense_rope_attention(q, K, V, S, 10000.0)
    assert sorted(out["idx"].tolist()) == list(range(S))
    np.testing.assert_allclose(out["y"], want, atol=1e-10, rtol=0)
    # a query placed on the last cached position (self-attention row of Alg. 1)
    out2 = oracle.decode_step(q, S - 1, Kc, Vc, Uk, Uv, H_kv, top_k=S + 5, theta=500000.0)
    np.testing.assert_allclose(out2["y"], dense_rope_attention(q, K, V, S - 1, 500000.0),
                               atol=1e-10, rtol=0)


def test_sparse_subset_equals_dense_attention_on_that_subset(oracle):
    """Eq. 5: attention restricted to C is dense attention over the rows of C."""
    rng = np.random.default_rng(8)
    H, H_kv, d, S = 4, 2, 8, 20
    D = H_kv * d
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((S, H_kv, d))
    V = rng.standard_normal((S, H_kv, d))
    Uk, Uv = _orthogonal(rng, D), _orthogonal(rng, D)
    C = np.array([17, 3, 4, 11, 0], dtype=np.int32)
    y = oracle.sparse_attend(q, 25, K.reshape(S, D) @ Uk, V.reshape(S, D) @ Uv, Uk, Uv, C,
                             H_kv, 10000.0)
    # brute force with positions of the selected tokens
    want = np.zeros((H, d))
    for h in range(H):
        g = h // (H // H_kv)
        qr = _rope_complex(q[h], 25, 10000.0)
        lg = np.array([qr @ _rope_complex(K[t, g], t, 10000.0) for t in C]) / math.sqrt(d)
        w = np.exp(lg - lg.max())
        w /= w.sum()
        want[h] = sum(w[m] * V[t, g] for m, t in enumerate(C))
    np.testing.assert_allclose(y, want, atol=1e-12, rtol=0)


# ---------------------------------------------------------------------------
# (ii) projection + latent scores
# ---------------------------------------------------------------------------

def test_project_hand_example(oracle):
    U = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])      # [D=3, r=2]
    np.testing.assert_array_equal(oracle.project([1.0, 10.0, 100.0], U), [531.0, 642.0])


def test_group_sum_hand_example(oracle):
    q = np.arange(12, dtype=float).reshape(6, 2)            # H=6, d=2
    np.testing.assert_array_equal(oracle.group_sum(q, 6), q)
    np.testing.assert_array_equal(oracle.group_sum(q, 2),
                                  [[0 + 2 + 4, 1 + 3 + 5], [6 + 8 + 10, 7 + 9 + 11]])
    np.testing.assert_array_equal(oracle.group_sum(q, 3), [[2, 4], [10, 12], [18, 20]])


def test_scores_hand_example_and_truncation(oracle):
    Kc = np.array([[1.0, 2.0, 3.0], [0.5, -1.0, 4.0]])
    qt = np.array([2.0, 10.0, 100.0])
    np.testing.assert_array_equal(oracle.scores(qt, Kc), [322.0, 391.0])
    np.testing.assert_array_equal(oracle.scores(qt, Kc, r_score=2), [22.0, -9.0])   # r* = 2
    np.testing.assert_array_equal(oracle.scores(qt, Kc, r_score=1), [2.0, 1.0])


@pytest.mark.parametrize("H,H_kv", [(4, 4), (8, 2)])
def test_full_rank_scores_equal_sum_of_head_dot_products(oracle, H, H_kv):
    """Eq. 2: with U U^T = I the latent score is sum_h q_h . k_{g(h)} on pre-RoPE vectors."""
    rng = np.random.default_rng(3)
    d, S = 4, 9
    D = H_kv * d
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((S, H_kv, d))
    U = _orthogonal(rng, D)
    qt = oracle.project(oracle.group_sum(q, H_kv), U)
    s = oracle.scores(qt, K.reshape(S, D) @ U)
    want = [sum(q[h] @ K[t, h // (H // H_kv)] for h in range(H)) for t in range(S)]
    np.testing.assert_allclose(s, want, atol=1e-11, rtol=0)


def test_low_rank_scores_equal_dot_with_reconstructed_keys(oracle):
    """q^T U U^T k = q^T (U k~): holds for ANY U when r* = r."""
    rng = np.random.default_rng(4)
    H, H_kv, d, r, S = 8, 2, 4, 5, 11
    D = H_kv * d
    q = rng.standard_normal((H, d))
    U = rng.standard_normal((D, r))                         # not orthonormal on purpose
    Kc = rng.standard_normal((S, r))
    s = oracle.scores(oracle.project(oracle.group_sum(q, H_kv), U), Kc)
    KC = oracle.reconstruct(Kc, np.arange(S), U).reshape(S, H_kv, d)
    want = [sum(q[h] @ KC[t, h // 4] for h in range(H)) for t in range(S)]
    np.testing.assert_allclose(s, want, atol=1e-11, rtol=0)


# ---------------------------------------------------------------------------
# (iii) selection
# ---------------------------------------------------------------------------

def _exhaustive_topk(s, k):
    order = sorted(range(len(s)), key=lambda j: (-s[j], j))
    return order[:k]


@pytest.mark.parametrize("seed", range(6))
def test_topk_matches_exhaustive_sort_with_ties(oracle, seed):
    rng = np.random.default_rng(seed)
    S = int(rng.integers(1, 65))
    s = rng.integers(-4, 5, size=S).astype(float) if seed % 2 else rng.standard_normal(S)
    for k in (1, 2, S // 2, S - 1, S, S + 3):
        if k < 1:
            continue
        got = oracle.topk(s, k)
        if k >= S:
            assert got.tolist() == list(range(S))
        else:
            assert got.tolist() == _exhaustive_topk(s, k)       # order too: score desc, idx asc


def test_topk_brute_force_subsets(oracle):
    """On a tiny input the selected set maximises the score sum over all k-subsets."""
    s = np.array([0.3, -1.0, 2.5, 0.31, 2.4, -0.2, 0.0])
    for k in range(1, 7):
        best = max(itertools.combinations(range(7), k), key=lambda c: sum(s[list(c)]))
        assert sorted(oracle.topk(s, k).tolist()) == sorted(best)


def test_topk_sink_critical_recent_composition(oracle):
    """Sec. 5.2: x=16 sink + y=432 critical + z=64 recent = 512 tokens."""
    rng = np.random.default_rng(5)
    S = 4096
    s = rng.standard_normal(S)
    s[:16] = 100.0        # sinks and window carry the largest scores: they must not
    s[-64:] = 100.0       # consume the critical budget
    idx = oracle.topk(s, 432, n_sink=16, n_recent=64)
    assert len(idx) == 512 and len(set(idx.tolist())) == 512
    assert idx[:16].tolist() == list(range(16))
    assert idx[-64:].tolist() == list(range(S - 64, S))
    mid = s[16:S - 64]
    assert sorted(idx[16:16 + 432].tolist()) == sorted((np.argsort(-mid, kind="stable")[:432] + 16).tolist())
    # short cache: everything is selected, once
    assert oracle.topk(s[:500], 432, 16, 64).tolist() == list(range(500))
    assert oracle.topk(s[:512], 432, 16, 64).tolist() == list(range(512))
    assert len(oracle.topk(s[:513], 432, 16, 64)) == 512


# ---------------------------------------------------------------------------
# reconstruction
# ---------------------------------------------------------------------------

def test_reconstruct_rank_one_hand_example(oracle):
    U = np.array([[2.0], [-1.0], [0.5]])                    # D=3, r=1
    Kc = np.array([[1.0], [4.0], [-2.0]])
    got = oracle.reconstruct(Kc, np.array([2, 0], dtype=np.int32), U)
    np.testing.assert_array_equal(got, [[-4.0, 2.0, -1.0], [2.0, -1.0, 0.5]])


def test_reconstruct_then_project_is_identity_for_orthonormal_columns(oracle):
    rng = np.random.default_rng(6)
    D, r, S = 24, 7, 5
    U, _ = np.linalg.qr(rng.standard_normal((D, r)))
    Kc = rng.standard_normal((S, r))
    X = oracle.reconstruct(Kc, np.arange(S), U)
    for t in range(S):
        np.testing.assert_allclose(oracle.project(X[t], U), Kc[t], atol=1e-13, rtol=0)
    # and against the definition written with a different routine
    np.testing.assert_allclose(X, np.einsum("tr,cr->tc", Kc, U), atol=1e-13, rtol=0)


# ---------------------------------------------------------------------------
# RoPE
# ---------------------------------------------------------------------------

def test_rope_d2_is_textbook_rotation(oracle):
    x = np.array([[[1.0, 0.0]], [[0.0, 1.0]]])              # [n_pos=2, m=1, d=2]
    got = oracle.rope(x, [1, 3], 10000.0)
    np.testing.assert_allclose(got[0, 0], [math.cos(1), math.sin(1)], atol=1e-15)
    np.testing.assert_allclose(got[1, 0], [-math.sin(3), math.cos(3)], atol=1e-15)


def test_rope_frequencies_and_pairing(oracle):
    # d=4: pair 0 turns by pos*1, pair 1 by pos*theta^(-1/2); theta=1e4, pos=100 -> 100 and 1 rad
    x = np.array([[[1.0, 2.0, 0.0, 0.0]]])
    half = oracle.rope(x, [100], 10000.0, style=0)[0, 0]
    np.testing.assert_allclose(half, [math.cos(100), 2 * math.cos(1), math.sin(100), 2 * math.sin(1)],
                               atol=1e-13)
    y = np.array([[[1.0, 0.0, 2.0, 0.0]]])
    inter = oracle.rope(y, [100], 10000.0, style=1)[0, 0]
    np.testing.assert_allclose(inter, [math.cos(100), math.sin(100), 2 * math.cos(1), 2 * math.sin(1)],
                               atol=1e-13)


def test_rope_invariants(oracle):
    rng = np.random.default_rng(9)
    d = 16
    x = rng.standard_normal((5, 3, d))
    pos = np.array([0, 1, 77, 4096, 131071])
    for style in (0, 1):
        y = oracle.rope(x, pos, 500000.0, style)
        np.testing.assert_array_equal(y[0], x[0])                       # position 0: identity
        np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1),
                                   rtol=1e-13)                          # rotations keep norms
    np.testing.assert_allclose(oracle.rope(x, pos, 10000.0, 0), _rope_complex(x, pos[:, None, None], 10000.0),
                               atol=1e-10)
    # relative property: <RoPE(q,m), RoPE(k,n)> depends on m-n only
    q, k = rng.standard_normal((1, 1, d)), rng.standard_normal((1, 1, d))
    a = oracle.rope(q, [10], 1e4)[0, 0] @ oracle.rope(k, [3], 1e4)[0, 0]
    b = oracle.rope(q, [1010], 1e4)[0, 0] @ oracle.rope(k, [1003], 1e4)[0, 0]
    assert abs(a - b) < 1e-11


def test_output_invariant_under_common_position_shift(oracle):
    """Shifting the query and token positions alike leaves y unchanged: emulate by
    prepending never-selected rows to the cache."""
    rng = np.random.default_rng(10)
    H, H_kv, d, r, S, pad = 4, 2, 8, 6, 10, 37
    D = H_kv * d
    q = rng.standard_normal((H, d))
    Uk, Uv = rng.standard_normal((D, r)), rng.standard_normal((D, r))
    Kc, Vc = rng.standard_normal((S, r)), rng.standard_normal((S, r))
    C = np.array([1, 4, 9, 6], dtype=np.int32)
    y0 = oracle.sparse_attend(q, S, Kc, Vc, Uk, Uv, C, H_kv, 1e4)
    z = np.zeros((pad, r))
    y1 = oracle.sparse_attend(q, S + pad, np.vstack([z, Kc]), np.vstack([z, Vc]), Uk, Uv, C + pad,
                              H_kv, 1e4)
    np.testing.assert_allclose(y0, y1, atol=1e-11, rtol=0)


# ---------------------------------------------------------------------------
# softmax attention
# ---------------------------------------------------------------------------

def test_attend_special_cases(oracle):
    rng = np.random.default_rng(11)
    H, H_kv, d, n = 4, 2, 8, 6
    qR = rng.standard_normal((H, d))
    KR = rng.standard_normal((n, H_kv, d))
    V = rng.standard_normal((n, H_kv, d))
    y, p = oracle.attend(qR, KR, V, return_p=True)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-14)           # softmax sums to one
    perm = rng.permutation(n)
    np.testing.assert_allclose(oracle.attend(qR, KR[perm], V[perm]), y, atol=1e-14)
    # equal logits -> plain mean of the values of the head's KV group
    y_eq = oracle.attend(np.zeros((H, d)), KR, V)
    for h in range(H):
        np.testing.assert_allclose(y_eq[h], V[:, h // 2].mean(axis=0), atol=1e-15)
    # one selected token -> its value
    y_one = oracle.attend(qR, KR[:1], V[:1])
    for h in range(H):
        np.testing.assert_array_equal(y_one[h], V[0, h // 2])
    # logits use 1/sqrt(d) with the HEAD width: two tokens, closed form
    q1 = np.zeros((1, 4)); q1[0, 0] = 2.0
    K2 = np.zeros((2, 1, 4)); K2[0, 0, 0] = 3.0
    V2 = np.zeros((2, 1, 4)); V2[0, 0, 1] = 1.0
    w = math.exp(2.0 * 3.0 / 2.0) / (math.exp(3.0) + 1.0)
    np.testing.assert_allclose(oracle.attend(q1, K2, V2)[0], [0, w, 0, 0], atol=1e-15)
    # huge logits (2000 vs 1998) must not overflow: p = 1/(1+e^-2)
    K3 = np.zeros((2, 1, 4)); K3[0, 0, 0] = 2000.0; K3[1, 0, 0] = 1998.0
    np.testing.assert_allclose(oracle.attend(q1, K3, V2)[0], [0, 1 / (1 + math.exp(-2.0)), 0, 0],
                               atol=1e-15)


def test_value_path_associativity(oracle):
    """y[h] = (p_h . V~_C) U_v[block g(h)]^T : the same sum in another order."""
    rng = np.random.default_rng(12)
    H, H_kv, d, r, S = 4, 2, 8, 5, 9
    D = H_kv * d
    Uv = rng.standard_normal((D, r))
    Vc = rng.standard_normal((S, r))
    C = np.array([8, 2, 5], dtype=np.int32)
    VC = oracle.reconstruct(Vc, C, Uv).reshape(len(C), H_kv, d)
    qR = rng.standard_normal((H, d))
    KR = rng.standard_normal((len(C), H_kv, d))
    y, p = oracle.attend(qR, KR, VC, return_p=True)
    for h in range(H):
        g = h // 2
        t = p[h] @ Vc[C]                                   # [r]
        np.testing.assert_allclose(y[h], Uv[g * d:(g + 1) * d] @ t, atol=1e-13)


# ---------------------------------------------------------------------------
# composition and the synthetic workloads
# ---------------------------------------------------------------------------

def test_decode_step_is_the_chain_of_steps(oracle):
    rng = np.random.default_rng(13)
    H, H_kv, d, r, S, k = 8, 4, 8, 12, 50, 7
    D = H_kv * d
    q = rng.standard_normal((H, d))
    Uk, Uv = rng.standard_normal((D, r)), rng.standard_normal((D, r))
    Kc, Vc = rng.standard_normal((S, r)), rng.standard_normal((S, r))
    out = oracle.decode_step(q, S, Kc, Vc, Uk, Uv, H_kv, k, 1e4, r_score=6, n_sink=2, n_recent=3)
    qt = oracle.project(oracle.group_sum(q, H_kv), Uk)
    s = oracle.scores(qt, Kc, 6)
    idx = oracle.topk(s, k, 2, 3)
    KC = oracle.rope(oracle.reconstruct(Kc, idx, Uk).reshape(len(idx), H_kv, d), idx, 1e4)
    VC = oracle.reconstruct(Vc, idx, Uv).reshape(len(idx), H_kv, d)
    y = oracle.attend(oracle.rope(q[None], [S], 1e4)[0], KC, VC)
    np.testing.assert_array_equal(out["qt"], qt)
    np.testing.assert_array_equal(out["s"], s)
    np.testing.assert_array_equal(out["idx"], idx)
    np.testing.assert_array_equal(out["y"], y)
    assert len(idx) == 12


def test_planted_tokens_are_selected(oracle):
    from paper_2510_24273_amd import synth
    w = synth.shrink(synth.CONFIGS["cfg2"], S=512, H=8, H_kv=8, d=16, r=48, top_k=32)
    L = synth.make_layer(w, layer=3)
    wd = synth.widen
    out = oracle.decode_step(wd(L["q"][0]), w.S, wd(L["Kc"][0]), wd(L["Vc"][0]), wd(L["Uk"]),
                             wd(L["Uv"]), w.H_kv, w.top_k, w.theta)
    assert len(L["planted"][0]) == 3
    assert set(L["planted"][0].tolist()) <= set(out["idx"].tolist())
    # the three planted rows hold the three largest scores
    assert set(np.argsort(-out["s"])[:3].tolist()) == set(L["planted"][0].tolist())


def test_dense_decode_matches_brute_force(oracle):
    """The dense baseline over a cache of rotated keys equals dense RoPE attention written with
    complex rotations on the pre-RoPE keys (GQA, odd length)."""
    rng = np.random.default_rng(33)
    H, H_kv, d, S, theta = 6, 2, 16, 23, 1e4
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((S, H_kv, d))
    V = rng.standard_normal((S, H_kv, d))
    KR = np.stack([_rope_complex(K[t], t, theta) for t in range(S)])
    y = oracle.dense_decode(q, S + 3, KR, V, theta)
    np.testing.assert_allclose(y, dense_rope_attention(q, K, V, S + 3, theta), rtol=0, atol=1e-12)
    assert not oracle.dense_decode(q, 0, KR[:0], V[:0], theta).any()


def test_traffic_model_fixture():
    """Sec. 4.5: full attention moves 2sd, SALS s r* + 2kr; the printed speed-up range
    7.69x..14.28x is the reciprocal of Table 2's memory-access column 0.13 / 0.07."""
    from paper_2510_24273_amd import roofline
    rows = {}
    with open(os.path.join(GOLDEN, "traffic_model.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split()
                rows[key] = float(val)
    assert abs(1.0 / rows["memory_access_sals25"] - rows["speedup_low"]) < 0.01
    assert abs(1.0 / rows["memory_access_sals12p5"] - rows["speedup_high"]) < 0.01
    # the closed form 1/(d_r*/2 + d_r k_s) equals 2sd/(s r* + 2 k r)
    s, nd = 4096, 4096
    for d_r, k_s in ((0.25, 0.25), (0.125, 0.125)):
        r, k = int(d_r * nd), int(k_s * s)
        model = roofline.paper_traffic_elements(s, r, r // 2, k)
        assert model == s * (r // 2) + 2 * k * r
        assert abs(2 * s * nd / model - 1.0 / ((r / 2 / nd) / 2 + d_r * k_s)) < 1e-12


# ---------------------------------------------------------------------------
# interleaved RoPE pairing (pairs (2i, 2i+1)) through the composed functions:
# brute force written here with explicit 2x2 rotations, independent of oracle.rope
# ---------------------------------------------------------------------------

def _rope_interleaved(x, pos, theta):
    """Pairs (2i, 2i+1), angle pos * theta^(-2i/d), as a plain 2x2 rotation per pair."""
    d = x.shape[-1]
    y = np.array(x, dtype=np.float64, copy=True)
    for i in range(d // 2):
        ang = pos * theta ** (-2.0 * i / d)
        c, s = math.cos(ang), math.sin(ang)
        a, b = x[..., 2 * i], x[..., 2 * i + 1]
        y[..., 2 * i] = a * c - b * s
        y[..., 2 * i + 1] = b * c + a * s
    return y


def _attention_interleaved(q, K, V, tokens, q_pos, theta, rotate_keys=True):
    """Softmax attention of q [H,d] over the rows `tokens` of K, V [S,H_kv,d] (keys rotated here
    unless they already are), interleaved pairing, 1/sqrt(d) scaling."""
    H, d = q.shape
    G = H // K.shape[1]
    y = np.zeros((H, d))
    for h in range(H):
        g = h // G
        qr = _rope_interleaved(q[h], q_pos, theta)
        lg = np.array([qr @ (_rope_interleaved(K[t, g], int(t), theta) if rotate_keys else K[t, g])
                       for t in tokens]) / math.sqrt(d)
        w = np.exp(lg - lg.max())
        w /= w.sum()
        for m, t in enumerate(tokens):
            y[h] += w[m] * V[t, g]
    return y


@pytest.mark.parametrize("H,H_kv", [(4, 4), (6, 2)])
def test_interleaved_rope_through_sparse_attend_and_decode_step(oracle, H, H_kv):
    rng = np.random.default_rng(31 + H)
    d, S, theta = 8, 15, 500000.0
    D = H_kv * d
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((S, H_kv, d))
    V = rng.standard_normal((S, H_kv, d))
    Uk, Uv = _orthogonal(rng, D), _orthogonal(rng, D)
    Kc, Vc = K.reshape(S, D) @ Uk, V.reshape(S, D) @ Uv
    C = np.array([12, 0, 7, 3, 14, 9], dtype=np.int32)
    y = oracle.sparse_attend(q, 21, Kc, Vc, Uk, Uv, C, H_kv, theta, 1)
    np.testing.assert_allclose(y, _attention_interleaved(q, K, V, C, 21, theta), atol=1e-11, rtol=0)
    # the two pairings are different functions of the same inputs: a swapped flag must show
    assert np.max(np.abs(y - oracle.sparse_attend(q, 21, Kc, Vc, Uk, Uv, C, H_kv, theta, 0))) > 1e-3
    out = oracle.decode_step(q, S, Kc, Vc, Uk, Uv, H_kv, top_k=S, theta=theta, rope_style=1)
    assert sorted(out["idx"].tolist()) == list(range(S))
    np.testing.assert_allclose(out["y"], _attention_interleaved(q, K, V, range(S), S, theta), atol=1e-11, rtol=0)
    # a proper subset chosen by the scores (which do not depend on the pairing) with sink and recent tokens
    out2 = oracle.decode_step(q, S, Kc, Vc, Uk, Uv, H_kv, top_k=4, theta=theta, n_sink=1, n_recent=2, rope_style=1)
    assert len(out2["idx"]) == 7
    np.testing.assert_allclose(out2["y"], _attention_interleaved(q, K, V, out2["idx"], S, theta), atol=1e-11, rtol=0)


def test_interleaved_rope_through_quantised_values_and_dense_decode(oracle):
    rng = np.random.default_rng(41)
    H, H_kv, d, S, theta = 4, 2, 32, 11, 10000.0    # d = 32: one quantisation group per head
    D = H_kv * d
    q = rng.standard_normal((H, d))
    K = rng.standard_normal((S, H_kv, d))
    Uk = _orthogonal(rng, D)
    Kc = K.reshape(S, D) @ Uk
    # values that lie on a 4-bit grid survive quantisation exactly: zero + scale * code
    codes = rng.integers(0, 16, size=(S, D)).astype(np.uint8)
    scale = 0.25 * np.ones((S, D // 32))
    zero = -1.5 * np.ones((S, D // 32))
    V = (zero.repeat(32, axis=1) + scale.repeat(32, axis=1) * codes).reshape(S, H_kv, d)
    C = np.array([10, 2, 5, 6], dtype=np.int32)
    y = oracle.sparse_attend_qv(q, 13, Kc, Uk, codes, scale, zero, C, H_kv, theta, 1)
    np.testing.assert_allclose(y, _attention_interleaved(q, K, V, C, 13, theta), atol=1e-11, rtol=0)
    # dense baseline: the cache holds keys already rotated at their positions
    KR = np.stack([_rope_interleaved(K[t], t, theta) for t in range(S)])
    y_d = oracle.dense_decode(q, S, KR, V, theta, 1)
    np.testing.assert_allclose(y_d, _attention_interleaved(q, KR, V, range(S), S, theta, rotate_keys=False),
                               atol=1e-11, rtol=0)
    assert np.max(np.abs(y_d - oracle.dense_decode(q, S, KR, V, theta, 0))) > 1e-3

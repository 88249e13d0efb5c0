"""ctypes/numpy wrapper of the fp64 SALS oracle (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It imports nothing from the HIP package.

Every function takes and returns float64 numpy arrays (int32 for indices) and
forwards to the plain C implementation in ``sals_oracle.c``, one call per step
of Algorithm 1 of the paper (arXiv 2510.24273).  The quantised value cache of
Sec. 5.1 (quantise, de-quantise, byte packing, attention over it) is plain
numpy further down; its pins are in ``tests/test_oracle_qv_pins.py``.  The dense
baseline, the overlap score of Sec. 3.2 and the recent window of Sec. 5.1 follow,
composed from the same C steps; their pins are in ``tests/test_oracle_window_pins.py``
and, with those of everything else, in ``tests/test_oracle_pins.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sals_oracle.c")
_LIB = os.path.join(_HERE, "libsals_oracle.so")

_f64p = ctypes.POINTER(ctypes.c_double)
_i32p = ctypes.POINTER(ctypes.c_int32)
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over rows, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.sals_oracle_num_threads.restype = ctypes.c_int
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_f64p)


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(_i32p)


def num_threads() -> int:
    return int(_load().sals_oracle_num_threads())


def group_sum(q, H_kv):
    """q [H,d] -> q_sum [H_kv,d]: sum of the query heads sharing each KV head."""
    q, qp = _d(q)
    H, d = q.shape
    out = np.empty((H_kv, d), dtype=np.float64)
    _load().sals_oracle_group_sum(qp, H, H_kv, d, out.ctypes.data_as(_f64p))
    return out


def project(x, U):
    """x [D], U [D,r] -> U^T x [r]  (Sec. 4.3)."""
    x, xp = _d(np.reshape(x, -1))
    U, Up = _d(U)
    D, r = U.shape
    assert x.shape[0] == D
    out = np.empty(r, dtype=np.float64)
    _load().sals_oracle_project(xp, Up, D, r, out.ctypes.data_as(_f64p))
    return out


def scores(qt, Kc, r_score=None):
    """qt [r], Kc [S,r] -> s [S], s_j = qt[:r*] . Kc[j,:r*]  (Sec. 4.3)."""
    qt, qp = _d(qt)
    Kc, Kp = _d(Kc)
    S, r = Kc.shape
    r_score = r if r_score is None else int(r_score)
    assert 1 <= r_score <= r and qt.shape[0] == r
    out = np.empty(S, dtype=np.float64)
    _load().sals_oracle_scores(qp, Kp, S, r, r_score, out.ctypes.data_as(_f64p))
    return out


def topk(s, top_k, n_sink=0, n_recent=0):
    """s [S] -> selected indices (sinks, critical by decreasing score, recent)."""
    s, sp = _d(s)
    S = s.shape[0]
    idx = np.empty(max(1, top_k + n_sink + n_recent, ), dtype=np.int32)
    if S <= top_k + n_sink + n_recent:
        idx = np.empty(max(1, S), dtype=np.int32)
    n = _load().sals_oracle_topk(sp, S, int(top_k), int(n_sink), int(n_recent),
                                 idx.ctypes.data_as(_i32p))
    return idx[:n].copy()


def reconstruct(Xc, idx, U):
    """Xc [S,r], idx [n], U [D,r] -> Xc[idx] U^T  [n,D]  (Algorithm 1, reconstruction)."""
    Xc, Xp = _d(Xc)
    idx, ip = _i(idx)
    U, Up = _d(U)
    D, r = U.shape
    assert Xc.shape[1] == r
    n = idx.shape[0]
    assert n == 0 or (idx.min() >= 0 and idx.max() < Xc.shape[0])
    out = np.empty((n, D), dtype=np.float64)
    _load().sals_oracle_reconstruct(Xp, ip, n, Up, D, r, out.ctypes.data_as(_f64p))
    return out


def rope(x, pos, theta, style=0):
    """x [..., n_pos, m, d] rotated at pos [n_pos] (m vectors share a position)."""
    x = np.array(x, dtype=np.float64, order="C", copy=True)
    pos, pp = _i(np.reshape(pos, -1))
    d = x.shape[-1]
    n_vec = x.size // d
    assert n_vec % max(1, pos.shape[0]) == 0
    vec_per_pos = n_vec // pos.shape[0] if pos.shape[0] else 1
    _load().sals_oracle_rope(x.ctypes.data_as(_f64p), n_vec, d, pp, vec_per_pos,
                             ctypes.c_double(theta), int(style))
    return x


def attend(qR, KR, V, return_p=False):
    """qR [H,d], KR,V [n,H_kv,d] -> y [H,d] (and p [H,n])  (Eq. 5)."""
    qR, qp = _d(qR)
    KR, Kp = _d(KR)
    V, Vp = _d(V)
    H, d = qR.shape
    n, H_kv, _ = KR.shape
    y = np.empty((H, d), dtype=np.float64)
    p = np.empty((H, n), dtype=np.float64) if return_p else None
    _load().sals_oracle_attend(qp, Kp, Vp, n, H, H_kv, d, y.ctypes.data_as(_f64p),
                               p.ctypes.data_as(_f64p) if return_p else None)
    return (y, p) if return_p else y


def sparse_attend(q, q_pos, Kc, Vc, Uk, Uv, idx, H_kv, theta, rope_style=0):
    """Algorithm 1 from the reconstruction step on, for a given selected set."""
    q, qp = _d(q)
    Kc, Kp = _d(Kc)
    Vc, Vp = _d(Vc)
    Uk, Ukp = _d(Uk)
    Uv, Uvp = _d(Uv)
    idx, ip = _i(idx)
    H, d = q.shape
    r = Kc.shape[1]
    assert Uk.shape == (H_kv * d, r) and Uv.shape == (H_kv * d, r) and Vc.shape == Kc.shape
    y = np.empty((H, d), dtype=np.float64)
    _load().sals_oracle_sparse_attend(qp, int(q_pos), Kp, Vp, Ukp, Uvp, ip, idx.shape[0], H,
                                      H_kv, d, r, ctypes.c_double(theta), int(rope_style),
                                      y.ctypes.data_as(_f64p))
    return y


def decode_step(q, q_pos, Kc, Vc, Uk, Uv, H_kv, top_k, theta, r_score=None, n_sink=0,
                n_recent=0, rope_style=0):
    """Whole Algorithm 1 for one sequence.  Returns dict(y, qt, s, idx)."""
    q, qp = _d(q)
    Kc, Kp = _d(Kc)
    Vc, Vp = _d(Vc)
    Uk, Ukp = _d(Uk)
    Uv, Uvp = _d(Uv)
    H, d = q.shape
    S, r = Kc.shape
    r_score = r if r_score is None else int(r_score)
    k_tot = top_k + n_sink + n_recent
    y = np.empty((H, d), dtype=np.float64)
    qt = np.empty(r, dtype=np.float64)
    s = np.empty(max(S, 1), dtype=np.float64)
    idx = np.empty(max(k_tot, S if S <= k_tot else 0, 1), dtype=np.int32)
    n_sel = ctypes.c_int32(0)
    _load().sals_oracle_decode_step(qp, int(q_pos), Kp, Vp, Ukp, Uvp, S, H, H_kv, d, r,
                                    r_score, int(top_k), int(n_sink), int(n_recent),
                                    ctypes.c_double(theta), int(rope_style),
                                    y.ctypes.data_as(_f64p), qt.ctypes.data_as(_f64p),
                                    s.ctypes.data_as(_f64p), idx.ctypes.data_as(_i32p),
                                    ctypes.byref(n_sel))
    return {"y": y, "qt": qt, "s": s[:S], "idx": idx[: n_sel.value].copy()}


# ---------------------------------------------------------------------------
# Quantised full-rank value cache (Sec. 5.1: values are not projected; they are
# stored with channel-wise group quantisation, 4 bit at the 25 % setting and
# 2 bit at 12.5 %, following KIVI's asymmetric uniform scheme; Algorithm 1's
# V-hat).  Plain numpy.  Reading taken where the paper is silent: a token's
# D_kv channels are cut into groups of 32 consecutive channels; a group stores
# its minimum (zero point) and step (scale) in the storage type and one
# unsigned code per channel:
#     scale = (max - min) / (2^bits - 1),  code = round((v - min) / scale),
#     v^    = min + scale * code.
# The code is an integer decided by floating point, so it is decided in the
# precision the kernels use: float32, IEEE subtraction and division, ties to
# even, with the *stored* (rounded) scale.  Everything downstream is float64.
# ---------------------------------------------------------------------------
QV_GROUP = 32


def _round_to_storage(x32, dtype):
    """float32 array -> nearest value of the storage type, returned as float32."""
    x32 = np.ascontiguousarray(x32, dtype=np.float32)
    if dtype == "f32":
        return x32
    assert dtype == "bf16"
    u = x32.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return u.view(np.float32)


def quantize_values(v, bits, dtype):
    """v [n, D] (values exact in the storage type `dtype`) -> (codes uint8 [n, D],
    scale float64 [n, D/32], zero float64 [n, D/32]); scale and zero are exact in `dtype`."""
    v32 = np.ascontiguousarray(v, dtype=np.float32)
    n, D = v32.shape
    assert D % QV_GROUP == 0 and bits in (2, 4, 8)   # 8: the recent window's rows (Sec. 5.1: half the size of 16-bit values)
    levels = np.float32((1 << bits) - 1)
    g = v32.reshape(n, D // QV_GROUP, QV_GROUP)
    mn, mx = g.min(axis=-1), g.max(axis=-1)
    scale = _round_to_storage((mx - mn) / levels, dtype)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.rint((g - mn[..., None]) / scale[..., None])
    t = np.where(scale[..., None] > 0, t, np.float32(0))
    codes = np.clip(t, 0, levels).astype(np.uint8).reshape(n, D)
    return codes, scale.astype(np.float64), mn.astype(np.float64)


def dequantize_values(codes, scale, zero):
    """codes [n, D], scale / zero [n, D/32] -> v^ [n, D] = zero + scale * code (float64)."""
    codes = np.asarray(codes)
    n, D = codes.shape
    c = codes.astype(np.float64).reshape(n, D // QV_GROUP, QV_GROUP)
    return (np.asarray(zero, dtype=np.float64)[..., None]
            + np.asarray(scale, dtype=np.float64)[..., None] * c).reshape(n, D)


def pack_codes(codes, bits):
    """codes [n, D] -> bytes [n, D*bits/8]: channel c sits in byte c*bits/8 at bit (c*bits) % 8."""
    codes = np.asarray(codes, dtype=np.uint8)
    per = 8 // bits
    n, D = codes.shape
    c = codes.reshape(n, D // per, per).astype(np.uint32)
    out = np.zeros((n, D // per), dtype=np.uint32)
    for i in range(per):
        out |= c[:, :, i] << np.uint32(i * bits)
    return out.astype(np.uint8)


def unpack_codes(packed, bits):
    packed = np.asarray(packed, dtype=np.uint8)
    per = 8 // bits
    parts = [(packed >> np.uint8(i * bits)) & np.uint8((1 << bits) - 1) for i in range(per)]
    return np.stack(parts, axis=-1).reshape(packed.shape[0], -1)


def sparse_attend_qv(q, q_pos, Kc, Uk, codes, scale, zero, idx, H_kv, theta, rope_style=0):
    """Algorithm 1 from the reconstruction step on, with the paper's value path: keys are
    reconstructed from the latent cache and rotated; values are the de-quantised rows of the
    quantised full-rank cache (codes [S, D_kv], scale / zero [S, D_kv/32])."""
    q = np.asarray(q, dtype=np.float64)
    H, d = q.shape
    idx = np.asarray(idx, dtype=np.int32)
    n = idx.shape[0]
    K_C = reconstruct(Kc, idx, Uk).reshape(n, H_kv, d)
    KR = rope(K_C, idx, theta, rope_style) if n else K_C
    qR = rope(q.reshape(1, H, d), [q_pos], theta, rope_style).reshape(H, d)
    V_C = dequantize_values(np.asarray(codes)[idx], np.asarray(scale)[idx],
                            np.asarray(zero)[idx]).reshape(n, H_kv, d)
    return attend(qR, KR, V_C)


# ---------------------------------------------------------------------------
# Dense decode attention, the baseline the paper measures against (Sec. 5.3,
# Table 6: attention over the whole full-rank cache).  K is the cache as a
# dense model keeps it, keys already rotated at their positions.
# ---------------------------------------------------------------------------

def dense_decode(q, q_pos, KR, V, theta, rope_style=0):
    """q [H,d] pre-RoPE, KR [S,H_kv,d] rotated keys, V [S,H_kv,d] -> y [H,d]:
    softmax(RoPE(q, q_pos) . KR^T / sqrt(d)) V over all S tokens (Eq. 5 with C = everything)."""
    q = np.asarray(q, dtype=np.float64)
    H, d = q.shape
    if np.asarray(KR).shape[0] == 0:
        return np.zeros((H, d))
    qR = rope(q.reshape(1, H, d), [q_pos], theta, rope_style).reshape(H, d)
    return attend(qR, KR, V)


# ---------------------------------------------------------------------------
# Overlap score (Sec. 3.2): the share of the full attention mass that a selected
# index set captures, OS = sum_{i in C} p_i / sum_i p_i with p the attention
# distribution over all cached tokens.
# ---------------------------------------------------------------------------

def overlap_score(q, q_pos, KR, idx, theta, rope_style=0):
    """q [H,d] pre-RoPE, KR [S,H_kv,d] rotated keys of every cached token, idx [n] -> OS [H]."""
    q = np.asarray(q, dtype=np.float64)
    KR = np.asarray(KR, dtype=np.float64)
    H, d = q.shape
    S = KR.shape[0]
    if S == 0:
        return np.zeros(H)
    qR = rope(q.reshape(1, H, d), [q_pos], theta, rope_style).reshape(H, d)
    _, p = attend(qR, KR, np.zeros_like(KR), return_p=True)   # p [H,S], rows sum to one
    idx = np.asarray(idx, dtype=np.int64)
    return p[:, idx].sum(axis=1) / p.sum(axis=1)


# ---------------------------------------------------------------------------
# Mixed-precision recent window (Sec. 5.1): the most recent w tokens are kept at
# a milder compression than the rest, and this window coincides with the recent
# tokens the selection always keeps (Sec. 5.2).  Reading taken where the paper
# is silent: the window is a second latent cache of rank r_hi > r with its own
# projectors (the leading r_hi principal directions; r_hi = D_kv/2 is the 50 %
# setting), held as a ring of w rows: token t lives in row t mod w while
# S - w <= t < S.  A token is written to both caches when it is appended (the
# low-rank row is what remains once the ring row is overwritten), so nothing is
# re-compressed when a token leaves the window.  Attention runs one softmax
# over the union of the selected tokens, each reconstructed from the cache that
# holds it.
# ---------------------------------------------------------------------------

def window_append(Kw, Vw, k_new, v_new, Uk_hi, Uv_hi, t):
    """Writes token t (its latent images under the window's projectors) into ring row t mod w
    of Kw, Vw [w, r_hi], in place."""
    w = Kw.shape[0]
    Kw[t % w] = project(k_new, Uk_hi)
    Vw[t % w] = project(v_new, Uv_hi)


def sparse_attend_window(q, q_pos, Kc, Vc, Uk, Uv, Kw, Vw, Uk_hi, Uv_hi, idx, S, H_kv, theta,
                         rope_style=0):
    """Algorithm 1 from the reconstruction step on with the recent window of Sec. 5.1.
    Kc, Vc [S_max, r] with Uk, Uv [D_kv, r]; Kw, Vw [w, r_hi] with Uk_hi, Uv_hi [D_kv, r_hi];
    idx [n] selected tokens of a cache of S tokens.  Token t is read from ring row t mod w if
    S - w <= t < S, else from row t of the low-rank caches."""
    q = np.asarray(q, dtype=np.float64)
    H, d = q.shape
    idx = np.asarray(idx, dtype=np.int32)
    n = idx.shape[0]
    w = np.asarray(Kw).shape[0]
    in_win = (idx >= S - w) & (idx < S)
    K_C = np.empty((n, H_kv * d))
    V_C = np.empty((n, H_kv * d))
    lo, hi = idx[~in_win], idx[in_win]
    K_C[~in_win] = reconstruct(Kc, lo, Uk)
    V_C[~in_win] = reconstruct(Vc, lo, Uv)
    K_C[in_win] = reconstruct(Kw, hi % w, Uk_hi)
    V_C[in_win] = reconstruct(Vw, hi % w, Uv_hi)
    KR = rope(K_C.reshape(n, H_kv, d), idx, theta, rope_style) if n else K_C.reshape(n, H_kv, d)
    qR = rope(q.reshape(1, H, d), [q_pos], theta, rope_style).reshape(H, d)
    return attend(qR, KR, V_C.reshape(n, H_kv, d))


# ---------------------------------------------------------------------------
# Recent window of the paper's own setting (Sec. 5.1): latent keys + quantised
# full-rank values, with the most recent w tokens kept at half their original
# size.  Reading taken where the paper is silent: for keys that is the rank-r_hi
# ring of the window above (r_hi = D_kv/2); for values, whose codes take 16 bits
# per channel uncompressed, it is the same group quantiser at 8 bits, in a ring of
# w rows (token t in row t mod w).  One softmax runs over the union.
# ---------------------------------------------------------------------------

def sparse_attend_qv_window(q, q_pos, Kc, Uk, codes, scale, zero, Kw, Uk_hi, codes_w, scale_w, zero_w, idx, S,
                            H_kv, theta, rope_style=0):
    """Kc [S_max, r] with Uk [D_kv, r]; codes [S_max, D_kv], scale / zero [S_max, D_kv/32] (low-bit cache);
    Kw [w, r_hi] with Uk_hi [D_kv, r_hi]; codes_w [w, D_kv], scale_w / zero_w [w, D_kv/32] (8-bit ring);
    idx [n] selected tokens of a cache of S tokens.  Token t is read from ring row t mod w if S - w <= t < S,
    else from row t of the main caches."""
    q = np.asarray(q, dtype=np.float64)
    H, d = q.shape
    idx = np.asarray(idx, dtype=np.int32)
    n = idx.shape[0]
    w = np.asarray(Kw).shape[0]
    in_win = (idx >= S - w) & (idx < S)
    K_C = np.empty((n, H_kv * d))
    V_C = np.empty((n, H_kv * d))
    lo, hi = idx[~in_win], idx[in_win]
    K_C[~in_win] = reconstruct(Kc, lo, Uk)
    K_C[in_win] = reconstruct(Kw, hi % w, Uk_hi)
    V_C[~in_win] = dequantize_values(np.asarray(codes)[lo], np.asarray(scale)[lo], np.asarray(zero)[lo])
    V_C[in_win] = dequantize_values(np.asarray(codes_w)[hi % w], np.asarray(scale_w)[hi % w], np.asarray(zero_w)[hi % w])
    KR = rope(K_C.reshape(n, H_kv, d), idx, theta, rope_style) if n else K_C.reshape(n, H_kv, d)
    qR = rope(q.reshape(1, H, d), [q_pos], theta, rope_style).reshape(H, d)
    return attend(qR, KR, V_C.reshape(n, H_kv, d))

"""ctypes/numpy wrapper of the fp64 SALS oracle (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module.  It imports nothing from the HIP package.

Every function takes and returns float64 numpy arrays (int32 for indices) and
forwards to the plain C implementation in ``sals_oracle.c``, one call per step
of Algorithm 1 of the paper (arXiv 2510.24273).
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

"""Thin ctypes binding of ``libsals.so`` (see ``include/sals.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the current stream.
Importing this module fails loudly when the library has not been built
(``python -m paper_2510_24273_amd.build``); there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

import torch  # noqa: F401  (must be imported first: it brings the HIP runtime in)

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SALS_LIB") or os.path.join(_HERE, "libsals.so")   # SALS_LIB: another build of the same library

SALS_OK = 0
SALS_ERR_INVALID_ARG = 1
SALS_ERR_UNSUPPORTED = 2
SALS_ERR_WORKSPACE = 3
SALS_ERR_HIP = 4
SALS_F32, SALS_BF16 = 0, 1

EXPORTS = (
    "sals_status_string", "sals_workspace_bytes", "sals_create", "sals_prepare", "sals_destroy",
    "sals_compress_append", "sals_latent_scores", "sals_topk_select", "sals_sparse_attend",
    "sals_decode_step", "sals_kernel_name", "sals_profile_enable", "sals_profile_collect",
    "sals_packed_weight_bytes", "sals_pack_weights",
    "sals_qv_row_bytes", "sals_compress_append_qv", "sals_sparse_attend_qv", "sals_decode_step_qv",
    "sals_dense_attend",
    "sals_window_append", "sals_sparse_attend_window", "sals_decode_step_window", "sals_overlap_score",
    "sals_latent_scores_noalloc", "sals_compress_prefill",
    "sals_window_append_qv", "sals_sparse_attend_qv_window", "sals_decode_step_qv_window",
    "sals_calib_accumulate_workspace_bytes", "sals_calib_accumulate",
    "sals_calib_eigenvectors_workspace_bytes", "sals_calib_eigenvectors",
)
N_KERNELS = 9


class SalsDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "S_max", "H_q", "H_kv", "d", "r", "r_score", "top_k", "n_recent", "n_sink")] + \
               [("rope_theta", ctypes.c_float), ("rope_style", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class SalsError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)}")


def load_library() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2510_24273_amd.build` "
            "(hipcc, gfx950). There is no fallback implementation.")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32p, f32p = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
    lib.sals_status_string.restype = ctypes.c_char_p
    lib.sals_status_string.argtypes = [ctypes.c_int]
    lib.sals_workspace_bytes.argtypes = [ctypes.POINTER(SalsDesc), ctypes.POINTER(ctypes.c_size_t)]
    lib.sals_create.argtypes = [ctypes.POINTER(SalsDesc), vp, ctypes.c_size_t, ctypes.POINTER(vp)]
    lib.sals_prepare.argtypes = [vp, vp]
    lib.sals_destroy.argtypes = [vp]
    lib.sals_destroy.restype = None
    lib.sals_packed_weight_bytes.argtypes = [ctypes.POINTER(SalsDesc), ctypes.POINTER(ctypes.c_size_t)]
    lib.sals_pack_weights.argtypes = [vp, vp, vp, vp, vp]
    lib.sals_compress_append.argtypes = [vp, vp, vp, vp, vp, vp, i32p, vp]
    lib.sals_compress_prefill.argtypes = [vp, vp, vp, vp, vp, vp, i32p, i32p, ctypes.c_int32, vp]
    lib.sals_latent_scores.argtypes = [vp, vp, vp, vp, i32p, f32p, vp]
    lib.sals_latent_scores_noalloc.argtypes = [ctypes.POINTER(SalsDesc), vp, vp, vp, i32p, f32p, vp]
    lib.sals_topk_select.argtypes = [vp, f32p, i32p, i32p, i32p, vp]
    lib.sals_sparse_attend.argtypes = [vp, vp, i32p, vp, vp, vp, i32p, i32p, vp, vp]
    lib.sals_decode_step.argtypes = [vp, vp, i32p, vp, vp, vp, i32p, vp, f32p, i32p, i32p, vp]
    lib.sals_qv_row_bytes.argtypes = [ctypes.POINTER(SalsDesc), ctypes.c_int, ctypes.POINTER(ctypes.c_size_t),
                                      ctypes.POINTER(ctypes.c_size_t)]
    lib.sals_compress_append_qv.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, i32p, vp]
    lib.sals_sparse_attend_qv.argtypes = [vp, vp, i32p, vp, vp, vp, ctypes.c_int, vp, i32p, i32p, vp, vp]
    lib.sals_decode_step_qv.argtypes = [vp, vp, i32p, vp, vp, vp, ctypes.c_int, vp, i32p, vp, f32p, i32p, i32p, vp]
    lib.sals_dense_attend.argtypes = [vp, vp, i32p, vp, vp, i32p, vp, vp]
    lib.sals_window_append.argtypes = [vp, vp, vp, vp, vp, vp, i32p, vp]
    lib.sals_sparse_attend_window.argtypes = [vp, vp, vp, i32p, vp, vp, vp, vp, vp, vp, i32p, i32p, vp, vp]
    lib.sals_decode_step_window.argtypes = [vp, vp, vp, i32p, vp, vp, vp, vp, vp, vp, i32p, vp, f32p, i32p, i32p, vp]
    lib.sals_window_append_qv.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32p, vp]
    lib.sals_sparse_attend_qv_window.argtypes = [vp, vp, vp, i32p, vp, vp, vp, ctypes.c_int, vp, vp, vp, vp, vp, i32p,
                                                 i32p, vp, vp]
    lib.sals_decode_step_qv_window.argtypes = [vp, vp, vp, i32p, vp, vp, vp, ctypes.c_int, vp, vp, vp, vp, vp, i32p, vp,
                                               f32p, i32p, i32p, vp]
    lib.sals_overlap_score.argtypes = [vp, vp, i32p, vp, i32p, i32p, i32p, f32p, vp]
    lib.sals_calib_accumulate_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.sals_calib_accumulate.argtypes = [ctypes.c_int32, vp, ctypes.c_int64, ctypes.c_int32, vp, vp, ctypes.c_size_t, vp]
    lib.sals_calib_eigenvectors_workspace_bytes.argtypes = [ctypes.c_int32]
    lib.sals_calib_eigenvectors.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp,
                                            ctypes.c_size_t, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), vp]
    lib.sals_kernel_name.restype = ctypes.c_char_p
    lib.sals_kernel_name.argtypes = [ctypes.c_int]
    lib.sals_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.sals_profile_collect.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    for name in EXPORTS[1:]:
        if name.endswith("_workspace_bytes") and name.startswith("sals_calib"):
            getattr(lib, name).restype = ctypes.c_size_t
        elif name not in ("sals_destroy", "sals_kernel_name"):
            getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = load_library()


def status_string(code: int) -> str:
    return _lib.sals_status_string(int(code)).decode()


def make_desc(B, S_max, H_q, H_kv, d, r, top_k, dtype, r_score=None, n_recent=0, n_sink=0,
              rope_theta=10000.0, rope_style=0) -> SalsDesc:
    dt = {"bf16": SALS_BF16, "f32": SALS_F32, torch.bfloat16: SALS_BF16, torch.float32: SALS_F32}[dtype]
    return SalsDesc(B, S_max, H_q, H_kv, d, r, r if r_score is None else r_score, top_k, n_recent,
                    n_sink, rope_theta, rope_style, dt)


def workspace_bytes(desc: SalsDesc) -> int:
    n = ctypes.c_size_t(0)
    st = _lib.sals_workspace_bytes(ctypes.byref(desc), ctypes.byref(n))
    if st != SALS_OK:
        raise SalsError(st, "sals_workspace_bytes")
    return int(n.value)


def packed_weight_bytes(desc: SalsDesc) -> int:
    n = ctypes.c_size_t(0)
    st = _lib.sals_packed_weight_bytes(ctypes.byref(desc), ctypes.byref(n))
    if st != SALS_OK:
        raise SalsError(st, "sals_packed_weight_bytes")
    return int(n.value)


def qv_row_bytes(desc: SalsDesc, bits: int):
    """(code bytes, meta bytes) per token of the quantised value cache."""
    c, m = ctypes.c_size_t(0), ctypes.c_size_t(0)
    st = _lib.sals_qv_row_bytes(ctypes.byref(desc), int(bits), ctypes.byref(c), ctypes.byref(m))
    if st != SALS_OK:
        raise SalsError(st, "sals_qv_row_bytes")
    return int(c.value), int(m.value)


def latent_scores_noalloc(desc: SalsDesc, q, W, Kc, seq_len, scores):
    """sals_latent_scores without a context or workspace (scratch inside the library's device image)."""
    st = _lib.sals_latent_scores_noalloc(ctypes.byref(desc), _p(q), _p(W), _p(Kc), _p(seq_len), _p(scores), _stream())
    if st != SALS_OK:
        raise SalsError(st, "sals_latent_scores_noalloc")


def _dtype_code(t):
    return {torch.bfloat16: SALS_BF16, torch.float32: SALS_F32}[t]


def calib_accumulate(keys, C):
    """Offline calibration (Sec. 4.2): C += keys^T keys.  keys [n_tok, D] bf16 | f32, C [D, D] float64, both on the
    device; the transposed-chunk workspace is a torch tensor allocated here."""
    n_tok, D = keys.shape
    dt = _dtype_code(keys.dtype)
    nbytes = int(_lib.sals_calib_accumulate_workspace_bytes(dt, D))
    if nbytes == 0:
        raise SalsError(1, "sals_calib_accumulate_workspace_bytes")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=keys.device)
    st = _lib.sals_calib_accumulate(dt, _p(keys), int(n_tok), int(D), _p(C), _p(ws), nbytes, _stream())
    if st != SALS_OK:
        raise SalsError(st, "sals_calib_accumulate")
    return ws  # (kept alive by the caller until the stream has run)


def calib_eigenvectors(C, r, dtype, max_sweeps=80):
    """Offline calibration (Sec. 4.2): eigenvalues (descending, float64 [D]) and the r leading eigenvectors
    (U [D, r] in `dtype`) of the covariance C [D, D] float64, which is overwritten.  Blocking.
    Returns (eigval, U, sweeps)."""
    D = C.shape[0]
    nbytes = int(_lib.sals_calib_eigenvectors_workspace_bytes(D))
    if nbytes == 0:
        raise SalsError(1, "sals_calib_eigenvectors_workspace_bytes")
    ws = torch.empty(nbytes, dtype=torch.uint8, device=C.device)
    eigval = torch.empty(D, dtype=torch.float64, device=C.device)
    U = torch.empty(D, r, dtype=dtype, device=C.device)
    sweeps = ctypes.c_int32(0)
    st = _lib.sals_calib_eigenvectors(_p(C), int(D), int(r), _dtype_code(dtype), _p(eigval), _p(U), _p(ws), nbytes,
                                      int(max_sweeps), ctypes.byref(sweeps), _stream())
    if st != SALS_OK:
        raise SalsError(st, "sals_calib_eigenvectors")
    return eigval, U, int(sweeps.value)


def _p(t):
    """Device pointer of a tensor (None -> NULL)."""
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


class Sals:
    """One context: descriptor + caller-owned (torch) workspace."""

    def __init__(self, desc: SalsDesc, device="cuda:0"):
        self.desc = desc
        self.device = torch.device(device)
        self.k_tot = desc.top_k + desc.n_sink + desc.n_recent
        nbytes = workspace_bytes(desc)
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8, device=self.device)
        h = ctypes.c_void_p()
        st = _lib.sals_create(ctypes.byref(desc), self.workspace.data_ptr(), nbytes, ctypes.byref(h))
        if st != SALS_OK:
            raise SalsError(st, "sals_create")
        self._h = h
        # one-time device set-up (cos/sin table, kernel attributes): afterwards any stream, graph capture included
        st = _lib.sals_prepare(h, torch.cuda.current_stream(self.device).cuda_stream)
        if st != SALS_OK:
            _lib.sals_destroy(h)
            self._h = None
            raise SalsError(st, "sals_prepare")
        self._destroy = _lib.sals_destroy   # kept on the instance: module globals may be gone at interpreter exit

    def close(self):
        h, self._h = getattr(self, "_h", None), None
        destroy = getattr(self, "_destroy", None)
        if h and destroy is not None:
            destroy(h)

    def __del__(self):
        try:
            self.close()
        except Exception:   # interpreter shutdown: the library may already be unloaded
            pass

    @staticmethod
    def _check(st, where):
        if st != SALS_OK:
            raise SalsError(st, where)

    def profile(self, on: bool):
        self._check(_lib.sals_profile_enable(self._h, 1 if on else 0), "sals_profile_enable")

    def profile_collect(self) -> dict:
        """{kernel name: (total ms, launches)} since profiling was enabled / last collected."""
        ms = (ctypes.c_double * N_KERNELS)()
        n = (ctypes.c_int32 * N_KERNELS)()
        self._check(_lib.sals_profile_collect(self._h, ms, n), "sals_profile_collect")
        return {_lib.sals_kernel_name(k).decode(): (float(ms[k]), int(n[k])) for k in range(N_KERNELS)}

    def pack_weights(self, Uk, Uv):
        """One-time repacking of a layer's projectors; returns the packed device buffer W."""
        W = torch.empty(packed_weight_bytes(self.desc), dtype=torch.uint8, device=self.device)
        self._check(_lib.sals_pack_weights(self._h, _p(Uk), _p(Uv), _p(W), _stream()), "sals_pack_weights")
        return W

    def compress_append(self, k_new, v_new, W, Kc, Vc, seq_len):
        self._check(_lib.sals_compress_append(self._h, _p(k_new), _p(v_new), _p(W), _p(Kc), _p(Vc),
                                              _p(seq_len), _stream()), "sals_compress_append")

    def compress_prefill(self, k_new, v_new, W, Kc, Vc, seq_len, n_tok, n_new=None):
        """Bulk compression of n_tok prompt tokens per sequence (k_new, v_new [B, n_tok, D_kv])."""
        self._check(_lib.sals_compress_prefill(self._h, _p(k_new), _p(v_new), _p(W), _p(Kc), _p(Vc), _p(seq_len),
                                               _p(n_new), int(n_tok), _stream()), "sals_compress_prefill")

    def latent_scores(self, q, W, Kc, seq_len, scores):
        self._check(_lib.sals_latent_scores(self._h, _p(q), _p(W), _p(Kc), _p(seq_len), _p(scores),
                                            _stream()), "sals_latent_scores")

    def topk_select(self, scores, seq_len, idx, n_sel):
        self._check(_lib.sals_topk_select(self._h, _p(scores), _p(seq_len), _p(idx), _p(n_sel),
                                          _stream()), "sals_topk_select")

    def sparse_attend(self, q, q_pos, Kc, Vc, W, idx, n_sel, out):
        self._check(_lib.sals_sparse_attend(self._h, _p(q), _p(q_pos), _p(Kc), _p(Vc), _p(W), _p(idx),
                                            _p(n_sel), _p(out), _stream()), "sals_sparse_attend")

    def decode_step(self, q, q_pos, Kc, Vc, W, seq_len, out, scores=None, idx=None, n_sel=None):
        self._check(_lib.sals_decode_step(self._h, _p(q), _p(q_pos), _p(Kc), _p(Vc), _p(W), _p(seq_len),
                                          _p(out), _p(scores), _p(idx), _p(n_sel), _stream()),
                    "sals_decode_step")

    # ---- quantised full-rank value cache (codes Vq, per-group (scale, zero) Vmeta) ----
    def compress_append_qv(self, k_new, v_new, W, Kc, Vq, Vmeta, bits, seq_len):
        self._check(_lib.sals_compress_append_qv(self._h, _p(k_new), _p(v_new), _p(W), _p(Kc), _p(Vq), _p(Vmeta),
                                                 int(bits), _p(seq_len), _stream()), "sals_compress_append_qv")

    def sparse_attend_qv(self, q, q_pos, Kc, Vq, Vmeta, bits, W, idx, n_sel, out):
        self._check(_lib.sals_sparse_attend_qv(self._h, _p(q), _p(q_pos), _p(Kc), _p(Vq), _p(Vmeta), int(bits),
                                               _p(W), _p(idx), _p(n_sel), _p(out), _stream()),
                    "sals_sparse_attend_qv")

    def decode_step_qv(self, q, q_pos, Kc, Vq, Vmeta, bits, W, seq_len, out, scores=None, idx=None, n_sel=None):
        self._check(_lib.sals_decode_step_qv(self._h, _p(q), _p(q_pos), _p(Kc), _p(Vq), _p(Vmeta), int(bits), _p(W),
                                             _p(seq_len), _p(out), _p(scores), _p(idx), _p(n_sel), _stream()),
                    "sals_decode_step_qv")

    # ---- dense baseline over a full-rank cache of rotated keys ----
    def dense_attend(self, q, q_pos, K, V, seq_len, out):
        self._check(_lib.sals_dense_attend(self._h, _p(q), _p(q_pos), _p(K), _p(V), _p(seq_len), _p(out),
                                           _stream()), "sals_dense_attend")

    # ---- high-precision recent window: `win` is the window's own context (rank r_hi, top_k = w) ----
    def window_append(self, k_new, v_new, W_hi, Kw, Vw, seq_len):
        """Called on the window's context, before the compress_append that advances seq_len."""
        self._check(_lib.sals_window_append(self._h, _p(k_new), _p(v_new), _p(W_hi), _p(Kw), _p(Vw), _p(seq_len),
                                            _stream()), "sals_window_append")

    def sparse_attend_window(self, win, q, q_pos, Kc, Vc, W, Kw, Vw, W_hi, idx, n_sel, out):
        self._check(_lib.sals_sparse_attend_window(self._h, win._h, _p(q), _p(q_pos), _p(Kc), _p(Vc), _p(W), _p(Kw),
                                                   _p(Vw), _p(W_hi), _p(idx), _p(n_sel), _p(out), _stream()),
                    "sals_sparse_attend_window")

    def decode_step_window(self, win, q, q_pos, Kc, Vc, W, Kw, Vw, W_hi, seq_len, out, scores=None, idx=None,
                           n_sel=None):
        self._check(_lib.sals_decode_step_window(self._h, win._h, _p(q), _p(q_pos), _p(Kc), _p(Vc), _p(W), _p(Kw),
                                                 _p(Vw), _p(W_hi), _p(seq_len), _p(out), _p(scores), _p(idx),
                                                 _p(n_sel), _stream()), "sals_decode_step_window")

    # ---- the window over latent keys + quantised values: keys in the ring Kw, values as 8-bit codes Vqw / Vmeta_w ----
    def window_append_qv(self, k_new, v_new, W_hi, Kw, Vqw, Vmeta_w, seq_len):
        """Called on the window's context, before the compress_append_qv that advances seq_len."""
        self._check(_lib.sals_window_append_qv(self._h, _p(k_new), _p(v_new), _p(W_hi), _p(Kw), _p(Vqw), _p(Vmeta_w),
                                               _p(seq_len), _stream()), "sals_window_append_qv")

    def sparse_attend_qv_window(self, win, q, q_pos, Kc, Vq, Vmeta, bits, W, Kw, Vqw, Vmeta_w, W_hi, idx, n_sel, out):
        self._check(_lib.sals_sparse_attend_qv_window(self._h, win._h, _p(q), _p(q_pos), _p(Kc), _p(Vq), _p(Vmeta),
                                                      int(bits), _p(W), _p(Kw), _p(Vqw), _p(Vmeta_w), _p(W_hi), _p(idx),
                                                      _p(n_sel), _p(out), _stream()), "sals_sparse_attend_qv_window")

    def decode_step_qv_window(self, win, q, q_pos, Kc, Vq, Vmeta, bits, W, Kw, Vqw, Vmeta_w, W_hi, seq_len, out,
                              scores=None, idx=None, n_sel=None):
        self._check(_lib.sals_decode_step_qv_window(self._h, win._h, _p(q), _p(q_pos), _p(Kc), _p(Vq), _p(Vmeta),
                                                    int(bits), _p(W), _p(Kw), _p(Vqw), _p(Vmeta_w), _p(W_hi),
                                                    _p(seq_len), _p(out), _p(scores), _p(idx), _p(n_sel), _stream()),
                    "sals_decode_step_qv_window")

    # ---- overlap score of a selection against dense attention over rotated full-rank keys ----
    def overlap_score(self, q, q_pos, K, seq_len, idx, n_sel, os):
        self._check(_lib.sals_overlap_score(self._h, _p(q), _p(q_pos), _p(K), _p(seq_len), _p(idx), _p(n_sel),
                                            _p(os), _stream()), "sals_overlap_score")

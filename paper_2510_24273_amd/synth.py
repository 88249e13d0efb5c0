"""Seeded synthetic decode workloads shaped like the paper's models.

This module only *makes inputs*: projectors, latent caches and queries with
the shapes of LLaMA2-7B, Mistral-7B and LLaMA3.1-8B decode (Sec. 5.1 of arXiv
2510.24273), which stand in for the paper's real activations.  It holds none
of the operator's arithmetic that is under test and produces no expected
values; both the HIP path and the CPU oracle are fed from here.  The only
linear algebra it does is to orient a few planted cache rows along the latent
image of the query, so that the selection stage has known winners.

Storage rounding happens here, so both sides see bit-identical inputs: every
array is returned in its storage form (float32, or bf16 as uint16 bit
patterns) and ``widen`` turns either into the float64 the oracle reads.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int
    B: int
    S: int
    H: int
    H_kv: int
    d: int
    r: int
    top_k: int
    dtype: str = "bf16"          # storage type: "bf16" | "f32"
    r_score: int | None = None   # None -> r
    n_sink: int = 0
    n_recent: int = 0
    theta: float = 10000.0
    rope_style: int = 0
    n_layers: int = 1
    plant: int = 0               # planted high-score tokens per query
    corr_frac: float = 0.0       # fraction of rows correlated with the query
    corr_rho: float = 0.3
    scale: float = 1.0           # extra cache scale (stress cases only)
    qv_bits: int = 0             # > 0: values live in the quantised full-rank cache (2 | 4 bits)
    r_hi: int = 0                # > 0: the n_recent last tokens live in a ring cache of this rank (Sec. 5.1)
    fill: float = 1.0            # share of the cache capacity S that holds tokens (sequence length = S * fill)

    @property
    def D_kv(self):
        return self.H_kv * self.d

    @property
    def k_tot(self):
        return self.top_k + self.n_sink + self.n_recent

    @property
    def rs(self):
        return self.r if self.r_score is None else self.r_score

    @property
    def S_live(self):
        """Tokens per sequence (the cache holds S rows, the first S_live of them are written)."""
        return int(self.S * self.fill)

    @property
    def esize(self):
        return 2 if self.dtype == "bf16" else 4


# The five configurations the build is measured on.
CONFIGS = {
    "cfg1": Workload("cfg1_tiny_f32_B1_S1024_r512_k128", 1, 1, 1024, 32, 32, 128, 512, 128,
                     dtype="f32"),
    "cfg2": Workload("cfg2_llama2_7b_B1_S4096_r640_k512", 2, 1, 4096, 32, 32, 128, 640, 512,
                     n_layers=32, plant=3),
    "cfg3a": Workload("cfg3a_llama2_7b_B16_S4096_r640_k512", 3, 16, 4096, 32, 32, 128, 640,
                      512, plant=3),
    "cfg3b": Workload("cfg3b_mistral_7b_gqa8_B16_S4096_r640_k512", 3, 16, 4096, 32, 8, 128,
                      640, 512, plant=3),
    "cfg4": Workload("cfg4_long_B4_S32768_r640_k2048", 4, 4, 32768, 32, 32, 128, 640, 2048,
                     corr_frac=0.01),
    "cfg5": Workload("cfg5_llama31_8b_gqa8_B1_S131072_r512_k4096_w64", 5, 1, 131072, 32, 8,
                     128, 512, 4096, n_recent=64, theta=500000.0),
}


def shrink(w: Workload, **kw) -> Workload:
    return replace(w, **kw)


# The paper's own scoring rank r* = r/2 (Sec. 4.3, Sec. 5.1) on the measured shapes: same inputs,
# scores taken over the leading half of the latent coordinates only.
VARIANTS = {
    name + "_rhalf": replace(w, name=w.name + "_rscore" + str(w.r // 2), r_score=w.r // 2)
    for name, w in CONFIGS.items() if name in ("cfg2", "cfg3a", "cfg4")
}
# The paper's own value path (Sec. 5.1): quantised full-rank value cache, 4 bit (25 % setting) / 2 bit.
VARIANTS.update({
    f"{name}_qv{bits}": replace(w, name=f"{w.name}_qvalue{bits}bit", qv_bits=bits)
    for name, w in CONFIGS.items() if name in ("cfg2", "cfg3a", "cfg3b", "cfg4") for bits in (4, 2)
})


# The paper's selection composition for LLaMA2-7B (Sec. 5.2: 16 sink + 432 critical + 64 recent tokens) with
# the recent tokens in a high-precision window (Sec. 5.1) of rank D_kv/2, the paper's 50 % setting.
VARIANTS.update({
    f"{name}_comp": replace(w, name=f"{w.name}_sink16_crit432_recent64", top_k=432, n_sink=16, n_recent=64)
    for name, w in CONFIGS.items() if name in ("cfg2", "cfg3a")
})
VARIANTS.update({
    f"{name}_win": replace(w, name=f"{w.name}_sink16_crit432_win64_rhi2048", top_k=432, n_sink=16,
                           n_recent=64, r_hi=2048)
    for name, w in CONFIGS.items() if name in ("cfg2", "cfg3a")
})


# The shapes of the paper's operator-latency table (Table 6: LLaMA2-7B, batch 8 / 16, 1k / 2k / 4k tokens, token
# sparsity 1/8) in its two settings: SALS-25 % (rank D_kv/4, 4-bit values) and SALS-12.5 % (rank D_kv/8, 2-bit
# values), scores over the leading half of the latent coordinates (Sec. 5.1), selection = 16 sink + critical +
# 64 recent tokens = S/8 (Sec. 5.2).
for _B in (8, 16):
    for _S in (1024, 2048, 4096):
        for _tag, _r, _bits in (("25", 1024, 4), ("12", 512, 2)):
            VARIANTS[f"t6_b{_B}_s{_S}_{_tag}"] = Workload(
                f"table6_llama2_7b_B{_B}_S{_S}_r{_r}_rscore{_r // 2}_k{_S // 8}_qvalue{_bits}bit", 6, _B, _S, 32, 32,
                128, _r, _S // 8 - 80, r_score=_r // 2, n_sink=16, n_recent=64, plant=3, qv_bits=_bits)


# A decode loop's cache is allocated for more tokens than it holds: the long-context shape with twice the capacity
# (the score stream and the selection must cost the 32768 tokens present, not the 65536 rows allocated).
VARIANTS["cfg4_cap2x"] = replace(CONFIGS["cfg4"], name="cfg4_long_B4_S32768_capacity65536_r640_k2048", S=65536, fill=0.5)


# The same table shapes with the paper's mixed precision (Sec. 5.1): the 64 recent tokens in the window formats,
# keys at rank D_kv/2 and values at 8 bits; and the LLaMA2 composition at the B = 1 shape in the 25 % setting.
for _name in [n for n in VARIANTS if n.startswith("t6_")]:
    _w = VARIANTS[_name]
    VARIANTS["t6w_" + _name[3:]] = replace(_w, name=_w.name + "_win64_rhi2048_8bit", r_hi=2048)
VARIANTS["cfg2_qvwin"] = replace(CONFIGS["cfg2"], name="cfg2_llama2_7b_B1_S4096_r1024_rscore512_sink16_crit432_win64_rhi2048_qvalue4bit",
                                 r=1024, r_score=512, top_k=432, n_sink=16, n_recent=64, r_hi=2048, qv_bits=4)


def lookup(name: str) -> Workload:
    """A measured configuration or one of its variants, by short name."""
    return CONFIGS[name] if name in CONFIGS else VARIANTS[name]


# ---- storage rounding ------------------------------------------------------

def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float -> bf16 bit patterns (uint16), round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round a float array to its storage form."""
    if dtype == "bf16":
        return to_bf16_bits(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(dtype)


def widen(x: np.ndarray) -> np.ndarray:
    """Storage form -> float64 (exact)."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


# ---- generators ------------------------------------------------------------

def seed_of(w: Workload, layer: int, b: int) -> int:
    return 10_000 * w.cfg_id + 100 * layer + b


def make_projector(rng: np.random.Generator, D: int, r: int) -> np.ndarray:
    """[D x r] with orthonormal columns (rows of its transpose are the
    orthonormal rows of the up-projection): Q factor of a Gaussian matrix."""
    if r <= D:
        qm, _ = np.linalg.qr(rng.standard_normal((D, r)))
        return qm
    # over-complete rank (tests only): orthonormal rows instead
    qm, _ = np.linalg.qr(rng.standard_normal((r, D)))
    return qm.T


def make_weights(w: Workload, layer: int = 0):
    """Per-layer projectors U_k, U_v [D_kv x r], storage-rounded."""
    rng = np.random.default_rng(seed_of(w, layer, 99))
    Uk = make_projector(rng, w.D_kv, w.r)
    Uv = make_projector(rng, w.D_kv, w.r)
    return store(Uk, w.dtype), store(Uv, w.dtype)


def make_sequence(w: Workload, layer: int, b: int, Uk_stored: np.ndarray, S: int | None = None):
    """One sequence's query and latent caches, storage-rounded.

    Cache entries are N(0,1) scaled by the decaying spectrum (c+1)^-1/2 of the
    latent coordinate c.  Returns dict(q [H,d], Kc [S,r], Vc [S,r], planted)."""
    S = w.S if S is None else S
    rng = np.random.default_rng(seed_of(w, layer, b))
    sigma = (np.arange(1, w.r + 1, dtype=np.float64)) ** -0.5 * w.scale
    q = rng.standard_normal((w.H, w.d))
    Kc = rng.standard_normal((S, w.r), dtype=np.float32).astype(np.float64) * sigma
    Vc = rng.standard_normal((S, w.r), dtype=np.float32).astype(np.float64) * sigma
    planted = np.zeros(0, dtype=np.int64)
    if (w.plant or w.corr_frac > 0) and S > 0:
        # latent image of the (group-summed) query, used only to orient rows
        G = w.H // w.H_kv
        q_sum = widen(store(q, w.dtype)).reshape(w.H_kv, G, w.d).sum(axis=1).reshape(-1)
        qt = widen(Uk_stored).T @ q_sum
        qn = float(np.linalg.norm(qt))
        if w.plant:
            s_max = float(np.max(np.abs(Kc[:, : w.rs] @ qt[: w.rs])))
            planted = rng.choice(S, size=min(w.plant, S), replace=False)
            for m, t in enumerate(planted):
                Kc[t, :] += (2.0 + 0.1 * m) * s_max * qt / (qn * qn)
        if w.corr_frac > 0:
            n_c = max(1, int(round(w.corr_frac * S)))
            planted = rng.choice(S, size=n_c, replace=False)
            rows = Kc[planted, :]
            norms = np.linalg.norm(rows, axis=1, keepdims=True)
            Kc[planted, :] = (w.corr_rho * norms / qn) * qt[None, :] \
                + np.sqrt(1.0 - w.corr_rho ** 2) * rows
    return {"q": store(q, w.dtype), "Kc": store(Kc, w.dtype), "Vc": store(Vc, w.dtype),
            "planted": np.sort(planted)}


def make_layer(w: Workload, layer: int = 0, seq_lens=None):
    """A full batch for one layer: dict of stacked storage arrays.

    q [B,H,d], Kc/Vc [B,S,r] (rows past seq_len[b] are zero), Uk/Uv [D_kv,r],
    seq_len [B] int32, q_pos [B] int32 (= seq_len: the query follows the cache)."""
    Uk, Uv = make_weights(w, layer)
    seq_lens = [w.S_live] * w.B if seq_lens is None else list(seq_lens)
    assert len(seq_lens) == w.B and max(seq_lens) <= w.S
    st = np.uint16 if w.dtype == "bf16" else np.float32
    q = np.zeros((w.B, w.H, w.d), dtype=st)
    Kc = np.zeros((w.B, w.S, w.r), dtype=st)
    Vc = np.zeros((w.B, w.S, w.r), dtype=st)
    planted = []
    for b in range(w.B):
        s = make_sequence(w, layer, b, Uk, seq_lens[b])
        q[b] = s["q"]
        Kc[b, : seq_lens[b]] = s["Kc"]
        Vc[b, : seq_lens[b]] = s["Vc"]
        planted.append(s["planted"])
    sl = np.asarray(seq_lens, dtype=np.int32)
    return {"q": q, "Kc": Kc, "Vc": Vc, "Uk": Uk, "Uv": Uv, "seq_len": sl,
            "q_pos": sl.copy(), "planted": planted}


# ---- quantised full-rank value cache (the paper's value path, Sec. 5.1) ----------------

QV_GROUP = 32   # channels per quantisation group (layout constant of the cache format)


def make_values(w: Workload, layer: int = 0, n_rows: int | None = None) -> np.ndarray:
    """Full-rank value rows [B, n_rows, D_kv], storage-rounded: N(0,1) times a per-channel
    magnitude drawn once per layer (log-normal, sigma 0.5), as value activations have
    channel-dependent ranges.  Input of the quantiser under test."""
    n_rows = w.S if n_rows is None else n_rows
    rng = np.random.default_rng(seed_of(w, layer, 77))
    mag = np.exp(0.5 * rng.standard_normal(w.D_kv))
    v = rng.standard_normal((w.B, n_rows, w.D_kv), dtype=np.float32).astype(np.float64) * mag
    return store(v, w.dtype)


def make_qv_cache(w: Workload, layer: int, bits: int):
    """A quantised value cache made directly in its stored form (no quantiser involved):
    code bytes [B, S, D_kv*bits/8] uniformly random (every code value equally likely) and
    per-group (scale, zero) [B, S, D_kv/32, 2] in the storage type, with
    scale = |N(0,1)| * 4/(2^bits - 1) + a small floor and zero = -2 + 0.5 N(0,1): the
    ranges a unit-variance group of 32 channels produces."""
    rng = np.random.default_rng(seed_of(w, layer, 78) + bits)
    codes = rng.integers(0, 256, size=(w.B, w.S, w.D_kv * bits // 8), dtype=np.uint8)
    ng = w.D_kv // QV_GROUP
    scale = (np.abs(rng.standard_normal((w.B, w.S, ng), dtype=np.float32)) + 0.05) * (4.0 / ((1 << bits) - 1))
    zero = -2.0 + 0.5 * rng.standard_normal((w.B, w.S, ng), dtype=np.float32)
    meta = store(np.stack([scale, zero], axis=-1), w.dtype)
    return codes, meta


def make_qv_window(w: Workload, layer: int = 0):
    """The 8-bit value ring of the recent window, made directly in its stored form like make_qv_cache:
    code bytes [B, n_recent, D_kv] uniformly random, (scale, zero) [B, n_recent, D_kv/32, 2] in the storage type with
    scale = |N(0,1)| * 4/255 + a small floor and zero = -2 + 0.5 N(0,1)."""
    rng = np.random.default_rng(seed_of(w, layer, 89))
    codes = rng.integers(0, 256, size=(w.B, w.n_recent, w.D_kv), dtype=np.uint8)
    ng = w.D_kv // QV_GROUP
    scale = (np.abs(rng.standard_normal((w.B, w.n_recent, ng), dtype=np.float32)) + 0.05) * (4.0 / 255.0)
    zero = -2.0 + 0.5 * rng.standard_normal((w.B, w.n_recent, ng), dtype=np.float32)
    return codes, store(np.stack([scale, zero], axis=-1), w.dtype)


# ---- dense baseline: a full-rank cache as a dense model keeps it ------------------------

def make_dense_cache(w: Workload, layer: int = 0):
    """q [B,H,d] and a full-rank cache K, V [B,S,H_kv,d], storage-rounded.  K stands for keys
    already rotated at their positions (a rotation leaves the N(0,1) entries N(0,1)); with q
    also N(0,1) the logits have unit variance after the 1/sqrt(d)."""
    rng = np.random.default_rng(seed_of(w, layer, 79))
    q = rng.standard_normal((w.B, w.H, w.d))
    K = rng.standard_normal((w.B, w.S, w.H_kv, w.d), dtype=np.float32)
    V = rng.standard_normal((w.B, w.S, w.H_kv, w.d), dtype=np.float32)
    return {"q": store(q, w.dtype), "K": store(K, w.dtype), "V": store(V, w.dtype)}


# ---- high-precision recent window (Sec. 5.1) ----------------------------------------------

def make_window(w: Workload, L: dict, layer: int = 0):
    """The window caches that go with a layer `L` from make_layer: projectors Uk_hi, Uv_hi
    [D_kv, r_hi] whose first r columns are the layer's (stored) projectors and whose other
    columns are an orthonormal completion, and ring caches Kw, Vw [B, n_recent, r_hi]: for
    each of a sequence's last n_recent tokens t, row t mod n_recent holds the token's low-rank
    row followed by r_hi - r further coordinates drawn with the same decaying spectrum
    ((c+1)^-1/2 at coordinate c); rows no token maps to stay zero.  Storage-rounded."""
    assert w.r_hi > w.r and w.n_recent > 0
    rng = np.random.default_rng(seed_of(w, layer, 88))
    out = {}
    for name in ("Uk", "Uv"):
        U = widen(L[name])
        E = rng.standard_normal((w.D_kv, w.r_hi - w.r))
        E -= U @ (U.T @ E)
        E, _ = np.linalg.qr(E)
        out[name + "_hi"] = np.concatenate([L[name], store(E, w.dtype)], axis=1)
    st = np.uint16 if w.dtype == "bf16" else np.float32
    sigma = (np.arange(w.r + 1, w.r_hi + 1, dtype=np.float64)) ** -0.5 * w.scale
    n_w = w.n_recent
    for name, src in (("Kw", "Kc"), ("Vw", "Vc")):
        ring = np.zeros((w.B, n_w, w.r_hi), dtype=st)
        for b in range(w.B):
            S = int(L["seq_len"][b])
            for t in range(max(0, S - n_w), S):
                extra = rng.standard_normal(w.r_hi - w.r, dtype=np.float32).astype(np.float64) * sigma
                ring[b, t % n_w, : w.r] = L[src][b, t]
                ring[b, t % n_w, w.r:] = store(extra, w.dtype)
        out[name] = ring
    return out


# ---- offline calibration (Sec. 4.2) ----------------------------------------------------------

def make_calibration_keys(seed: int, n_tok: int, D: int, dtype: str = "bf16", decay: float = 0.97, heads: int = 1):
    """Stand-in for the pre-RoPE keys of a calibration set (the paper collects them from 512 sequences of 4096 C4
    tokens): n_tok rows of width D = n*d with a planted spectrum.  Row t = sum_c z[t, c] * sigma_c * dir_c with
    z ~ N(0, 1), sigma_c = decay^(c/2) (eigenvalues of the covariance decay geometrically, so neighbouring
    eigenvectors are separated by a fixed relative gap) and dir_c the columns of a seeded orthogonal matrix.  With
    heads > 1 the directions mix the heads' coordinate blocks (a joint basis, the situation of Lemma 1).
    Storage-rounded; returns the stored array [n_tok, D]."""
    rng = np.random.default_rng(seed)
    dirs, _ = np.linalg.qr(rng.standard_normal((D, D)))
    sigma = decay ** (0.5 * np.arange(D))
    z = rng.standard_normal((n_tok, D))
    return store((z * sigma) @ dirs.T, dtype)

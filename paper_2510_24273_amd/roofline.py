"""Algorithmic byte / flop accounting of one SALS layer-step (host arithmetic only).

The paper's traffic model (Sec. 4.5) counts s*r_score + 2*k*r cache elements per
sequence.  The figures used for the roofline add what that model leaves out and
the path still has to move: the two projectors (read once per layer-step for the
whole batch) and the fp32 score vector (written once, read once).
"""
from __future__ import annotations

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
VALU_F32_PEAK_TFLOPS = 157.3


def paper_traffic_elements(s: int, r: int, r_score: int, k: int) -> int:
    """Sec. 4.5: cache elements SALS moves per sequence, s*r* + 2*k*r."""
    return s * r_score + 2 * k * r


def stage_bytes(w, seq_len=None) -> dict:
    """Algorithmic HBM bytes per layer-step of workload w, by stage."""
    e = w.esize
    S = getattr(w, "S_live", w.S) if seq_len is None else seq_len
    n_sel = min(S, w.k_tot)
    small = w.B * (w.H * w.d * e * 2 + w.r * 4 + n_sel * 4)   # q, out, q~, idx
    return {
        "project": w.r * w.D_kv * e,                      # U_k, once per batch
        "scores": w.B * (S * w.rs * e + 4 * S),          # K~ stream + score write
        "select": w.B * 4 * S,                            # score read
        "attend_k": w.B * n_sel * w.r * e + w.r * w.D_kv * e,   # gathered K~ rows + U_k
        # gathered V~ rows + U_v, or (quantised value cache) gathered code rows + per-group (scale, zero)
        "attend_v": (w.B * n_sel * w.r * e + w.r * w.D_kv * e) if not getattr(w, "qv_bits", 0)
        else w.B * n_sel * (w.D_kv * w.qv_bits // 8 + w.D_kv // 32 * 2 * e),
        "small": small,
        # high-precision recent window: ring rows of both caches for the recent tokens + the window's projectors
        # (with the quantised value path the window's values are 8-bit rows and only the key projector is read)
        "window": 0 if not getattr(w, "r_hi", 0) else
        (2 * w.B * min(S, w.n_recent) * w.r_hi * e + 2 * w.r_hi * w.D_kv * e) if not getattr(w, "qv_bits", 0) else
        (w.B * min(S, w.n_recent) * (w.r_hi * e + w.D_kv + w.D_kv // 32 * 2 * e) + w.r_hi * w.D_kv * e),
    }


def algorithmic_bytes(w, seq_len=None) -> int:
    """Pipeline bytes: U_k is counted once (projection and reconstruction share it)."""
    b = stage_bytes(w, seq_len)
    return b["scores"] + b["select"] + b["attend_k"] + b["attend_v"] + b["small"] + b["window"]


def stage_flops(w, seq_len=None) -> dict:
    S = getattr(w, "S_live", w.S) if seq_len is None else seq_len
    n_sel = min(S, w.k_tot)
    return {
        "project": 2 * w.B * w.r * w.D_kv,
        "scores": 2 * w.B * S * w.rs,
        "reconstruct_k": 2 * w.B * n_sel * w.r * w.D_kv,
        "reconstruct_v_literal": 2 * w.B * n_sel * w.r * w.D_kv,
        "value_reassociated": 2 * w.B * w.H * (n_sel * w.r + w.r * w.d),
        "attention": 4 * w.B * n_sel * w.H * w.d,
    }

# HBM bytes per launch (read + written) measured with rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE,
# each scaled by the same counter's reading for a 64 MiB device-to-device copy in the same run
# (FETCH_SIZE reads half of the copied bytes on this chip, WRITE_SIZE all of them).  The figures are
# read from the committed summaries profiles/hbm_traffic_<workload>.txt, so they change with those files;
# a stage that runs as several kernels is the sum of their rows.  The scaling assumes full 128-byte
# requests, so kernels that fetch 64-byte pieces are over-counted by up to 2x.
_STAGE_OF_KERNEL = (
    ("project_kernel", "project"), ("scores_kernel", "scores"), ("topk", "topk"),
    ("attend_logits", "attend_logits"), ("logits_finish", "attend_logits"), ("attend_pv", "attend_pv"),
    ("attend_out", "attend_out"), ("attend_qv", "attend_qv"), ("qv_merge", "attend_qv"),
)


def measured_traffic(workload: str, stage: str, profiles_dir: str | None = None):
    """HBM bytes per launch of `stage` at `workload` from profiles/hbm_traffic_<workload>.txt, or None when
    that summary (or a row for the stage) does not exist."""
    import os
    if profiles_dir is None:
        profiles_dir = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles")
    path = os.path.join(profiles_dir, f"hbm_traffic_{workload}.txt")
    if not os.path.exists(path):
        return None
    total, seen = 0.0, False
    with open(path) as f:
        for line in f:
            name = line.split("<")[0].split(" ")[0]
            st = next((s for k, s in _STAGE_OF_KERNEL if name.startswith(k)), None)
            cols = line.split()
            if st != stage or len(cols) < 6:
                continue
            try:
                total += (float(cols[-2]) + float(cols[-1])) * 1e6   # scaled MB read + scaled MB written
                seen = True
            except ValueError:
                continue
    return int(round(total)) if seen else None

#!/usr/bin/env python3
"""Benchmark of the SALS decode-step attention path on one MI355X.

A *step* is one decode step of the whole hot path (query projection, latent scores,
top-k, key reconstruction + RoPE, sparse attention) walked over every layer of the
workload, each layer with its own seeded synthetic caches and projectors resident in
HBM.  The headline workload is the LLaMA2-7B-shaped configuration (B=1, S=4096, r=640,
top-k=512, 32 layers); `value` is microseconds per layer-step.  Prints ONE JSON line on
stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer buffer sets (0 = workload default)")
    ap.add_argument("--extras", default="cfg3a,cfg3b,cfg4,cfg5,cfg4_rhalf,cfg2_qv4,cfg4_qv4,cfg2_comp,cfg2_win,cfg3a_win,cfg4_cap2x,cfg2_qvwin,t6_b16_s4096_12,t6w_b16_s4096_12,prefill_cfg2,prefill_cfg3b,calib_cfg3b",
                    help="other configurations reported under 'extra' (comma list, '' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense-attention baseline (full-rank cache of the same shape) timed beside each workload")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one device-to-device copy of this many MiB (a kernel of known HBM "
                         "traffic, to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


class LayerSet:
    """Device-resident inputs of every layer of a workload + one context."""

    def __init__(self, w, n_layers, torch, binding, synth):
        self.w, self.torch = w, torch
        dev = "cuda:0"

        def up(a):
            import numpy as np
            if a.dtype == np.uint16:
                return torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)
            return torch.from_numpy(a).to(dev)

        desc = binding.make_desc(w.B, w.S, w.H, w.H_kv, w.d, w.r, w.top_k, w.dtype, r_score=w.rs,
                                 n_recent=w.n_recent, n_sink=w.n_sink, rope_theta=w.theta,
                                 rope_style=w.rope_style)
        self.ctx = binding.Sals(desc, dev)
        self.win = None
        if w.r_hi:      # the recent tokens in a second, higher-rank ring cache with a context of its own
            self.win = binding.Sals(binding.make_desc(w.B, w.S, w.H, w.H_kv, w.d, w.r_hi, w.n_recent, w.dtype,
                                                      r_score=min(w.r_hi, 1024), rope_theta=w.theta,
                                                      rope_style=w.rope_style), dev)
        self.layers = []
        self.host0 = None
        for l in range(n_layers):
            L = synth.make_layer(w, l)
            if l == 0:
                self.host0 = L
            G = {k: up(v) for k, v in L.items() if hasattr(v, "dtype")}
            G["W"] = self.ctx.pack_weights(G.pop("Uk"), G.pop("Uv"))   # one-time repack, as at model load
            if w.r_hi:
                Wn = synth.make_window(w, L, l)
                G["Kw"], G["Vw"] = up(Wn["Kw"]), up(Wn["Vw"])
                G["W_hi"] = self.win.pack_weights(up(Wn["Uk_hi"]), up(Wn["Uv_hi"]))
                if w.qv_bits:   # the window's values as an 8-bit ring instead of the latent one
                    del G["Vw"]
                    cw, mw = synth.make_qv_window(w, l)
                    G["Vqw"], G["Vmeta_w"] = torch.from_numpy(cw).to(dev), up(mw)
            if w.qv_bits:   # quantised full-rank value cache in place of the latent one
                del G["Vc"]
                codes, meta = synth.make_qv_cache(w, l, w.qv_bits)
                G["Vq"], G["Vmeta"] = torch.from_numpy(codes).to(dev), up(meta)
            self.layers.append(G)
            if l % 8 == 7 or n_layers <= 4:
                log(f"  [{w.name}] layer {l + 1}/{n_layers} generated")
        torch.cuda.synchronize()
        odt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self.out = [torch.empty((w.B, w.H, w.d), dtype=odt, device=dev) for _ in range(n_layers)]

    def step(self):
        if self.win is not None and self.w.qv_bits:
            for G, o in zip(self.layers, self.out):
                self.ctx.decode_step_qv_window(self.win, G["q"], G["q_pos"], G["Kc"], G["Vq"], G["Vmeta"], self.w.qv_bits,
                                               G["W"], G["Kw"], G["Vqw"], G["Vmeta_w"], G["W_hi"], G["seq_len"], o)
            return
        if self.win is not None:
            for G, o in zip(self.layers, self.out):
                self.ctx.decode_step_window(self.win, G["q"], G["q_pos"], G["Kc"], G["Vc"], G["W"], G["Kw"], G["Vw"],
                                            G["W_hi"], G["seq_len"], o)
            return
        if self.w.qv_bits:
            for G, o in zip(self.layers, self.out):
                self.ctx.decode_step_qv(G["q"], G["q_pos"], G["Kc"], G["Vq"], G["Vmeta"], self.w.qv_bits, G["W"],
                                        G["seq_len"], o)
            return
        for G, o in zip(self.layers, self.out):
            self.ctx.decode_step(G["q"], G["q_pos"], G["Kc"], G["Vc"], G["W"], G["seq_len"], o)

    def bytes_resident(self):
        return sum(t.numel() * t.element_size() for G in self.layers for t in G.values())


class DenseSet:
    """Device-resident full-rank caches (keys as a dense model keeps them: already rotated) for the dense
    baseline at a workload's shape, generated on the device (seeded), + one context."""

    def __init__(self, w, n_layers, torch, binding):
        self.w, self.torch = w, torch
        dev = "cuda:0"
        desc = binding.make_desc(w.B, w.S, w.H, w.H_kv, w.d, w.r, w.top_k, w.dtype, rope_theta=w.theta,
                                 rope_style=w.rope_style)
        self.ctx = binding.Sals(desc, dev)
        dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        gen = torch.Generator(device=dev)
        gen.manual_seed(10_000 * w.cfg_id + 79)
        self.layers = []
        for _ in range(n_layers):
            self.layers.append({
                "q": torch.randn((w.B, w.H, w.d), generator=gen, device=dev, dtype=torch.float32).to(dt),
                "K": torch.randn((w.B, w.S, w.H_kv, w.d), generator=gen, device=dev, dtype=dt),
                "V": torch.randn((w.B, w.S, w.H_kv, w.d), generator=gen, device=dev, dtype=dt),
            })
        self.seq_len = torch.full((w.B,), w.S_live, dtype=torch.int32, device=dev)
        self.out = [torch.empty((w.B, w.H, w.d), dtype=dt, device=dev) for _ in range(n_layers)]
        torch.cuda.synchronize()

    def step(self):
        for G, o in zip(self.layers, self.out):
            self.ctx.dense_attend(G["q"], self.seq_len, G["K"], G["V"], self.seq_len, o)


def measure_dense(w, steps, warmup, use_graph, torch, binding):
    """us per layer-step of the dense baseline at w's shape (best of eager and graph replay) and its
    achieved HBM rate over the 2*B*S*D_kv cache elements it has to read."""
    per = 2 * w.B * w.S_live * w.D_kv * w.esize
    nl = max(2, min(8, int(600e6 // per) + 1))
    ds = DenseSet(w, nl, torch, binding)
    ms = timed(torch, ds.step, steps, warmup)
    if use_graph:
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            ds.step()
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                ds.step()
        torch.cuda.synchronize()
        ms = min(ms, timed(torch, g.replay, steps, warmup))
    us = ms * 1e3 / nl
    del ds
    torch.cuda.empty_cache()
    return {"us_per_layer_step": round(us, 2), "cache_bytes": per, "achieved_GBps": round(per / (us * 1e-6) / 1e9, 1),
            "hbm_frac": round(per / (us * 1e-6) / 1e9 / 8000.0, 4)}


def measure_prefill(w, steps, torch, binding, roofline):
    """Bulk compression of a whole prompt of w.S tokens per sequence (the prefill-time GEMM K~ = K U_k, V~ = V U_v):
    average kernel duration from the library's own event pairs, against the bf16 matrix peak."""
    dev = "cuda:0"
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    desc = binding.make_desc(w.B, w.S, w.H, w.H_kv, w.d, w.r, w.top_k, w.dtype, rope_theta=w.theta)
    ctx = binding.Sals(desc, dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(10_000 * w.cfg_id + 81)
    U = [torch.randn((w.D_kv, w.r), generator=gen, device=dev, dtype=torch.float32).to(dt) * (w.D_kv ** -0.5) for _ in range(2)]
    W = ctx.pack_weights(U[0], U[1])
    nset = max(2, min(6, int(600e6 // (2 * w.B * w.S * w.D_kv * w.esize)) + 1))
    X = [[torch.randn((w.B, w.S, w.D_kv), generator=gen, device=dev, dtype=dt) for _ in range(2)] for _ in range(nset)]
    Kc = torch.empty((w.B, w.S, w.r), dtype=dt, device=dev)
    Vc = torch.empty_like(Kc)
    sl = torch.zeros((w.B,), dtype=torch.int32, device=dev)
    for i in range(2):
        sl.zero_()
        ctx.compress_prefill(X[i % nset][0], X[i % nset][1], W, Kc, Vc, sl, w.S)
    torch.cuda.synchronize()
    ctx.profile(True)
    for i in range(steps):
        sl.zero_()
        ctx.compress_prefill(X[i % nset][0], X[i % nset][1], W, Kc, Vc, sl, w.S)
    torch.cuda.synchronize()
    ms, n = ctx.profile_collect()["prefill"]
    ctx.profile(False)
    us = ms * 1e3 / max(n, 1)
    flops = 2 * 2 * w.B * w.S * w.D_kv * w.r
    byts = 2 * (w.B * w.S * (w.D_kv + w.r) + w.D_kv * w.r) * w.esize
    peak = roofline.MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else roofline.VALU_F32_PEAK_TFLOPS
    ctx.close()
    del X
    torch.cuda.empty_cache()
    return {"workload": f"prefill_{w.name}", "tokens": w.B * w.S, "us_per_call": round(us, 2), "flops": flops,
            "achieved_TFLOPs": round(flops / (us * 1e-6) / 1e12, 1), "mfma_frac": round(flops / (us * 1e-6) / 1e12 / peak, 4),
            "bytes": byts, "hbm_frac": round(byts / (us * 1e-6) / 1e9 / roofline.HBM_PEAK_GBPS, 4)}


def measure_calibration(w, n_tok, steps, torch, binding, roofline):
    """Offline calibration at the key width of configuration w: covariance of n_tok synthetic calibration keys (timed
    with events on the launch stream, against the bf16 matrix peak) and the r leading eigenvectors (wall time of the
    blocking call; every Jacobi step reads and writes the whole fp64 matrix once, so the figure next to it is that
    stream's bytes per second: a matrix of up to 4096 rows stays in the 256 MB last-level cache, which is why the
    figure can exceed what HBM delivers)."""
    dev = "cuda:0"
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    D = w.D_kv
    gen = torch.Generator(device=dev)
    gen.manual_seed(10_000 * w.cfg_id + 91)
    # planted spectrum (eigenvalues decaying like 1/(c+1)) along seeded directions, generated on the device
    dirs = torch.linalg.qr(torch.randn((D, D), generator=gen, device=dev, dtype=torch.float32))[0]
    sigma = (torch.arange(1, D + 1, device=dev, dtype=torch.float32)) ** -0.5
    X = ((torch.randn((n_tok, D), generator=gen, device=dev, dtype=torch.float32) * sigma) @ dirs.T).to(dt)
    C = torch.zeros((D, D), dtype=torch.float64, device=dev)
    ws = binding.calib_accumulate(X, C)           # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    C.zero_()
    e0.record()
    for _ in range(steps):
        ws = binding.calib_accumulate(X, C)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / steps
    flops = 2 * n_tok * D * D
    peak = roofline.MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else roofline.VALU_F32_PEAK_TFLOPS
    C.div_(steps)
    t0 = time.perf_counter()
    lam, U, sweeps = binding.calib_eigenvectors(C, w.r, dt)
    torch.cuda.synchronize()
    eig_ms = (time.perf_counter() - t0) * 1e3
    n_steps = abs(sweeps) * (D - 1)
    step_bytes = 2 * D * D * 8    # every step reads and writes the whole matrix once
    del X, ws, dirs
    torch.cuda.empty_cache()
    return {"workload": f"calib_{w.name}", "D": D, "r": w.r, "tokens": n_tok, "covariance_us_per_call": round(us, 1),
            "covariance_flops": flops, "covariance_TFLOPs": round(flops / (us * 1e-6) / 1e12, 1),
            "covariance_mfma_frac": round(flops / (us * 1e-6) / 1e12 / peak, 4),
            "eigenvectors_ms": round(eig_ms, 1), "sweeps": sweeps, "jacobi_steps": n_steps,
            "jacobi_us_per_step": round(eig_ms * 1e3 / max(n_steps, 1), 2),
            "jacobi_matrix_GBps": round(step_bytes * n_steps / (eig_ms * 1e-3) / 1e9, 1),
            "lambda_ratio_r": float(lam[w.r - 1] / lam[0])}


def timed(torch, fn, steps, warmup):
    """ms per call of fn(): `warmup` untimed calls, then exactly `steps` timed ones."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_table(ls, steps, roofline, wall_us_per_layer_step):
    """Per-kernel average duration (us) over `steps` profiled steps + roofline figures.

    The library brackets every stage with a pair of HIP events on the launch stream.  A bracket also
    contains the gap between the previous kernel's end and this kernel's start, which back-to-back
    launches otherwise overlap; that gap is estimated live as (sum of bracketed times - wall time of the
    same un-profiled step) / brackets and taken off every stage ("us"; "us_events" is the raw reading).
    """
    torch, w = ls.torch, ls.w
    # three profiled rounds, per stage the smallest average: one stray stall (another process, a page
    # fault) would otherwise land in whichever bracket it hit and skew the gap estimate
    ls.ctx.profile(True)
    prof = None
    for _ in range(3):
        for _ in range(steps):
            ls.step()
        torch.cuda.synchronize()
        p1 = ls.ctx.profile_collect()
        prof = p1 if prof is None else {k: (min(prof[k], p1[k], key=lambda mn: mn[0] / max(mn[1], 1))) for k in p1}
    ls.ctx.profile(False)
    sb, sf = roofline.stage_bytes(w), roofline.stage_flops(w)
    model = {
        "project": ("hbm", sb["project"]),
        "scores": ("hbm", sb["scores"]),
        "topk": ("hbm", sb["select"] + w.B * w.k_tot * 4),
        "attend_logits": ("mfma", sf["reconstruct_k"]),
        "attend_pv": ("hbm", w.B * w.k_tot * w.r * w.esize),
        "attend_out": ("hbm", w.r * w.D_kv * w.esize),
        "attend_qv": ("hbm", w.B * w.k_tot * (w.D_kv * max(w.qv_bits, 1) // 8 + w.D_kv // 32 * 2 * w.esize)),
    }
    raw = {name: ms * 1e3 / n for name, (ms, n) in prof.items() if n > 0}
    gap = max(0.0, (sum(raw.values()) - wall_us_per_layer_step) / max(1, len(raw)))
    rows = {}
    for name, us_ev in raw.items():
        us = max(us_ev - gap, 0.25 * us_ev)
        bound, work = model[name]
        if bound == "hbm":
            ach, peak, unit = work / (us * 1e-6) / 1e9, roofline.HBM_PEAK_GBPS, "GB/s"
        else:
            peak = roofline.MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else roofline.VALU_F32_PEAK_TFLOPS
            ach, unit = work / (us * 1e-6) / 1e12, "TFLOP/s"
        rows[name] = {"us": round(us, 3), "us_events": round(us_ev, 3), "launches": prof[name][1], "bound": bound,
                      "work": int(work), "achieved": round(ach, 2), "peak": peak, "unit": unit,
                      "frac": round(ach / peak, 4)}
    return rows, gap


def measure(ls, steps, warmup, use_graph, roofline):
    torch, w = ls.torch, ls.w
    n_layers = len(ls.layers)
    eager_ms = timed(torch, ls.step, steps, warmup)
    res = {"eager_ms_per_step": eager_ms, "graph_ms_per_step": None}
    if use_graph:
        ref = [o.clone() for o in ls.out]
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            ls.step()
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                ls.step()
        torch.cuda.synchronize()
        graph_ms = timed(torch, g.replay, steps, warmup)
        same = all(torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
                   for a, b in zip(ref, ls.out))
        res["graph_ms_per_step"] = graph_ms if same else None
        res["graph_matches_eager"] = bool(same)
    best = min(x for x in (res["eager_ms_per_step"], res["graph_ms_per_step"]) if x is not None)
    res["ms_per_step"] = best
    res["mode"] = "hip_graph" if best == res["graph_ms_per_step"] else "eager"
    res["us_per_layer_step"] = best * 1e3 / n_layers
    res["algorithmic_bytes"] = roofline.algorithmic_bytes(w)
    res["pipeline_GBps"] = res["algorithmic_bytes"] / (res["us_per_layer_step"] * 1e-6) / 1e9
    res["pipeline_hbm_frac"] = res["pipeline_GBps"] / roofline.HBM_PEAK_GBPS
    res["kernels"], res["event_gap_us"] = kernel_table(ls, max(3, steps // 3), roofline,
                                                       res["eager_ms_per_step"] * 1e3 / n_layers)
    return res


def cpu_baseline(w, host_layers, synth, budget_s=12.0):
    """The fp64 oracle, as it stands, on the host cores: whole decode steps of layer 0.."""
    from oracle import sals_oracle
    wd = synth.widen
    done, t_total = 0, 0.0
    for L in host_layers:
        t0 = time.perf_counter()
        for b in range(w.B):
            S = int(L["seq_len"][b])
            sals_oracle.decode_step(wd(L["q"][b]), S, wd(L["Kc"][b][:S]), wd(L["Vc"][b][:S]), wd(L["Uk"]),
                                    wd(L["Uv"]), w.H_kv, w.top_k, w.theta, r_score=w.rs, n_sink=w.n_sink,
                                    n_recent=w.n_recent, rope_style=w.rope_style)
        t_total += time.perf_counter() - t0
        done += 1
        if t_total > budget_s:
            break
    return {"value": round(t_total / done * 1e6, 1), "unit": "us/layer-step", "cores": sals_oracle.num_threads(),
            "kind": "oracle", "sample": f"{done} layer-step(s) of {w.name} (layers 0..{done - 1}), fp64, "
                                        f"inputs widened from the same storage-rounded arrays"}


def main():
    a = parse()
    if a.gpus != 1:
        log("bench.py: this build is single-GPU by design (one MI355X); run with --gpus 1. "
            "Sequences and layers shard trivially across GPUs, no multi-GPU figure is produced.")
        sys.exit(2)
    import torch
    from paper_2510_24273_amd import binding, roofline, synth   # fails loudly if libsals.so is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    w = synth.lookup(a.workload)
    n_layers = a.layers or w.n_layers
    if n_layers == 1:   # single-layer configs: rotate enough distinct sets to defeat the 256 MB LLC
        per = roofline.algorithmic_bytes(w) + w.r * w.D_kv * w.esize
        n_layers = max(2, min(8, int(600e6 // per) + 1))
    log(f"[bench] generating {w.name}: {n_layers} layers")
    ls = LayerSet(w, n_layers, torch, binding, synth)
    log(f"[bench] resident inputs: {ls.bytes_resident() / 1e6:.0f} MB; timing")
    res = measure(ls, a.steps, a.warmup, not a.no_graph, roofline)
    if a.calib_copy_mib > 0:
        src = torch.ones(a.calib_copy_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    kern = res["kernels"]
    dom = max(kern, key=lambda k: kern[k]["us"])
    dk = kern[dom]
    traffic = roofline.measured_traffic(a.workload, dom)   # from profiles/hbm_traffic_<workload>.txt, None if absent
    out = {
        "metric": "sals_decode_attn_us_per_layer_step", "value": round(res["us_per_layer_step"], 3),
        "unit": "us", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(res["ms_per_step"], 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers_per_step": n_layers, "B": w.B, "S": w.S, "H": w.H,
                   "H_kv": w.H_kv, "d": w.d, "r": w.r, "r_score": w.rs, "top_k": w.top_k,
                   "n_recent": w.n_recent, "launch": res["mode"],
                   "eager_us_per_layer_step": round(res["eager_ms_per_step"] * 1e3 / n_layers, 3),
                   "graph_us_per_layer_step": None if res["graph_ms_per_step"] is None
                   else round(res["graph_ms_per_step"] * 1e3 / n_layers, 3)},
        "pipeline": {"algorithmic_bytes": res["algorithmic_bytes"], "achieved_GBps": round(res["pipeline_GBps"], 1),
                     "hbm_peak_GBps": roofline.HBM_PEAK_GBPS, "frac": round(res["pipeline_hbm_frac"], 4)},
        "roofline": {"kernel": dom, "bound": dk["bound"], "achieved": dk["achieved"], "peak": dk["peak"],
                     "unit": dk["unit"], "frac": dk["frac"], "traffic": traffic, "avg_us": dk["us"],
                     "avg_us_events": dk["us_events"], "event_gap_us": round(res["event_gap_us"], 3)},
        "kernels": kern,
    }
    dense_done = {}
    if not a.no_dense:
        log("[bench] dense baseline at the same shape")
        out["dense_baseline"] = measure_dense(w, max(5, a.steps // 2), 2, not a.no_graph, torch, binding)
        out["dense_baseline"]["speedup_of_sals"] = round(out["dense_baseline"]["us_per_layer_step"] / out["value"], 3)
        dense_done[(w.B, w.S, w.S_live, w.H, w.H_kv, w.dtype)] = out["dense_baseline"]
    if not a.no_cpu_baseline:
        log("[bench] timing the CPU oracle")
        host = [ls.host0] + [synth.make_layer(w, l) for l in range(1, min(3, n_layers))] if w.B == 1 else [ls.host0]
        out["cpu_baseline"] = cpu_baseline(w, host, synth)
    del ls
    torch.cuda.empty_cache()
    extra = {}
    for name in [x for x in a.extras.split(",") if x and x != a.workload]:
        if name.startswith("prefill_"):   # the prompt of that configuration compressed in one call
            log(f"[bench] extra {name}")
            extra[name] = measure_prefill(synth.lookup(name[len("prefill_"):]), max(5, a.steps // 3), torch, binding, roofline)
            continue
        if name.startswith("calib_"):     # offline calibration at that configuration's key width and rank
            log(f"[bench] extra {name}")
            extra[name] = measure_calibration(synth.lookup(name[len("calib_"):]), 65536, max(3, a.steps // 6), torch, binding, roofline)
            continue
        we = synth.lookup(name)
        per = roofline.algorithmic_bytes(we) + we.r * we.D_kv * we.esize
        nl = max(2, min(8, int(600e6 // per) + 1))
        log(f"[bench] extra {we.name}: {nl} layer sets")
        lse = LayerSet(we, nl, torch, binding, synth)
        r = measure(lse, max(5, a.steps // 3), 2, not a.no_graph, roofline)
        extra[name] = {"workload": we.name, "us_per_layer_step": round(r["us_per_layer_step"], 2),
                       "launch": r["mode"], "algorithmic_bytes": r["algorithmic_bytes"],
                       "achieved_GBps": round(r["pipeline_GBps"], 1), "hbm_frac": round(r["pipeline_hbm_frac"], 4),
                       "kernels_us": {k: v["us"] for k, v in r["kernels"].items()},
                       "kernels_frac": {k: v["frac"] for k, v in r["kernels"].items()}}
        del lse
        torch.cuda.empty_cache()
        if not a.no_dense and we.fill == 1.0:   # (a cache with spare capacity: the dense baseline of the full one applies)
            key = (we.B, we.S, we.S_live, we.H, we.H_kv, we.dtype)
            if key not in dense_done:
                dense_done[key] = measure_dense(we, max(5, a.steps // 3), 2, not a.no_graph, torch, binding)
            extra[name]["dense_us_per_layer_step"] = dense_done[key]["us_per_layer_step"]
            extra[name]["dense_hbm_frac"] = dense_done[key]["hbm_frac"]
            extra[name]["speedup_vs_dense"] = round(dense_done[key]["us_per_layer_step"] / r["us_per_layer_step"], 3)
    if extra:
        out["extra"] = extra
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

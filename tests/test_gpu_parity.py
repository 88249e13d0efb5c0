"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by
element, on seeded synthetic workloads.

Tolerances: selected index sets bit-exact against the oracle's rule applied to the same
fp32 scores, and against the fp64 oracle wherever its k-th/(k+1)-th score gap exceeds
1e-3 relative; outputs within max-abs 2e-2 (bf16) / 1e-4 (fp32) and within the tighter
bound derived in tests/gpu_util.py::out_tolerances.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2510_24273_amd import synth  # noqa: E402
from tests import gpu_util as gu  # noqa: E402

C = synth.CONFIGS


def _run(oracle, w, layer=0, seq_lens=None, seqs=None, label=""):
    print(f"[case] {label or w.name} layer={layer} seq_lens={seq_lens}", flush=True)
    L = synth.make_layer(w, layer, seq_lens)
    ctx = gu.make_ctx(w)
    G = gu.upload(L, ctx)
    R = gu.run_stages(ctx, w, G)
    # the fused entry point must reproduce the staged calls bit for bit
    out2 = torch.empty_like(R["out"])
    idx2 = torch.empty_like(R["idx"])
    n2 = torch.empty_like(R["n_sel"])
    ctx.decode_step(G["q"], G["q_pos"], G["Kc"], G["Vc"], G["W"], G["seq_len"], out2,
                    None, idx2, n2)
    torch.cuda.synchronize()
    assert torch.equal(idx2, R["idx"]) and torch.equal(n2, R["n_sel"])
    assert torch.equal(out2.view(torch.int16) if out2.dtype == torch.bfloat16 else out2,
                       R["out"].view(torch.int16) if out2.dtype == torch.bfloat16 else R["out"])
    figs = []
    for b in (range(w.B) if seqs is None else seqs):
        figs.append(gu.check_sequence(oracle, w, L, R, b))
    print("   ", figs[0], flush=True)
    ctx.close()
    return L, R, figs


# ---- configuration 1: the tiny fp32 case, whole --------------------------------------

def test_cfg1_tiny_f32(oracle):
    _run(oracle, C["cfg1"])


# ---- small cases that span several tiles and ragged tails ----------------------------

SMALL = synth.shrink(C["cfg2"], B=3, S=1000, r=192, top_k=100, n_layers=1, plant=2)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_ragged_batch(oracle, dtype):
    w = synth.shrink(SMALL, dtype=dtype)
    # full, odd length, shorter than k_tot
    _run(oracle, w, seq_lens=[1000, 777, 61])


def test_empty_and_single_token_sequences(oracle):
    w = synth.shrink(SMALL, B=4, plant=0)
    _run(oracle, w, seq_lens=[0, 1, 100, 101])


def test_gqa_groups(oracle):
    for H, H_kv in ((32, 8), (8, 1), (16, 16)):
        w = synth.shrink(SMALL, H=H, H_kv=H_kv, B=2, S=600)
        _run(oracle, w, seq_lens=[600, 333], label=f"gqa H={H} H_kv={H_kv}")


@pytest.mark.parametrize("rows", [16, 48, 128])
def test_capacity_above_length(oracle, rows, monkeypatch):
    """A cache allocated for more tokens than it holds: the score kernel stops loading at the sequence length
    (after the first 16-row pass of each workgroup, which is requested before the length is known) and fills the
    rest with -inf.  Lengths on both sides of every boundary of that logic: inside a workgroup's first pass, at a
    pass boundary, at a workgroup boundary, mid-range, empty, full; `rows` = cache rows per workgroup."""
    monkeypatch.setenv("SALS_TUNE_SCORE_ROWS", str(rows))
    w = synth.shrink(SMALL, B=6, S=3000, r=128, top_k=40, plant=0)
    _run(oracle, w, seq_lens=[3000, 2 * rows, 2 * rows + 1, 2 * rows + 16, 5, 1537], label=f"capacity rows={rows} a")
    _run(oracle, w, seq_lens=[0, 2999, 2 * rows - 1, 3 * rows + 17, 16, 2048], label=f"capacity rows={rows} b")


def test_odd_sizes(oracle):
    """A cache capacity that is not a multiple of 4 (score rows of later sequences start unaligned), an odd
    selection budget, an odd multiple of 8 as scoring rank."""
    w = synth.shrink(SMALL, B=3, S=997, top_k=97, n_sink=3, n_recent=5, r=192, r_score=72, plant=0)
    _run(oracle, w, seq_lens=[997, 501, 106], label="S_max=997")
    for dtype in ("bf16", "f32"):
        wq = synth.shrink(w, dtype=dtype)
        _run(oracle, wq, seq_lens=[997, 104, 105], label=f"S_max=997 {dtype}, cache barely longer than the selection")


def test_sixty_four_query_heads(oracle):
    """H_q = 64, the most the kernels take: as 64 KV heads, and as 8 groups of 8."""
    for H_kv in (64, 8):
        w = synth.shrink(SMALL, H=64, H_kv=H_kv, B=2, S=500, plant=0)
        _run(oracle, w, seq_lens=[500, 129], label=f"H=64 H_kv={H_kv}")


def test_truncated_scoring_rank(oracle):
    w = synth.shrink(SMALL, r=256, r_score=128, B=2)
    _run(oracle, w, seq_lens=[1000, 500])
    w = synth.shrink(SMALL, r=256, r_score=8, B=1, plant=0)
    _run(oracle, w)


def test_sink_and_recent_window(oracle):
    w = synth.shrink(SMALL, top_k=432, n_sink=16, n_recent=64, S=2048, B=2)
    L, R, _ = _run(oracle, w, seq_lens=[2048, 513])
    idx = gu.from_dev(R["idx"])
    assert idx[0, :16].tolist() == list(range(16))
    assert idx[0, -64:].tolist() == list(range(2048 - 64, 2048))


def test_interleaved_rope_and_large_theta(oracle):
    w = synth.shrink(SMALL, rope_style=1, theta=500000.0, B=1)
    _run(oracle, w)


def test_peaky_softmax_stress(oracle):
    """Caches scaled up so that logits spread over tens of units (near one-hot softmax)."""
    w = synth.shrink(SMALL, scale=30.0, B=2, plant=0)
    _run(oracle, w, seq_lens=[1000, 900])


def test_exact_ties_resolve_to_smaller_index(oracle):
    """Duplicate cache rows give bit-equal scores; the cut must keep the smaller indices."""
    w = synth.shrink(SMALL, B=1, S=512, top_k=64, plant=0)
    L = synth.make_layer(w)
    L["Kc"][0, 1::2] = L["Kc"][0, 0::2]          # rows 2m and 2m+1 identical
    ctx = gu.make_ctx(w)
    G = gu.upload(L, ctx)
    R = gu.run_stages(ctx, w, G)
    s = gu.from_dev(R["scores"][0])
    assert np.array_equal(s[0::2], s[1::2])
    gu.check_sequence(oracle, w, L, R, 0)
    # all scores equal: the first top_k tokens win
    scores = torch.zeros((1, 512), dtype=torch.float32, device=gu.DEV)
    scores[0, 100] = -0.0
    idx = torch.empty((1, 64), dtype=torch.int32, device=gu.DEV)
    n = torch.empty((1,), dtype=torch.int32, device=gu.DEV)
    ctx.topk_select(scores, G["seq_len"], idx, n)
    torch.cuda.synchronize()
    assert sorted(idx[0].tolist()) == list(range(64))
    ctx.close()


@pytest.mark.parametrize("case", ["random", "ragged", "plateaus", "constant", "short", "nonfinite"])
def test_long_sequence_selection(oracle, case):
    """S_max above 32768 takes the multi-workgroup selection; its index set must equal the
    oracle's on the same fp32 scores (the oracle's rule: larger score first, ties to the smaller
    index).  "plateaus" crowds the threshold bin and "constant" has an empty score range: both go
    through the single-workgroup kernel that the chain falls back to, as does "short" (a cache no
    longer than the selection) and a row holding infinities."""
    S, top_k, n_sink, n_recent = 40000, 300, 4, 16
    w = synth.shrink(SMALL, B=2, S=S, top_k=top_k, n_sink=n_sink, n_recent=n_recent, plant=0)
    rng = np.random.default_rng(11)
    sc = rng.standard_normal((2, S)).astype(np.float32) * 3.0
    seq = np.array([S, S], np.int32)
    if case == "ragged":
        seq = np.array([S - 7, 33001], np.int32)
    elif case == "plateaus":
        sc = np.round(sc)                      # a few dozen distinct values, thousands of ties each
    elif case == "constant":
        sc[:] = 1.25
        sc[1, 5000] = -0.0
        sc[1, :5000] = 0.0
        sc[1, 5001:] = 0.0
    elif case == "short":
        seq = np.array([top_k + n_sink + n_recent, 17], np.int32)
    elif case == "nonfinite":
        sc[0, 123] = np.inf
        sc[0, 456] = -np.inf
    ctx = gu.make_ctx(w)
    k_tot = top_k + n_sink + n_recent
    idx = torch.full((2, k_tot), -7, dtype=torch.int32, device=gu.DEV)
    n = torch.full((2,), -7, dtype=torch.int32, device=gu.DEV)
    d_sc = torch.from_numpy(sc).to(gu.DEV)
    ctx.topk_select(d_sc, torch.from_numpy(seq).to(gu.DEV), idx, n)
    torch.cuda.synchronize()
    for b in range(2):
        want = oracle.topk(sc[b, :seq[b]].astype(np.float64), top_k, n_sink, n_recent)
        got = idx[b, :int(n[b])].cpu().numpy()
        assert int(n[b]) == len(want), (case, b)
        assert np.array_equal(np.sort(got), np.sort(want)), (case, b)
    ctx.close()


def test_selection_random_shapes(oracle):
    """Seeded sweep over cache capacities up to 70000 (all four per-thread key counts of the single-workgroup
    kernel and the multi-workgroup chain), budgets, windows, ragged lengths and tie densities: the selected
    set must equal the oracle's on the same fp32 scores, bit for bit."""
    rng = np.random.default_rng(2024)
    caps = [5, 64, 1000, 4096, 4100, 8192, 9000, 16384, 20000, 32768, 33000, 70000]
    for case, S_max in enumerate(caps * 2):
        B = int(rng.integers(1, 4))
        top_k = int(rng.integers(1, max(2, min(S_max, 3000))))
        n_sink = int(rng.integers(0, 5))
        n_recent = int(rng.integers(0, 70)) if S_max > 200 else 0
        w = synth.shrink(SMALL, B=B, S=S_max, top_k=top_k, n_sink=n_sink, n_recent=n_recent, plant=0)
        sc = rng.standard_normal((B, S_max)).astype(np.float32)
        mode = case % 3
        if mode == 1:
            sc = np.round(sc * 4) / 4                      # dense ties
        elif mode == 2:
            sc = sc * np.float32(1e-3) + np.float32(7.0)   # narrow range far from zero
        seq = rng.integers(0, S_max + 1, size=B).astype(np.int32)
        seq[0] = S_max
        print(f"[case] selection S_max={S_max} B={B} top_k={top_k} sink={n_sink} recent={n_recent} mode={mode} "
              f"seq={seq.tolist()}", flush=True)
        ctx = gu.make_ctx(w)
        idx = torch.full((B, w.k_tot), -7, dtype=torch.int32, device=gu.DEV)
        n = torch.full((B,), -7, dtype=torch.int32, device=gu.DEV)
        ctx.topk_select(torch.from_numpy(sc).to(gu.DEV), torch.from_numpy(seq).to(gu.DEV), idx, n)
        torch.cuda.synchronize()
        for b in range(B):
            want = oracle.topk(sc[b, :seq[b]].astype(np.float64), top_k, n_sink, n_recent)
            got = idx[b, :int(n[b])].cpu().numpy()
            assert int(n[b]) == len(want), (S_max, b)
            assert np.array_equal(np.sort(got), np.sort(want)), (S_max, b)
            assert np.all(idx[b, int(n[b]):].cpu().numpy() == 0)
        ctx.close()


def test_decode_random_shapes(oracle):
    """Seeded sweep over descriptors: ranks, head layouts, batch sizes, budgets, windows, both storage types
    and both RoPE pairings; every stage of every sequence against the oracle."""
    rng = np.random.default_rng(77)
    for case in range(14):
        H_kv = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
        G = int(rng.choice([g for g in (1, 2, 3, 4, 8) if g * H_kv <= 64]))
        B = int(rng.integers(1, 5))
        r = 64 * int(rng.integers(1, 9))
        S = int(rng.integers(40, 2500))
        top_k = int(rng.integers(1, min(S, 700)))
        w = synth.shrink(SMALL, B=B, S=S, H=H_kv * G, H_kv=H_kv, r=r, r_score=8 * int(rng.integers(1, r // 8 + 1)),
                         top_k=top_k, n_sink=int(rng.integers(0, 4)), n_recent=int(rng.integers(0, 20)),
                         dtype=str(rng.choice(["bf16", "f32"])), rope_style=int(rng.integers(0, 2)),
                         theta=float(rng.choice([1e4, 5e5])), plant=int(rng.integers(0, 3)))
        seq = rng.integers(0, S + 1, size=B).tolist()
        seq[0] = S
        _run(oracle, w, seq_lens=seq, label=f"random #{case}: B={B} S={S} H={w.H}/{H_kv} r={r}/{w.rs} k={top_k} "
                                            f"{w.dtype} style={w.rope_style}")


def test_maximum_sizes(oracle):
    """The descriptor's upper limits in one case: a 2^20-row cache (128 selection chunks, the largest
    cos/sin table), 65536 selected tokens with sinks and a recent window, at the smallest rank."""
    w = synth.shrink(SMALL, B=1, S=1 << 20, H=8, H_kv=1, r=64, top_k=65536 - 16 - 64, n_sink=16, n_recent=64,
                     plant=0)
    _run(oracle, w, label="max S_max and k_tot")


def test_maximum_rank_and_batch_columns(oracle):
    """r = r_score = 1024 (the largest scoring rank), r = 2048 (the largest rank) in both storage types, and
    B * (H_q / H_kv) = 128 (the widest projection)."""
    _run(oracle, synth.shrink(SMALL, B=2, S=700, r=1024, plant=0), seq_lens=[700, 257], label="r=1024")
    _run(oracle, synth.shrink(SMALL, B=2, S=700, r=2048, r_score=1024, plant=0), seq_lens=[700, 257], label="r=2048")
    _run(oracle, synth.shrink(SMALL, B=1, S=300, r=2048, r_score=512, top_k=70, H=16, H_kv=16, plant=0, dtype="f32"),
         label="r=2048 f32")
    _run(oracle, synth.shrink(SMALL, B=16, S=300, H=8, H_kv=1, r=128, top_k=40, plant=0), seqs=[0, 15],
         label="B*G=128")


def test_compress_append_then_decode(oracle):
    """Algorithm 1 in order: compress the new token, append, then attend with the query on
    the appended row (q_pos = seq_len - 1)."""
    w = synth.shrink(SMALL, B=2, S=400, plant=0)
    L = synth.make_layer(w, seq_lens=[399, 200])
    G = gu.upload(L)
    rng = np.random.default_rng(5)
    k_new = synth.store(rng.standard_normal((w.B, w.D_kv)), w.dtype)
    v_new = synth.store(rng.standard_normal((w.B, w.D_kv)), w.dtype)
    ctx = gu.make_ctx(w)
    G["W"] = ctx.pack_weights(G["Uk"], G["Uv"])
    for rep in range(2):           # second call: sequence 0 is full and must be left alone
        before = G["Kc"].clone()
        ctx.compress_append(gu.to_dev(k_new), gu.to_dev(v_new), G["W"], G["Kc"], G["Vc"],
                            G["seq_len"])
        torch.cuda.synchronize()
        if rep == 0:
            assert G["seq_len"].tolist() == [400, 201]
            for b, row in ((0, 399), (1, 200)):
                for new, U, cache in ((k_new, "Uk", "Kc"), (v_new, "Uv", "Vc")):
                    want = oracle.project(synth.widen(new[b]), synth.widen(L[U]))
                    got = gu.from_dev(G[cache][b, row])
                    ulp = np.maximum(np.abs(want), 1e-30) * 2.0 ** -7     # one bf16 ulp
                    assert np.all(np.abs(got - want) <= ulp + 1e-6)
        else:
            assert G["seq_len"].tolist() == [400, 202]
            assert torch.equal(before[0].view(torch.int16), G["Kc"][0].view(torch.int16))
    # decode with the query sitting on the last appended row
    L2 = dict(L)
    for kname in ("Kc", "Vc"):
        t = G[kname].cpu()
        L2[kname] = t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()
    L2["seq_len"] = G["seq_len"].cpu().numpy()
    L2["q_pos"] = (L2["seq_len"] - 1).astype(np.int32)
    G["q_pos"] = gu.to_dev(L2["q_pos"])
    R = gu.run_stages(ctx, w, G)
    for b in range(w.B):
        gu.check_sequence(oracle, w, L2, R, b)
    ctx.close()


def test_query_position_beyond_the_cache(oracle):
    """q_pos far above S_max: the query's angles are then evaluated in the kernel instead of
    being read from the per-context cos/sin table."""
    w = synth.shrink(SMALL, B=2)
    L = synth.make_layer(w)
    L["q_pos"] = np.array([w.S + 1, 1_000_003], np.int32)
    ctx = gu.make_ctx(w)
    G = gu.upload(L, ctx)
    R = gu.run_stages(ctx, w, G)
    for b in range(w.B):
        gu.check_sequence(oracle, w, L, R, b)
    ctx.close()


def test_graph_replays_match_eager(oracle):
    """decode_step captured in a HIP graph: every replay (with eager work and synchronisations of the same
    context in between, and the inputs changed between replays) equals the eager result bit for bit."""
    w = synth.shrink(SMALL, B=2, S=1500, top_k=300, plant=1)
    ctx = gu.make_ctx(w)
    Ls = [synth.make_layer(w, layer) for layer in range(3)]
    Gs = [gu.upload(L, ctx) for L in Ls]
    eager = []
    for G in Gs:
        o = torch.empty((w.B, w.H, w.d), dtype=gu.out_dtype(w), device=gu.DEV)
        ctx.decode_step(G["q"], G["q_pos"], G["Kc"], G["Vc"], G["W"], G["seq_len"], o)
        eager.append(o)
    torch.cuda.synchronize()
    # static buffers the graph reads; refilled before every replay
    S = {k: Gs[0][k].clone() for k in ("q", "q_pos", "Kc", "Vc", "W", "seq_len")}
    out = torch.empty_like(eager[0])
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ctx.decode_step(S["q"], S["q_pos"], S["Kc"], S["Vc"], S["W"], S["seq_len"], out)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=side):
            ctx.decode_step(S["q"], S["q_pos"], S["Kc"], S["Vc"], S["W"], S["seq_len"], out)
    torch.cuda.synchronize()
    for rep in (1, 2, 0, 1):
        for k in S:
            S[k].copy_(Gs[rep][k])
        out.fill_(7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager[rep].view(torch.int16)), f"replay on layer {rep} differs"
        # eager work of the same context between the replays
        tmp = torch.empty_like(out)
        ctx.decode_step(Gs[2]["q"], Gs[2]["q_pos"], Gs[2]["Kc"], Gs[2]["Vc"], Gs[2]["W"], Gs[2]["seq_len"], tmp)
        torch.cuda.synchronize()
        assert torch.equal(tmp.view(torch.int16), eager[2].view(torch.int16))
    ctx.close()


def test_repeatable_bit_for_bit(oracle):
    w = synth.shrink(SMALL, B=2)
    L = synth.make_layer(w)
    ctx = gu.make_ctx(w)
    G = gu.upload(L, ctx)
    first = gu.run_stages(ctx, w, G)
    for _ in range(5):
        again = gu.run_stages(ctx, w, G)
        assert torch.equal(first["scores"], again["scores"])
        assert torch.equal(first["idx"], again["idx"])
        assert torch.equal(first["out"].view(torch.int16), again["out"].view(torch.int16))
    ctx.close()


# ---- the measured configurations at full size ----------------------------------------

def test_fp32_cache_large_enough_for_the_streaming_loads(oracle):
    """An fp32 cache of 32 MB and more takes the score kernel's read-once loads (the bf16 form runs at every batch
    configuration): all stages against the oracle."""
    w = synth.shrink(C["cfg1"], B=2, S=16384, r=256, top_k=64, plant=2)
    assert w.B * w.S * w.r * 4 >= 32 << 20
    _run(oracle, w, seq_lens=[16384, 9000], label="fp32, 33.5 MB cache")


def test_cfg2_full(oracle):
    L, R, _ = _run(oracle, C["cfg2"], layer=0)
    sel = set(gu.from_dev(R["idx"][0]).tolist())
    assert set(L["planted"][0].tolist()) <= sel
    _run(oracle, C["cfg2"], layer=17)


@pytest.mark.parametrize("name", ["cfg3a", "cfg3b"])
def test_cfg3_full_every_sequence(oracle, name):
    L, R, _ = _run(oracle, C[name])
    for b in range(C[name].B):
        assert set(L["planted"][b].tolist()) <= set(gu.from_dev(R["idx"][b]).tolist())


def test_cfg4_full_every_sequence(oracle):
    _run(oracle, C["cfg4"])


def test_cfg5_full(oracle):
    L, R, _ = _run(oracle, C["cfg5"])
    idx = gu.from_dev(R["idx"][0])
    S = C["cfg5"].S
    assert idx[-64:].tolist() == list(range(S - 64, S)) and len(idx) == 4160


# ---- context set-up: the cos/sin table -------------------------------------------------

def test_unprepared_context_fills_its_table_lazily_and_refuses_capture(oracle):
    """A context made through the C ABI without sals_prepare: the first attend call fills the table on its own
    stream, a call on another stream is ordered behind it, results equal a prepared context's; under graph capture
    an unprepared context is refused before anything is enqueued."""
    import ctypes
    from paper_2510_24273_amd import binding
    w = synth.shrink(SMALL, B=2, plant=0)
    L = synth.make_layer(w)
    ctx = gu.make_ctx(w)                      # prepared (the binding does it)
    G = gu.upload(L, ctx)
    want = gu.run_stages(ctx, w, G)
    lib = binding._lib

    def raw_ctx():
        ws = torch.zeros(binding.workspace_bytes(ctx.desc), dtype=torch.uint8, device=gu.DEV)
        h = ctypes.c_void_p()
        assert lib.sals_create(ctypes.byref(ctx.desc), ws.data_ptr(), ws.numel(), ctypes.byref(h)) == binding.SALS_OK
        return h, ws

    def attend(h, stream, out):
        return lib.sals_sparse_attend(h, G["q"].data_ptr(), G["q_pos"].data_ptr(), G["Kc"].data_ptr(), G["Vc"].data_ptr(),
                                      G["W"].data_ptr(), want["idx"].data_ptr(), want["n_sel"].data_ptr(), out.data_ptr(),
                                      stream.cuda_stream)

    # lazily, first on a side stream, then at once on the default stream
    h, ws = raw_ctx()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    o1, o2 = torch.empty_like(want["out"]), torch.empty_like(want["out"])
    assert attend(h, side, o1) == binding.SALS_OK
    assert attend(h, torch.cuda.current_stream(), o2) == binding.SALS_OK
    torch.cuda.synchronize()
    for o in (o1, o2):
        assert torch.equal(o.view(torch.int16), want["out"].view(torch.int16))
    lib.sals_destroy(h)
    # refused under capture while unprepared; accepted after sals_prepare
    h, ws = raw_ctx()
    o3 = torch.empty_like(want["out"])
    g = torch.cuda.CUDAGraph()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    codes = []
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            codes.append(attend(h, s, o3))
            if codes[0] != binding.SALS_OK:
                o3.fill_(0)              # (something to capture, so that the capture itself is well formed)
    torch.cuda.synchronize()
    assert codes[0] == binding.SALS_ERR_HIP or codes[0] == binding.SALS_ERR_INVALID_ARG
    assert lib.sals_prepare(h, torch.cuda.current_stream().cuda_stream) == binding.SALS_OK
    g2 = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g2, stream=s):
            assert attend(h, s, o3) == binding.SALS_OK
    o3.fill_(7.0)
    g2.replay()
    torch.cuda.synchronize()
    assert torch.equal(o3.view(torch.int16), want["out"].view(torch.int16))
    lib.sals_destroy(h)
    ctx.close()

"""GPU parity of the prefill-time bulk compression (Eq. 1 over a whole prompt) against the oracle's
projection applied row by row: every written cache row within one ulp of the storage type of the fp64
projection (the bar of the one-token append), rows and lengths exactly where Algorithm 1's append
would have put them, nothing else touched."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2510_24273_amd import synth  # noqa: E402
from tests import gpu_util as gu  # noqa: E402

SMALL = synth.shrink(synth.CONFIGS["cfg2"], B=3, S=700, r=192, top_k=50, n_layers=1, plant=0)


def _rows_close(got, want, dtype, x=None, U=None):
    """bf16: one ulp of the stored value (one rounding dominates the fp32 sum).  fp32: the sum of D_kv products in
    fp32 against fp64, bounded like the score stage by 1e-5 |x| |u_i| (rows x [n, D], projector U [D, r])."""
    if dtype == "bf16":
        return np.all(np.abs(got - want) <= np.maximum(np.abs(want), 1e-30) * 2.0 ** -7 + 1e-6)
    bound = 1e-5 * np.linalg.norm(x, axis=-1, keepdims=True) * np.linalg.norm(U, axis=0)[None, :] + 1e-6
    return np.all(np.abs(got - want) <= bound)


def _prefill_case(oracle, w, n_tok, start, n_new, label):
    print(f"[case] prefill {label}: B={w.B} S_max={w.S} D={w.D_kv} r={w.r} {w.dtype} n_tok={n_tok} start={start} n_new={n_new}",
          flush=True)
    L = synth.make_layer(w, 0, seq_lens=start)
    ctx = gu.make_ctx(w)
    G = gu.upload(L, ctx)
    rng = np.random.default_rng(11)
    k_new = synth.store(rng.standard_normal((w.B, n_tok, w.D_kv)), w.dtype)
    v_new = synth.store(rng.standard_normal((w.B, n_tok, w.D_kv)), w.dtype)
    before = {c: G[c].clone() for c in ("Kc", "Vc")}
    nn = None if n_new is None else gu.to_dev(np.asarray(n_new, dtype=np.int32))
    ctx.compress_prefill(gu.to_dev(k_new), gu.to_dev(v_new), G["W"], G["Kc"], G["Vc"], G["seq_len"], n_tok, nn)
    torch.cuda.synchronize()
    counts = [n_tok] * w.B if n_new is None else [min(max(int(x), 0), n_tok) for x in n_new]
    assert G["seq_len"].tolist() == [min(s + c, w.S) for s, c in zip(start, counts)]
    wd = synth.widen
    for new, U, cache in ((k_new, "Uk", "Kc"), (v_new, "Uv", "Vc")):
        got_all = gu.from_dev(G[cache])
        old_all = gu.from_dev(before[cache])
        Uw = wd(L[U])
        for b in range(w.B):
            written = [t for t in range(counts[b]) if start[b] + t < w.S]
            rows = [start[b] + t for t in written]
            if written:
                want = wd(new[b][written]) @ Uw                      # a library matmul as the step; spot rows by the oracle
                assert _rows_close(got_all[b, rows], want, w.dtype, wd(new[b][written]), Uw), f"{cache} b={b}"
                for t in (written[0], written[len(written) // 2], written[-1]):
                    assert _rows_close(got_all[b, start[b] + t][None], oracle.project(wd(new[b, t]), Uw)[None], w.dtype,
                                       wd(new[b, t])[None], Uw)
            keep = np.ones(w.S, dtype=bool)
            keep[rows] = False
            assert np.array_equal(got_all[b, keep], old_all[b, keep]), f"{cache} b={b}: a row outside the append changed"
    ctx.close()
    return L, G, k_new, v_new


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_prefill_ragged_prompts(oracle, dtype):
    w = synth.shrink(SMALL, dtype=dtype)
    # several token tiles and a ragged tail; per-sequence prompt lengths incl. empty and full
    _prefill_case(oracle, w, 600, [0, 50, 0], [600, 257, 0], "ragged")
    _prefill_case(oracle, w, 300, [100, 0, 450], None, "uniform, one prompt hits the cache end")


def test_prefill_latent_tiles_of_128_and_gqa(oracle):
    w = synth.shrink(SMALL, B=2, S=520, H=32, H_kv=8, r=256)          # D_kv = 1024, two latent tiles of 128
    _prefill_case(oracle, w, 513, [0, 7], [513, 1], "gqa r=256")
    w = synth.shrink(SMALL, B=1, S=300, r=640)                          # five latent tiles of 128, D_kv = 4096
    _prefill_case(oracle, w, 290, [3], None, "r=640")


def test_prefill_large_grid_takes_the_256_token_tiles(oracle):
    """Enough (token tile, latent tile, sequence) items for the 256 x 128 tile (smaller grids take 128 x 128)."""
    w = synth.shrink(SMALL, B=4, S=2600, r=640)
    _prefill_case(oracle, w, 2560, [0, 40, 0, 13], [2560, 2560, 2047, 2305], "256x128 tiles")


def test_prefill_then_decode_matches_token_by_token_append(oracle):
    """A prompt compressed in one call, then a decode step on the resulting cache: every stage against the oracle,
    and the cache rows against the one-token append of the same tokens (same values up to one ulp)."""
    w = synth.shrink(SMALL, B=2, S=256, r=192, top_k=40)
    L, G, k_new, v_new = _prefill_case(oracle, w, 200, [0, 0], [200, 131], "then decode")
    ctx = gu.make_ctx(w)
    G["W"] = ctx.pack_weights(G["Uk"], G["Uv"])
    # token by token into a second cache
    K2, V2 = torch.zeros_like(G["Kc"]), torch.zeros_like(G["Vc"])
    sl2 = torch.zeros_like(G["seq_len"])
    kd, vd = gu.to_dev(k_new), gu.to_dev(v_new)
    for t in range(131):
        ctx.compress_append(kd[:, t].contiguous(), vd[:, t].contiguous(), G["W"], K2, V2, sl2)
    torch.cuda.synchronize()
    a, b2 = gu.from_dev(G["Kc"][:, :131]), gu.from_dev(K2[:, :131])
    assert np.all(np.abs(a - b2) <= np.maximum(np.abs(a), 1e-30) * 2.0 ** -7 + 1e-6)
    L2 = dict(L)
    for kname in ("Kc", "Vc"):
        t = G[kname].cpu()
        L2[kname] = t.view(torch.int16).numpy().view(np.uint16)
    L2["seq_len"] = G["seq_len"].cpu().numpy()
    L2["q_pos"] = L2["seq_len"].astype(np.int32)
    G["q_pos"] = gu.to_dev(L2["q_pos"])
    R = gu.run_stages(ctx, w, G)
    for bb in range(w.B):
        gu.check_sequence(oracle, w, L2, R, bb)
    ctx.close()

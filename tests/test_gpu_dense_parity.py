"""GPU parity of the dense baseline (attention over a full-rank cache of rotated keys, the
comparison point of Sec. 5.3 / Table 6) against the oracle, through the C ABI.  Same output
bounds as the sparse path (tests/gpu_util.py::out_tolerances)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("no GPU", allow_module_level=True)

from paper_2510_24273_amd import synth  # noqa: E402
from tests import gpu_util as gu  # noqa: E402

C = synth.CONFIGS
SMALL = synth.shrink(C["cfg2"], B=3, S=1000, r=192, top_k=100, n_layers=1, plant=0)


def _case(oracle, w, seq_lens=None, q_pos=None, seqs=None):
    print(f"[case] dense {w.name} B={w.B} S={w.S} H={w.H}/{w.H_kv} {w.dtype} seq_lens={seq_lens}", flush=True)
    seq_lens = [w.S] * w.B if seq_lens is None else list(seq_lens)
    L = synth.make_dense_cache(w, 0)
    sl = np.asarray(seq_lens, np.int32)
    qp = sl.copy() if q_pos is None else np.asarray(q_pos, np.int32)
    ctx = gu.make_ctx(w)
    q, K, V = gu.to_dev(L["q"]), gu.to_dev(L["K"]), gu.to_dev(L["V"])
    out = torch.empty((w.B, w.H, w.d), dtype=gu.out_dtype(w), device=gu.DEV)
    ctx.dense_attend(q, gu.to_dev(qp), K, V, gu.to_dev(sl), out)
    out2 = torch.empty_like(out)
    ctx.dense_attend(q, gu.to_dev(qp), K, V, gu.to_dev(sl), out2)
    torch.cuda.synchronize()
    as_bits = (lambda t: t.view(torch.int16)) if out.dtype == torch.bfloat16 else (lambda t: t)
    assert torch.equal(as_bits(out), as_bits(out2)), "not repeatable"
    wd = synth.widen
    worst = 0.0
    for b in (range(w.B) if seqs is None else seqs):
        S = int(sl[b])
        y_gpu = gu.from_dev(out[b])
        if S == 0:
            assert np.all(y_gpu == 0)
            continue
        y_ref = oracle.dense_decode(wd(L["q"][b]), int(qp[b]), wd(L["K"][b][:S]), wd(L["V"][b][:S]), w.theta,
                                    w.rope_style)
        star, tight = gu.out_tolerances(w, y_ref)
        err = float(np.max(np.abs(y_gpu - y_ref)))
        worst = max(worst, err)
        assert err <= star, f"b={b}: output error {err:.3e} > {star}"
        assert err <= tight, f"b={b}: output error {err:.3e} > derived bound {tight:.3e}"
    print(f"    worst output error {worst:.3e}", flush=True)
    ctx.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_small_ragged_batch(oracle, dtype):
    _case(oracle, synth.shrink(SMALL, dtype=dtype), seq_lens=[1000, 37, 513])


def test_empty_and_single_token_sequences(oracle):
    _case(oracle, synth.shrink(SMALL, B=4), seq_lens=[0, 1, 16, 17])


@pytest.mark.parametrize("H_kv,H", [(8, 32), (4, 32), (2, 4), (1, 8), (3, 6), (64, 64), (8, 64)])
def test_gqa_groups(oracle, H_kv, H):
    _case(oracle, synth.shrink(SMALL, B=2, S=600, H=H, H_kv=H_kv), seq_lens=[600, 333])


def test_interleaved_rope_and_query_beyond_the_table(oracle):
    w = synth.shrink(SMALL, B=2, rope_style=1, theta=500000.0)
    _case(oracle, w, q_pos=[w.S + 1, 1_000_003])


def test_random_shapes(oracle):
    """Seeded sweep over head layouts, cache lengths (one and several chunks), storage types, RoPE pairings and
    ragged lengths."""
    rng = np.random.default_rng(123)
    for case in range(10):
        H_kv = int(rng.choice([1, 2, 3, 4, 8, 16, 32]))
        G = int(rng.choice([g for g in (1, 2, 3, 4, 8) if g * H_kv <= 64]))
        B = int(rng.integers(1, 4))
        S = int(rng.integers(1, 6000))
        w = synth.shrink(SMALL, B=B, S=S, H=H_kv * G, H_kv=H_kv, top_k=1, dtype=str(rng.choice(["bf16", "f32"])),
                         rope_style=int(rng.integers(0, 2)), theta=float(rng.choice([1e4, 5e5])))
        seq = rng.integers(0, S + 1, size=B).tolist()
        seq[0] = S
        _case(oracle, w, seq_lens=seq, q_pos=[int(x) + int(rng.integers(0, 3)) for x in seq])


def test_maximum_cache_length(oracle):
    """2^20 cached tokens (64 chunks of 16384)."""
    _case(oracle, synth.shrink(SMALL, B=1, S=1 << 20, H=8, H_kv=1, r=64))


def test_cfg2_shape_full(oracle):
    _case(oracle, C["cfg2"])


def test_cfg3b_shape_sampled_sequences(oracle):
    _case(oracle, C["cfg3b"], seqs=[0, 9])

"""Pins of the oracle's quantised-value functions (CPU only): the paper's value path of
Sec. 5.1 (channel-wise group quantisation, 4 / 2 bit) and Algorithm 1's last step over the
quantised cache.  Pinned by hand-worked values, the nearest-grid-point definition by brute
force, error bounds and invariances, and dense attention written independently below."""
import math

import numpy as np
import pytest


def test_hand_worked_group_4bit(oracle):
    # one group whose values already sit on a 16-point grid: min -2, step 0.5
    k = (np.arange(32) * 7) % 16
    v = (-2.0 + 0.5 * k)[None, :]
    codes, scale, zero = oracle.quantize_values(v, 4, "f32")
    assert scale.tolist() == [[0.5]] and zero.tolist() == [[-2.0]]
    assert codes[0].tolist() == k.tolist()
    np.testing.assert_array_equal(oracle.dequantize_values(codes, scale, zero), v)


def test_hand_worked_group_2bit_rounding(oracle):
    # min 0, max 3 -> step 1; 0.49 -> 0, 0.51 -> 1, 1.5 -> 2 and 2.5 -> 2 (ties to even), 2.51 -> 3
    v = np.zeros((1, 32))
    v[0, :7] = [0.0, 3.0, 0.49, 0.51, 1.5, 2.5, 2.51]
    codes, scale, zero = oracle.quantize_values(v, 2, "f32")
    assert scale[0, 0] == 1.0 and zero[0, 0] == 0.0
    assert codes[0, :7].tolist() == [0, 3, 0, 1, 2, 2, 3]


def test_constant_group_is_exact(oracle):
    v = np.full((2, 64), 1.25)
    v[1, 32:] = -3.0
    codes, scale, zero = oracle.quantize_values(v, 4, "bf16")
    assert not codes.any() and not scale.any()
    np.testing.assert_array_equal(oracle.dequantize_values(codes, scale, zero), v)


@pytest.mark.parametrize("bits", [2, 4])
def test_codes_are_the_nearest_grid_points(oracle, bits):
    """Brute force over all 2^bits grid points: the chosen code is a nearest one, the group
    minimum gets code 0, the maximum the top code, and the error is at most half a step."""
    rng = np.random.default_rng(5 + bits)
    v = rng.standard_normal((40, 128)).astype(np.float32).astype(np.float64)
    codes, scale, zero = oracle.quantize_values(v, bits, "f32")
    levels = (1 << bits) - 1
    assert codes.max() == levels and codes.min() == 0
    g = v.reshape(40, 4, 32)
    grid = zero[..., None, None] + scale[..., None, None] * np.arange(levels + 1)[None, None, None, :]
    err_all = np.abs(g[..., None] - grid)                     # [40,4,32,levels+1]
    chosen = np.take_along_axis(err_all, codes.reshape(40, 4, 32)[..., None].astype(np.int64), -1)[..., 0]
    assert np.all(chosen <= err_all.min(-1) + 1e-6 * scale[..., None])
    assert np.all(chosen <= 0.5 * scale[..., None] * (1 + 1e-5))
    c3 = codes.reshape(40, 4, 32)
    assert np.all(c3[g == g.min(-1, keepdims=True)] == 0)
    assert np.all(c3[g == g.max(-1, keepdims=True)] == levels)


def test_shift_and_power_of_two_scaling(oracle):
    rng = np.random.default_rng(11)
    v = np.round(rng.standard_normal((3, 64)) * 64) / 64       # exact in float32 with room to spare
    c0, s0, z0 = oracle.quantize_values(v, 4, "f32")
    c1, s1, z1 = oracle.quantize_values(v + 8.0, 4, "f32")
    np.testing.assert_array_equal(c0, c1)
    np.testing.assert_array_equal(s0, s1)
    np.testing.assert_array_equal(z0 + 8.0, z1)
    c2, s2, z2 = oracle.quantize_values(v * 4.0, 4, "f32")
    np.testing.assert_array_equal(c0, c2)
    np.testing.assert_array_equal(s0 * 4.0, s2)


def test_bf16_scale_is_storage_exact_and_bound_holds(oracle):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((16, 256)).astype(np.float32)
    u = x.view(np.uint32) & np.uint32(0xFFFF0000)               # truncate to bf16-exact inputs
    v = u.view(np.float32).astype(np.float64)
    codes, scale, zero = oracle.quantize_values(v, 4, "bf16")
    for a in (scale, zero):
        bits = a.astype(np.float32).view(np.uint32)
        assert not (bits & np.uint32(0xFFFF)).any()
    # the stored step differs from (max-min)/15 by at most one bf16 rounding (2^-9 relative), so the
    # top of the range may be clipped by 15 * 2^-9 steps on top of the half step
    err = np.abs(oracle.dequantize_values(codes, scale, zero) - v).reshape(16, 8, 32)
    assert np.all(err <= scale[..., None] * (0.5 + 15 * 2.0 ** -9 + 1e-6))


def test_bf16_scale_rounds_to_nearest(oracle):
    # min 0, max 15.1875 (exact in bf16): 15.1875 / 15 = 1.0125 lies above the midpoint 1.01171875 of the
    # bf16 neighbours 1.0078125 and 1.015625, so the stored step is 1.015625 (truncation would give 1.0078125);
    # with that step 8.0 / 1.015625 = 7.88 -> code 8 and 7.6 -> 7.48 -> code 7
    v = np.zeros((1, 32))
    v[0, 1] = 15.1875
    v[0, 2] = 8.0
    v[0, 3] = 7.59375
    codes, scale, zero = oracle.quantize_values(v, 4, "bf16")
    assert scale[0, 0] == 1.015625 and zero[0, 0] == 0.0
    assert codes[0, :4].tolist() == [0, 15, 8, 7]
    # the same group stored in fp32 keeps the unrounded step
    _, scale32, _ = oracle.quantize_values(v, 4, "f32")
    assert scale32[0, 0] == float(np.float32(15.1875) / np.float32(15.0))


def test_pack_layout(oracle):
    c = np.array([[1, 2, 3, 4, 15, 0, 7, 8]], dtype=np.uint8)
    assert oracle.pack_codes(c, 4).tolist() == [[0x21, 0x43, 0x0F, 0x87]]
    c2 = np.array([[1, 2, 3, 0, 3, 3, 0, 1]], dtype=np.uint8)
    assert oracle.pack_codes(c2, 2).tolist() == [[0b00111001, 0b01001111]]
    np.testing.assert_array_equal(oracle.unpack_codes(oracle.pack_codes(c, 4), 4), c)
    np.testing.assert_array_equal(oracle.unpack_codes(oracle.pack_codes(c2, 2), 2), c2)


def _rope_complex(x, pos, theta):
    d = x.shape[-1]
    f = theta ** (-2.0 * np.arange(d // 2) / d)
    z = (x[..., : d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * pos * f)
    return np.concatenate([z.real, z.imag], axis=-1)


def test_attention_over_grid_valued_cache_equals_dense_attention(oracle):
    """Values that lie on each group's 16-point grid survive quantisation exactly, so with every
    token selected and a square orthogonal key projector the output must equal dense RoPE
    attention over the original keys and values (written here with complex rotations)."""
    rng = np.random.default_rng(21)
    H, H_kv, d, S, theta = 4, 2, 32, 19, 1e4
    D = H_kv * d
    K = rng.standard_normal((S, D))
    Uk, _ = np.linalg.qr(rng.standard_normal((D, D)))
    Kc = K @ Uk                                                  # latent keys, full rank
    V = -1.0 + 0.25 * rng.integers(0, 16, size=(S, D))
    V[:, ::32] = -1.0
    V[:, 1::32] = 2.75                                           # every group spans the whole grid
    q = rng.standard_normal((H, d))
    codes, scale, zero = oracle.quantize_values(V, 4, "f32")
    np.testing.assert_array_equal(oracle.dequantize_values(codes, scale, zero), V)
    idx = rng.permutation(S).astype(np.int32)
    y = oracle.sparse_attend_qv(q, S, Kc, Uk, codes, scale, zero, idx, H_kv, theta)
    G = H // H_kv
    want = np.zeros((H, d))
    for h in range(H):
        g = h // G
        qr = _rope_complex(q[h], S, theta)
        lg = np.array([qr @ _rope_complex(K[t, g * d:(g + 1) * d], t, theta) for t in range(S)]) / math.sqrt(d)
        p = np.exp(lg - lg.max())
        p /= p.sum()
        want[h] = p @ V[:, g * d:(g + 1) * d]
    np.testing.assert_allclose(y, want, rtol=0, atol=1e-10)


def test_single_selected_token_returns_its_dequantised_row(oracle):
    rng = np.random.default_rng(4)
    H, H_kv, d, S, r = 4, 2, 32, 9, 16
    D = H_kv * d
    V = rng.standard_normal((S, D)).astype(np.float32).astype(np.float64)
    codes, scale, zero = oracle.quantize_values(V, 2, "f32")
    Kc = rng.standard_normal((S, r))
    Uk = rng.standard_normal((D, r))
    q = rng.standard_normal((H, d))
    y = oracle.sparse_attend_qv(q, S, Kc, Uk, codes, scale, zero, np.array([6], dtype=np.int32), H_kv, 1e4)
    vhat = oracle.dequantize_values(codes, scale, zero)[6].reshape(H_kv, d)
    np.testing.assert_allclose(y, vhat[np.arange(H) // (H // H_kv)], rtol=0, atol=1e-12)

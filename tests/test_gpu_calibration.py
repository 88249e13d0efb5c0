"""GPU parity of the offline calibration (Sec. 4.2) through the C ABI: the covariance against the fp64 oracle element
by element, the eigen-decomposition against the oracle's on the same matrix (eigenvalues, eigenvectors up to sign,
orthonormality, the defining equation), the cases where eigenvectors are not unique through what is, and the whole
step through the captured energy of Lemma 1."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2510_24273_amd import binding, synth
from tests import gpu_util as gu
from oracle import calibration_oracle as cal

pytestmark = pytest.mark.gpu


def _cov_gpu(X_store, split=None):
    n, D = X_store.shape
    C = torch.zeros(D, D, dtype=torch.float64, device=gu.DEV)
    X = gu.to_dev(X_store)
    keep = []
    parts = [(0, n)] if split is None else [(0, split), (split, n)]
    for a, b in parts:
        keep.append(binding.calib_accumulate(X[a:b].contiguous(), C))
    torch.cuda.synchronize()
    return C


def _check_cov(C_gpu, X_store, chunk_tokens=4096):
    Xd = synth.widen(X_store)
    C_ref = cal.covariance(Xd)
    got = C_gpu.cpu().numpy()
    dg = np.sqrt(np.diag(C_ref))
    # products of stored values are exact in fp32; a chunk's sum of at most 4096 of them carries at most
    # 4096 * 2^-24 relative to sum |x_i x_j| <= sqrt(C_ii C_jj); typical error is the square root of that count
    bound = 2e-5 * np.outer(dg, dg) + 1e-30
    err = np.abs(got - C_ref)
    assert np.all(err <= bound), float(np.max(err / bound))
    assert np.array_equal(got, got.T) or np.max(np.abs(got - got.T)) <= 1e-6 * np.max(dg) ** 2
    return C_ref


@pytest.mark.parametrize("dtype,D,n", [("bf16", 256, 1000), ("bf16", 512, 9001), ("f32", 256, 4200),
                                        ("bf16", 1024, 5000), ("bf16", 2048, 300), ("bf16", 128, 64), ("f32", 384, 1)])
def test_covariance_matches_the_oracle(dtype, D, n):
    print(f"[case] covariance {dtype} D={D} n={n}", flush=True)
    X = synth.make_calibration_keys(100 + D + n, n, D, dtype, decay=0.98)
    C = _cov_gpu(X)
    _check_cov(C, X)


def test_covariance_accumulates_over_calls():
    print("[case] covariance in two calls", flush=True)
    X = synth.make_calibration_keys(7, 6000, 256, "bf16", decay=0.95)
    C = _cov_gpu(X, split=1777)
    _check_cov(C, X)


def _same_up_to_sign(a, b, tol):
    worst = 0.0
    for i in range(a.shape[1]):
        worst = max(worst, min(np.max(np.abs(a[:, i] - b[:, i])), np.max(np.abs(a[:, i] + b[:, i]))))
    assert worst <= tol, worst


def _eig_gpu(C_np, r, dtype=torch.float32, max_sweeps=80):
    C = torch.from_numpy(np.ascontiguousarray(C_np)).to(gu.DEV)
    lam, U, sweeps = binding.calib_eigenvectors(C, r, dtype, max_sweeps)
    torch.cuda.synchronize()
    return lam.cpu().numpy(), gu.from_dev(U), sweeps


@pytest.mark.parametrize("D,r,decay", [(256, 64, 0.9), (512, 128, 0.95), (256, 256, 0.97)])
def test_eigenvectors_match_the_oracle_on_a_separated_spectrum(D, r, decay):
    print(f"[case] eigenvectors D={D} r={r}", flush=True)
    X = synth.widen(synth.make_calibration_keys(11 + D, 4 * D, D, "f32", decay=decay))
    C = cal.covariance(X)
    lam_ref, U_ref = cal.leading_eigenvectors(C, r)
    lam, U, sweeps = _eig_gpu(C, r)
    assert 0 < sweeps <= 60, sweeps
    print('    sweeps', sweeps, flush=True)
    np.testing.assert_allclose(lam[:r], lam_ref[:r], rtol=0, atol=1e-11 * lam_ref[0])
    np.testing.assert_allclose(lam, lam_ref, rtol=0, atol=1e-3 * lam_ref[0])
    np.testing.assert_allclose(lam[:r], lam_ref[:r], rtol=1e-8)
    # eigenvectors: fp64 on both sides, stored as fp32 by the GPU: half an ulp of fp32 plus the conditioning
    # (1e-16 * lambda_0 / gap, gaps of at least a few percent of lambda_i)
    _same_up_to_sign(U, U_ref, 2e-7)
    np.testing.assert_allclose(U.T @ U, np.eye(r), atol=5e-7)
    resid = C @ U - U * lam[:r]
    assert np.max(np.abs(resid)) <= 5e-7 * lam_ref[0]
    # sign convention: the largest component of every column is positive
    big = U[np.argmax(np.abs(U), axis=0), np.arange(r)]
    assert np.all(big > 0)


def test_eigenvectors_in_bf16_are_the_rounded_fp64_vectors():
    print("[case] eigenvectors bf16", flush=True)
    D, r = 256, 32
    X = synth.widen(synth.make_calibration_keys(3, 1024, D, "f32", decay=0.85))
    C = cal.covariance(X)
    _, U_ref = cal.leading_eigenvectors(C, r)
    _, U, _ = _eig_gpu(C, r, torch.bfloat16)
    # one rounding to bf16 (8 significant bits): half an ulp of the component, plus the fp64 agreement
    for i in range(r):
        ref = U_ref[:, i] * np.sign(U_ref[np.argmax(np.abs(U_ref[:, i])), i])
        assert np.all(np.abs(U[:, i] - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-7), i


def test_repeated_eigenvalues_give_a_valid_basis():
    print("[case] repeated eigenvalues", flush=True)
    D = 256
    rng = np.random.default_rng(5)
    Q, _ = np.linalg.qr(rng.standard_normal((D, D)))
    lam_true = np.concatenate([np.full(8, 5.0), np.full(8, 2.0), np.linspace(1.0, 0.1, D - 16)])
    C = (Q * lam_true) @ Q.T
    C = 0.5 * (C + C.T)
    lam, U, sweeps = _eig_gpu(C, 16)
    assert sweeps > 0
    np.testing.assert_allclose(lam[:16], np.sort(lam_true)[::-1][:16], rtol=0, atol=1e-11 * 5.0)
    np.testing.assert_allclose(U.T @ U, np.eye(16), atol=5e-7)
    # each block of columns spans the eigenspace of its eigenvalue: the projector is unique
    for a, b in ((0, 8), (8, 16)):
        P_ref = Q[:, a:b] @ Q[:, a:b].T
        P = U[:, a:b] @ U[:, a:b].T
        assert np.max(np.abs(P - P_ref)) <= 2e-6


def test_rank_deficient_covariance_and_diagonal_input():
    print("[case] rank deficient, diagonal", flush=True)
    D = 256
    X = synth.widen(synth.make_calibration_keys(9, 100, D, "f32", decay=0.9))   # 100 tokens: rank 100
    C = cal.covariance(X)
    lam_ref, U_ref = cal.leading_eigenvectors(C, 40)
    lam, U, sweeps = _eig_gpu(C, 40)
    assert sweeps > 0
    np.testing.assert_allclose(lam[:40], lam_ref[:40], rtol=0, atol=1e-10 * lam_ref[0])
    # past the r requested ones the values are the row norms when the leading rows had converged: approximations
    np.testing.assert_allclose(lam[40:], lam_ref[40:], rtol=0, atol=1e-3 * lam_ref[0])
    _same_up_to_sign(U, U_ref, 5e-7)
    # asked for as many vectors as the rank: every non-zero eigenvalue converges and what is left of the other rows
    # is zero to working precision
    lam_ref, U_ref = cal.leading_eigenvectors(C, 100)
    lam, U, sweeps = _eig_gpu(C, 100)
    assert sweeps > 0
    np.testing.assert_allclose(lam[:100], lam_ref[:100], rtol=0, atol=1e-10 * lam_ref[0])
    assert np.all(np.abs(lam[100:]) <= 1e-9 * lam_ref[0])
    _same_up_to_sign(U[:, :60], U_ref[:, :60], 5e-7)
    # a diagonal matrix needs no rotation: one sweep, eigenvalues sorted, unit vectors
    d = np.linspace(0.5, 3.0, D)
    lam, U, sweeps = _eig_gpu(np.diag(d), 5)
    assert sweeps == 1
    np.testing.assert_array_equal(lam, np.sort(d)[::-1])
    for i in range(5):
        e = np.zeros(D); e[D - 1 - i] = 1.0
        np.testing.assert_array_equal(U[:, i], e)


def test_sweep_limit_is_reported():
    D = 256
    X = synth.widen(synth.make_calibration_keys(13, 1024, D, "f32", decay=0.9))
    lam, U, sweeps = _eig_gpu(cal.covariance(X), 8, max_sweeps=1)
    assert sweeps == -1


def test_whole_calibration_captures_the_energy_of_the_oracle_basis():
    print("[case] keys -> covariance -> eigenvectors", flush=True)
    D, r, n = 512, 128, 6000
    Xs = synth.make_calibration_keys(21, n, D, "bf16", decay=0.97, heads=4)
    C_gpu = _cov_gpu(Xs)
    C_ref, lam_ref, U_ref = cal.calibrate(synth.widen(Xs), r)
    Cg = C_gpu.clone()
    lam, U, sweeps = binding.calib_eigenvectors(Cg, r, torch.bfloat16)
    torch.cuda.synchronize()
    assert sweeps > 0
    U = gu.from_dev(U)
    np.testing.assert_allclose(lam.cpu().numpy()[:r], lam_ref[:r], rtol=2e-5)
    e_ref = cal.captured_energy(C_ref, U_ref)
    # bf16 columns are no longer exactly orthonormal: measure the energy of their span
    Qn, _ = np.linalg.qr(U)
    assert cal.captured_energy(C_ref, Qn) >= (1.0 - 1e-5) * e_ref
    assert np.max(np.abs(U.T @ U - np.eye(r))) <= 2.0 ** -7


def test_bad_arguments_are_refused():
    C = torch.zeros(256, 256, dtype=torch.float64, device=gu.DEV)
    X = torch.zeros(10, 200, dtype=torch.bfloat16, device=gu.DEV)          # D not a multiple of 128
    assert binding._lib.sals_calib_accumulate_workspace_bytes(binding.SALS_BF16, 200) == 0
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=gu.DEV)
    st = binding._lib.sals_calib_accumulate(binding.SALS_BF16, X.data_ptr(), 10, 200, C.data_ptr(), ws.data_ptr(), 1 << 20, None)
    assert binding.status_string(st) == "SALS_ERR_INVALID_ARG"
    X = torch.zeros(10, 256, dtype=torch.bfloat16, device=gu.DEV)
    st = binding._lib.sals_calib_accumulate(binding.SALS_BF16, X.data_ptr(), 10, 256, C.data_ptr(), ws.data_ptr(), 1024, None)
    assert binding.status_string(st) == "SALS_ERR_WORKSPACE"
    ev = torch.empty(256, dtype=torch.float64, device=gu.DEV)
    U = torch.empty(256, 4, dtype=torch.float32, device=gu.DEV)
    n = ctypes.c_int32(0)
    st = binding._lib.sals_calib_eigenvectors(C.data_ptr(), 256, 0, binding.SALS_F32, ev.data_ptr(), U.data_ptr(), ws.data_ptr(),
                                              1 << 20, 5, ctypes.byref(n), None)
    assert binding.status_string(st) == "SALS_ERR_INVALID_ARG"
    st = binding._lib.sals_calib_eigenvectors(C.data_ptr(), 256, 4, binding.SALS_F32, ev.data_ptr(), U.data_ptr(), ws.data_ptr(),
                                              1024, 5, ctypes.byref(n), None)
    assert binding.status_string(st) == "SALS_ERR_WORKSPACE"
    torch.cuda.synchronize()


def test_calibrated_projector_feeds_the_decode_path(oracle):
    """The projector the calibration returns has the layout the rest of the library takes: pack it, compress keys
    with it and run a decode step; every stage against the oracle with the same projector."""
    print("[case] calibrated projector in a decode step", flush=True)
    w = synth.shrink(synth.CONFIGS["cfg2"], B=2, S=600, H=4, H_kv=4, r=128, top_k=64, n_layers=1, plant=2)
    keys = synth.make_calibration_keys(31, 3000, w.D_kv, w.dtype, decay=0.985)
    C = _cov_gpu(keys)
    _, U, sweeps = binding.calib_eigenvectors(C, w.r, torch.bfloat16)
    torch.cuda.synchronize()
    assert sweeps > 0
    L = synth.make_layer(w, 0)
    U_bits = U.view(torch.int16).cpu().numpy().view(np.uint16)
    L["Uk"] = U_bits.copy()
    L["Uv"] = U_bits.copy()
    ctx = gu.make_ctx(w)
    G = gu.upload(L, ctx)
    R = gu.run_stages(ctx, w, G)
    for b in range(w.B):
        gu.check_sequence(oracle, w, L, R, b)
    # compression with the calibrated projector keeps what the spectrum says it keeps
    x = synth.widen(keys[:64])
    kt = x @ synth.widen(U_bits)
    lam_ref, _ = cal.leading_eigenvectors(cal.covariance(synth.widen(keys)), w.r)
    kept = np.sum(kt * kt) / np.sum(x * x)
    assert abs(kept - np.sum(lam_ref[: w.r]) / np.sum(lam_ref)) < 0.05
    ctx.close()

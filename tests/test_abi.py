"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the
header declares, and rejects bad descriptors / pointers before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def sb():
    from paper_2510_24273_amd import build
    if build.is_stale():
        build.build()
    from paper_2510_24273_amd import binding
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "sals.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sals_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(sb):
    names = _declared_functions()
    assert set(names) == set(sb.EXPORTS), names
    lib = ctypes.CDLL(sb.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(sb):
    assert sb.status_string(0) == "SALS_OK"
    assert sb.status_string(3) == "SALS_ERR_WORKSPACE"
    assert "UNKNOWN" in sb.status_string(99)


def _desc(sb, **kw):
    base = dict(B=2, S_max=1024, H_q=32, H_kv=8, d=128, r=512, top_k=64, dtype="bf16")
    base.update(kw)
    return sb.make_desc(**base)


def test_workspace_bytes_and_validation(sb):
    n = sb.workspace_bytes(_desc(sb))
    assert n > 0 and n % 256 == 0
    assert sb.workspace_bytes(_desc(sb, S_max=8192)) > n
    for bad, code in [
        (dict(B=0), sb.SALS_ERR_INVALID_ARG),
        (dict(H_kv=5), sb.SALS_ERR_INVALID_ARG),          # 32 % 5 != 0
        (dict(r_score=1024), sb.SALS_ERR_INVALID_ARG),    # r_score > r
        (dict(top_k=0), sb.SALS_ERR_INVALID_ARG),
        (dict(n_recent=-1), sb.SALS_ERR_INVALID_ARG),
        (dict(rope_theta=0.0), sb.SALS_ERR_INVALID_ARG),
        (dict(rope_style=2), sb.SALS_ERR_INVALID_ARG),
        (dict(d=64), sb.SALS_ERR_UNSUPPORTED),
        (dict(r=520), sb.SALS_ERR_UNSUPPORTED),
        (dict(r=4096), sb.SALS_ERR_UNSUPPORTED),
        (dict(r=2048, r_score=2048), sb.SALS_ERR_UNSUPPORTED),   # scoring rank above 1024
        (dict(r_score=100), sb.SALS_ERR_UNSUPPORTED),
        (dict(H_q=128, H_kv=8), sb.SALS_ERR_UNSUPPORTED),
        (dict(B=64), sb.SALS_ERR_UNSUPPORTED),            # B * (H_q/H_kv) > 128
    ]:
        with pytest.raises(sb.SalsError) as e:
            sb.workspace_bytes(_desc(sb, **bad))
        assert e.value.code == code, bad
    nbytes = ctypes.c_size_t()
    assert sb._lib.sals_workspace_bytes(None, ctypes.byref(nbytes)) == sb.SALS_ERR_INVALID_ARG
    d = _desc(sb)
    assert sb._lib.sals_workspace_bytes(ctypes.byref(d), None) == sb.SALS_ERR_INVALID_ARG


def test_create_checks_workspace_and_calls_check_pointers(sb):
    d = _desc(sb)
    n = sb.workspace_bytes(d)
    h = ctypes.c_void_p()
    lib = sb._lib
    assert lib.sals_create(ctypes.byref(d), None, n, ctypes.byref(h)) == sb.SALS_ERR_WORKSPACE
    assert lib.sals_create(ctypes.byref(d), 4096 + 8, n, ctypes.byref(h)) == sb.SALS_ERR_WORKSPACE   # misaligned
    assert lib.sals_create(ctypes.byref(d), 4096, n - 1, ctypes.byref(h)) == sb.SALS_ERR_WORKSPACE   # too small
    assert lib.sals_create(ctypes.byref(d), 4096, n, None) == sb.SALS_ERR_INVALID_ARG
    # a context over a fake (never dereferenced) workspace address: host object only
    assert lib.sals_create(ctypes.byref(d), 4096, n, ctypes.byref(h)) == sb.SALS_OK and h.value
    ok = 1 << 20   # any aligned non-NULL value; rejected calls never reach the device
    assert lib.sals_latent_scores(h, None, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_latent_scores(h, ok, ok, ok + 4, ok, ok, None) == sb.SALS_ERR_INVALID_ARG   # misaligned cache
    assert lib.sals_latent_scores(None, ok, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_topk_select(h, ok, ok, None, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_sparse_attend(h, ok, ok, ok, ok, ok, ok, ok, None, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_compress_append(h, ok, ok, ok, ok, ok, None, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_decode_step(h, ok, ok, ok, ok, ok, ok, None, None, None, None, None) \
        == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_pack_weights(h, ok, ok, None, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_pack_weights(h, ok, ok, ok + 16, None) == sb.SALS_ERR_INVALID_ARG   # W not 256-aligned
    assert sb.packed_weight_bytes(d) == 4 * 8 * 128 * 512 * 2
    # quantised value cache: sizes, and argument checks ahead of any launch
    assert sb.qv_row_bytes(d, 4) == (8 * 128 // 2, 8 * 128 // 32 * 2 * 2)
    assert sb.qv_row_bytes(d, 2) == (8 * 128 // 4, 8 * 128 // 32 * 2 * 2)
    assert sb.qv_row_bytes(_desc(sb, dtype="f32"), 4)[1] == 8 * 128 // 32 * 2 * 4
    with pytest.raises(sb.SalsError) as e:
        sb.qv_row_bytes(d, 3)
    assert e.value.code == sb.SALS_ERR_UNSUPPORTED
    assert lib.sals_compress_append_qv(h, ok, ok, ok, ok, ok, ok, 8, ok, None) == sb.SALS_ERR_UNSUPPORTED
    assert lib.sals_compress_append_qv(h, ok, ok, ok, ok, None, ok, 4, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_compress_append_qv(h, ok, ok, ok, ok, ok, ok, 4, None, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_sparse_attend_qv(h, ok, ok, ok, ok, ok, 1, ok, ok, ok, ok, None) == sb.SALS_ERR_UNSUPPORTED
    assert lib.sals_sparse_attend_qv(h, ok, ok, ok, ok + 8, ok, 4, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_decode_step_qv(h, ok, ok, ok, ok, None, 2, ok, ok, ok, None, None, None, None) \
        == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_decode_step_qv(h, ok, ok, ok, ok, ok, 16, ok, ok, ok, None, None, None, None) \
        == sb.SALS_ERR_UNSUPPORTED
    assert lib.sals_dense_attend(h, ok, ok, ok, None, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_dense_attend(h, ok, None, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    # recent window and overlap score: the pairing rules and pointers are checked ahead of any launch
    dm = _desc(sb, n_recent=64)
    dw = _desc(sb, r=1024, top_k=64)
    hm, hw, hx = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    assert lib.sals_create(ctypes.byref(dm), 4096, sb.workspace_bytes(dm), ctypes.byref(hm)) == sb.SALS_OK
    assert lib.sals_create(ctypes.byref(dw), 4096, sb.workspace_bytes(dw), ctypes.byref(hw)) == sb.SALS_OK
    dx = _desc(sb, r=1024, top_k=32)                      # ring size differs from the main context's n_recent
    assert lib.sals_create(ctypes.byref(dx), 4096, sb.workspace_bytes(dx), ctypes.byref(hx)) == sb.SALS_OK
    win_args = (ok,) * 10
    for ctx_h, win_h in ((hm, hx), (hm, hm), (hm, None), (None, hw), (h, hw)):    # h: no recent tokens
        assert lib.sals_decode_step_window(ctx_h, win_h, *win_args, None, None, None, None) == sb.SALS_ERR_INVALID_ARG
        assert lib.sals_sparse_attend_window(ctx_h, win_h, *win_args, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_decode_step_window(hm, hw, ok, ok, ok, ok, ok, None, ok, ok, ok, ok, None, None, None, None) \
        == sb.SALS_ERR_INVALID_ARG                                                 # Kw missing
    assert lib.sals_window_append(hw, ok, ok, ok, ok, ok, None, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_window_append(hm, ok, ok, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG   # not a window context
    assert lib.sals_window_append(None, ok, ok, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_overlap_score(h, ok, ok, ok, ok, ok, ok, None, None) == sb.SALS_ERR_INVALID_ARG
    assert lib.sals_overlap_score(h, ok, ok, ok + 2, ok, ok, ok, ok, None) == sb.SALS_ERR_INVALID_ARG
    for hh in (hm, hw, hx):
        lib.sals_destroy(hh)
    lib.sals_destroy(h)
    lib.sals_destroy(None)

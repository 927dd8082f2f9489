"""Host-side checks of the C ABI: the library loads, exports what the header declares,
and turns bad arguments into error codes before anything is enqueued (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def rk():
    import paper_2605_08840_amd as r
    if not os.path.exists(r.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return r


def good(rk, **kw):
    base = dict(n_q_heads=4, n_kv_heads=2, head_dim=64, seq_len=1024, window=32, budget=128, dtype="f32")
    base.update(kw)
    return rk.make_params(**base)


def test_exports_every_declared_symbol(rk):
    text = open(os.path.join(ROOT, "include", "restkv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(restkv_[a-z_]+)\s*\(", text)))
    assert {"restkv_score", "restkv_score_smooth", "restkv_smooth", "restkv_smooth_b", "restkv_select_b", "restkv_select", "restkv_compact", "restkv_prepare_wo",
            "restkv_workspace_bytes", "restkv_strerror", "restkv_version"} <= set(names)
    L = rk.lib()
    for n in names:
        assert hasattr(L, n), n
    assert rk.restkv_version() >= 100


def test_param_block_layout_matches_header(rk):
    # 14 four-byte fields then 5 eight-byte fields, no padding
    assert ctypes.sizeof(rk.RestkvParams) == 14 * 4 + 5 * 8


def test_workspace_bytes(rk):
    assert rk.restkv_workspace_bytes(good(rk)) > 0
    big = good(rk, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=131072, window=64, budget=2048, dtype="bf16")
    assert rk.restkv_workspace_bytes(big) > 32 * 131008 * 4      # holds v M v^T for every head
    for bad in (dict(budget=32), dict(budget=2000), dict(n_q_heads=5), dict(window=0),
                dict(window=1024), dict(base_window=4), dict(ema_alpha=1.5), dict(beta=0.0),
                dict(beta=1e-7),           # floor(|x| / beta) would leave the 32-bit range
                dict(variant=3), dict(variant=0x30), dict(variant=0x80), dict(variant=8)):
        assert rk.restkv_workspace_bytes(good(rk, **bad)) == 0, bad


def test_error_codes_without_launch(rk):
    L = rk.lib()
    p = good(rk)
    one = ctypes.c_void_p(256)            # never dereferenced on the host
    ws_n = rk.restkv_workspace_bytes(p)
    # null pointers
    assert L.restkv_score(ctypes.byref(p), None, one, one, None, one, one, ws_n, None) == -1
    assert L.restkv_smooth(ctypes.byref(p), None, None, one, None, None, one, ws_n, None) == -1
    assert L.restkv_select(ctypes.byref(p), one, None, None, 0, None) == -1
    assert L.restkv_select(ctypes.byref(p), one, one, None, 0, None) == -3
    assert L.restkv_compact(ctypes.byref(p), one, one, None, one, one, None) == -1
    assert L.restkv_prepare_wo(ctypes.byref(p), None, 128, one, None) == -1
    # workspace: missing, too small, misaligned
    assert L.restkv_score(ctypes.byref(p), one, one, one, None, one, None, 0, None) == -3
    assert L.restkv_score(ctypes.byref(p), one, one, one, None, one, one, 256, None) == -3
    assert L.restkv_score_smooth(ctypes.byref(p), one, one, one, None, one, None, one, None, None, one, 256, None) == -3
    assert L.restkv_score_smooth(ctypes.byref(p), one, one, one, None, None, None, one, None, None, one, ws_n, None) == -1
    assert L.restkv_score(ctypes.byref(p), one, one, one, None, one, ctypes.c_void_p(264), ws_n, None) == -3
    assert L.restkv_smooth(ctypes.byref(p), one, None, one, None, None, one, 8, None) == -3
    # unsupported / invalid blocks
    assert L.restkv_score(ctypes.byref(good(rk, head_dim=96)), one, one, one, None, one, one, ws_n, None) == -2
    assert L.restkv_score(ctypes.byref(good(rk, dtype=7)), one, one, one, None, one, one, ws_n, None) == -2
    assert L.restkv_score(ctypes.byref(good(rk, budget=32)), one, one, one, None, one, one, ws_n, None) == -1
    assert L.restkv_select(ctypes.byref(good(rk, budget=1025)), one, one, None, 0, None) == -1
    bad_ld = good(rk, ld_score=100)
    assert L.restkv_smooth(ctypes.byref(bad_ld), one, None, one, None, None, one, 1 << 20, None) == -1
    # the streaming reference: null, odd sizes, misaligned pointers; nothing to move is not an error
    assert L.restkv_stream_reference(None, 32, one, 16, None) == -1
    assert L.restkv_stream_reference(one, 32, None, 16, None) == -1
    assert L.restkv_stream_reference(one, 24, one, 16, None) == -1
    assert L.restkv_stream_reference(one, 32, one, 20, None) == -1
    assert L.restkv_stream_reference(ctypes.c_void_p(264), 32, one, 16, None) == -1
    assert L.restkv_stream_reference(None, 0, None, 0, None) == 0
    for code in (0, -1, -2, -3, -4, -99):
        assert len(rk.strerror(code)) > 0


def test_binding_has_no_cpu_fallback(rk, monkeypatch):
    import paper_2605_08840_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", "/nonexistent/librestkv.so")
    with pytest.raises(ImportError):
        b.lib()

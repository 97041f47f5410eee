"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before anything is launched (no GPU needed: the
pointers below are fake, validation never dereferences them)."""
import ctypes
import os
import re

import pytest

import paper_2601_07353_amd as T
from paper_2601_07353_amd.binding import _CTreeState

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(T.binding.LIB_PATH):
        from paper_2601_07353_amd import build
        build.build()
    return T.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "talon.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(talon_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert len(names) >= 10
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(T.binding.EXPORTS)


def fake_state(B=1, N=16, N_pad=64, ptr=0x10000):
    return _CTreeState(B, N, N_pad, *[ptr + 0x1000 * i for i in range(10)])


def err(lib):
    return lib.talon_last_error_string().decode()


P = 0x7000000  # aligned fake device address


def expand_call(lib, st, logits=P, dtype=1, row_stride=1024, seq_stride=1024 * 64, row_mode=0, vocab=1024, k=4,
                ws=P, ws_bytes=1 << 30, out=P):
    return lib.talon_expand_layer(logits, dtype, row_stride, seq_stride, row_mode, -1, ctypes.byref(st), vocab, k,
                                  out, out, out, out, out, out, ws, ws_bytes, None)


def test_expand_rejects_bad_arguments(lib):
    st = fake_state()
    assert expand_call(lib, st, k=0) == T.TALON_ERR_INVALID_ARG and "k=0" in err(lib)
    assert expand_call(lib, st, k=65) == T.TALON_ERR_INVALID_ARG
    assert expand_call(lib, st, vocab=0) == T.TALON_ERR_INVALID_ARG
    assert expand_call(lib, st, dtype=7) == T.TALON_ERR_UNSUPPORTED
    assert expand_call(lib, st, logits=0) == T.TALON_ERR_INVALID_ARG
    assert expand_call(lib, st, logits=P + 2) == T.TALON_ERR_INVALID_ARG and "aligned" in err(lib)
    assert expand_call(lib, st, row_stride=1000) == T.TALON_ERR_INVALID_ARG   # < vocab
    assert expand_call(lib, st, row_stride=1028) == T.TALON_ERR_INVALID_ARG   # not a multiple of 8 bf16
    assert expand_call(lib, st, row_mode=5) == T.TALON_ERR_INVALID_ARG
    assert expand_call(lib, st, ws_bytes=16) == T.TALON_ERR_WORKSPACE and "smaller" in err(lib)
    assert expand_call(lib, st, vocab=16 * 8192 * 9, row_stride=16 * 8192 * 9, k=16) == T.TALON_ERR_UNSUPPORTED
    assert expand_call(lib, fake_state(N=300, N_pad=320)) == T.TALON_ERR_INVALID_ARG
    assert expand_call(lib, fake_state(N_pad=48)) == T.TALON_ERR_INVALID_ARG
    assert expand_call(lib, fake_state(B=0)) == T.TALON_ERR_INVALID_ARG
    bad = fake_state(); bad.logp = 0
    assert expand_call(lib, bad) == T.TALON_ERR_INVALID_ARG


def test_workspace_size_queries(lib):
    a = lib.talon_expand_workspace_bytes(1, 64, 128256, 10, 1)
    b = lib.talon_expand_workspace_bytes(4, 128, 151936, 8, 1)
    assert 0 < a < b
    assert lib.talon_expand_workspace_bytes(1, 64, 128256, 0, 1) == 0
    assert lib.talon_tree_attention_workspace_bytes(1, 64, 32, 8, 128, 2048) > 0
    assert lib.talon_tree_attention_workspace_bytes(1, 64, 32, 8, 96, 2048) == 0
    assert lib.talon_expand_workspace_init(None, 1024, None) == T.TALON_ERR_INVALID_ARG


def select_call(lib, st, k=4, mu=0.03, K_init=4, init_layers=1, max_depth=8, cand=P):
    return lib.talon_select_budget(ctypes.byref(st), k, cand, cand, cand, ctypes.c_float(mu), K_init, init_layers,
                                   max_depth, None)


def test_select_rejects_bad_arguments(lib):
    st = fake_state()
    for mu in (0.0, -0.1, 1.5, float("nan")):
        assert select_call(lib, st, mu=mu) == T.TALON_ERR_INVALID_ARG and "mu" in err(lib)
    assert select_call(lib, st, K_init=0) == T.TALON_ERR_INVALID_ARG
    assert select_call(lib, st, init_layers=-1) == T.TALON_ERR_INVALID_ARG
    assert select_call(lib, st, max_depth=0) == T.TALON_ERR_INVALID_ARG
    assert select_call(lib, st, k=0) == T.TALON_ERR_INVALID_ARG
    assert select_call(lib, st, cand=0) == T.TALON_ERR_INVALID_ARG
    assert select_call(lib, fake_state(N=256, N_pad=256), k=32) == T.TALON_ERR_UNSUPPORTED   # 255 * 32 candidates per layer
    assert lib.talon_select_budget(None, 4, P, P, P, ctypes.c_float(0.03), 4, 1, 8, None) == T.TALON_ERR_INVALID_ARG


def fused_call(lib, fn, st, k=4, mu=0.03, K_init=4, init_layers=1, max_depth=8, vocab=1024, ws_bytes=1 << 30):
    args = [P, 1, 1024, 1024 * 64, 0]
    if fn == "talon_expand_select_layer":
        args.append(-1)
    args += [ctypes.byref(st), vocab, k, ctypes.c_float(mu), K_init, init_layers, max_depth, P, P, P, P, P, P, P,
             ws_bytes, None]
    return getattr(lib, fn)(*args)


@pytest.mark.parametrize("fn", ["talon_expand_select_layer", "talon_expand_tree"])
def test_fused_calls_reject_bad_arguments(lib, fn):
    st = fake_state()
    assert fused_call(lib, fn, st, k=0) == T.TALON_ERR_INVALID_ARG
    assert fused_call(lib, fn, st, vocab=0) == T.TALON_ERR_INVALID_ARG
    assert fused_call(lib, fn, st, mu=0.0) == T.TALON_ERR_INVALID_ARG and "mu" in err(lib)
    assert fused_call(lib, fn, st, mu=2.0) == T.TALON_ERR_INVALID_ARG
    assert fused_call(lib, fn, st, K_init=0) == T.TALON_ERR_INVALID_ARG
    assert fused_call(lib, fn, st, max_depth=0) == T.TALON_ERR_INVALID_ARG
    assert fused_call(lib, fn, st, ws_bytes=64) == T.TALON_ERR_WORKSPACE
    assert fused_call(lib, fn, fake_state(B=0)) == T.TALON_ERR_INVALID_ARG


def test_build_tree_rejects_bad_arguments(lib):
    st = fake_state()

    def call(root=P, mask=P, k=4, mu=0.03, ws_bytes=1 << 30):
        return lib.talon_build_tree(root, P, 1, 1024, 1024 * 64, 0, ctypes.byref(st), 1024, k, ctypes.c_float(mu), 4, 1,
                                    8, P, P, P, P, P, P, mask, P, ws_bytes, None)

    assert call(root=0) == T.TALON_ERR_INVALID_ARG and "root_token" in err(lib)
    assert call(mask=P + 4) == T.TALON_ERR_INVALID_ARG
    assert call(k=0) == T.TALON_ERR_INVALID_ARG
    assert call(mu=0.0) == T.TALON_ERR_INVALID_ARG
    assert call(ws_bytes=64) == T.TALON_ERR_WORKSPACE


def test_verification_and_prune_calls_reject_bad_arguments(lib):
    st = fake_state()
    assert lib.talon_verify_workspace_bytes(1, 64, 128256, 1) > lib.talon_expand_workspace_bytes(1, 64, 128256, 1, 1)
    assert lib.talon_verify_workspace_bytes(1, 60, 128256, 1) == 0
    ta = lambda **kw: lib.talon_target_argmax(kw.get("logits", P), kw.get("dtype", 1), kw.get("row_stride", 1024),
                                              1024 * 64, ctypes.byref(st), kw.get("vocab", 1024), kw.get("tok", P), None,
                                              kw.get("sstat", P), kw.get("ws", P), kw.get("ws_bytes", 1 << 30), None)
    assert ta(logits=0) == T.TALON_ERR_INVALID_ARG
    assert ta(tok=0) == T.TALON_ERR_INVALID_ARG
    assert ta(sstat=0) == T.TALON_ERR_INVALID_ARG
    assert ta(dtype=9) == T.TALON_ERR_UNSUPPORTED
    assert ta(row_stride=1000) == T.TALON_ERR_INVALID_ARG
    assert ta(ws=0) == T.TALON_ERR_INVALID_ARG
    assert ta(ws_bytes=1024) == T.TALON_ERR_WORKSPACE
    assert lib.talon_greedy_accept(ctypes.byref(st), P, P, None, P, P, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_greedy_accept(None, P, P, P, P, P, None) == T.TALON_ERR_INVALID_ARG
    ck = lambda **kw: lib.talon_compact_kv(kw.get("kt", P), P, P, P, P, P, P, P, kw.get("B", 1), kw.get("N_pad", 64), 8,
                                           kw.get("Dh", 128), kw.get("cap", 4096), 4096 * 1024, kw.get("st_", 1024), 128,
                                           None)
    assert ck(kt=0) == T.TALON_ERR_INVALID_ARG
    assert ck(kt=P + 2) == T.TALON_ERR_INVALID_ARG
    assert ck(Dh=100) == T.TALON_ERR_INVALID_ARG
    assert ck(cap=0) == T.TALON_ERR_INVALID_ARG
    assert ck(st_=1001) == T.TALON_ERR_INVALID_ARG
    assert ck(N_pad=48) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_prune_tree(ctypes.byref(st), 0, P, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_prune_tree(ctypes.byref(st), 65, P, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_prune_tree(ctypes.byref(st), 8, None, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_probe_read(None, 1 << 20, P, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_probe_mfma(0, 10, P, None, None) == T.TALON_ERR_INVALID_ARG


def test_literal_call_rejects_bad_arguments(lib):
    st = fake_state()
    need = lib.talon_literal_workspace_bytes(1, 64, 1024, 1)
    assert need > lib.talon_expand_workspace_bytes(1, 64, 1024, 1, 1) + 64 * 256 * 8
    assert lib.talon_literal_workspace_bytes(1, 60, 1024, 1) == 0
    assert lib.talon_literal_workspace_bytes(1, 64, 0, 1) == 0

    def call(logits=P, dtype=1, row_stride=1024, layers=1, state=st, vocab=1024, mu=0.03, K_init=4, init_layers=1,
             max_depth=8, ws=P, ws_bytes=1 << 30):
        return lib.talon_expand_literal(logits, dtype, row_stride, 1024 * 64, 0, layers,
                                        ctypes.byref(state) if state is not None else None, vocab, ctypes.c_float(mu),
                                        K_init, init_layers, max_depth, ws, ws_bytes, None)

    assert call(logits=0) == T.TALON_ERR_INVALID_ARG
    assert call(logits=P + 4) == T.TALON_ERR_INVALID_ARG
    assert call(dtype=7) == T.TALON_ERR_UNSUPPORTED
    assert call(row_stride=1001) == T.TALON_ERR_INVALID_ARG
    assert call(layers=0) == T.TALON_ERR_INVALID_ARG and "layers" in err(lib)
    assert call(state=None) == T.TALON_ERR_INVALID_ARG
    assert call(vocab=0) == T.TALON_ERR_INVALID_ARG
    assert call(mu=0.0) == T.TALON_ERR_INVALID_ARG and "mu" in err(lib)
    assert call(mu=1.5) == T.TALON_ERR_INVALID_ARG
    assert call(K_init=0) == T.TALON_ERR_INVALID_ARG
    assert call(init_layers=-1) == T.TALON_ERR_INVALID_ARG
    assert call(max_depth=0) == T.TALON_ERR_INVALID_ARG
    assert call(ws=0) == T.TALON_ERR_INVALID_ARG
    assert call(ws_bytes=need - 1) == T.TALON_ERR_WORKSPACE


def test_profile_hook_host_side(lib):
    n = ctypes.c_int32(-1)
    assert lib.talon_profile_read(None, 0, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_profile_read(None, 4, ctypes.byref(n)) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_profile_scan_launches(0) == T.TALON_OK
    assert lib.talon_profile_read(None, 0, ctypes.byref(n)) == T.TALON_OK and n.value == 0


def test_mask_and_init_reject_bad_arguments(lib):
    st = fake_state()
    assert lib.talon_build_tree_mask(ctypes.byref(st), None, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_build_tree_mask(None, P, None) == T.TALON_ERR_INVALID_ARG
    assert lib.talon_tree_init(ctypes.byref(st), None, None) == T.TALON_ERR_INVALID_ARG


def attn_call(lib, q=P, kp=P, vp=P, kt=P, vt=P, mask=P, n=P, pl=P, B=1, N_pad=64, Hq=32, Hkv=8, Dh=128, Lmax=2048,
              sb=2048 * 8 * 128, st_=8 * 128, sh=128, scale=0.0, out=P, ws=P, ws_bytes=1 << 40):
    return lib.talon_tree_attention(q, kp, vp, kt, vt, mask, n, pl, B, N_pad, Hq, Hkv, Dh, Lmax, sb, st_, sh,
                                    ctypes.c_float(scale), out, None, ws, ws_bytes, None)


def test_attention_rejects_bad_arguments(lib):
    assert attn_call(lib, Dh=96) == T.TALON_ERR_UNSUPPORTED
    assert attn_call(lib, Hq=30) == T.TALON_ERR_UNSUPPORTED
    assert attn_call(lib, Hq=34, Hkv=2) == T.TALON_ERR_UNSUPPORTED     # group of 17
    assert attn_call(lib, N_pad=60) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, q=0) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, q=P + 8) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, kp=0) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, st_=100) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, n=0) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, scale=-1.0) == T.TALON_ERR_INVALID_ARG
    assert attn_call(lib, ws_bytes=64) == T.TALON_ERR_WORKSPACE
    assert attn_call(lib, B=0) == T.TALON_ERR_INVALID_ARG


def test_binding_refuses_missing_library(monkeypatch):
    monkeypatch.setattr(T.binding, "_lib", None)
    monkeypatch.setattr(T.binding, "LIB_PATH", "/nonexistent/libtalon.so")
    with pytest.raises(RuntimeError, match="not built"):
        T.binding.load_library()

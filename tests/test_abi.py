"""The C-ABI library loads and exports every entry point include/lsp.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "lsp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(lsp_[a-z_]+)\s*\(", src)))


def test_header_declares_the_three_step_calls():
    names = _declared()
    for n in ("lsp_attn_step", "lsp_confidence", "lsp_commit"):
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_2603_05454_amd as lsp
    if not os.path.exists(lsp.LIB_PATH):
        from paper_2603_05454_amd.build import build
        build()
    L = lsp.lib()
    for n in _declared():
        assert hasattr(L, n), n
    assert set(lsp.EXPORTS) == set(_declared())
    assert b"gfx950" in L.lsp_version()


def test_argument_errors_are_reported_before_any_launch():
    """Host-side validation returns LSP_ERR_INVALID_ARG without touching a GPU."""
    import paper_2603_05454_amd as lsp
    L = lsp.lib()
    rc = L.lsp_confidence(7, None, 1, 1, 8, ctypes.c_int64(0), ctypes.c_int64(0), None, None, None, None,
                          None, ctypes.c_size_t(0), None)
    assert rc == -1 and b"dtype" in L.lsp_last_error()
    d = lsp.AttnDesc(dtype=1, B=1, S=4, Hq=3, Hkv=2, D=128, C=8)
    rc = L.lsp_attn_step(ctypes.byref(d), None, None, None, None, None, None, None, None, None,
                         ctypes.c_size_t(0), None)
    assert rc == -1 and b"multiple" in L.lsp_last_error()
    c = lsp.CommitDesc(B=1, S=4, V=8, C=8, min_commit=-1)
    commit_args = [None] * 17 + [ctypes.c_size_t(0), None]      # every pointer null: validation stops first
    rc = L.lsp_commit(ctypes.byref(c), *commit_args)
    assert rc == -1
    # the descriptor is checked field by field once the mandatory pointers are there
    buf = (ctypes.c_int32 * 64)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    ptrs = [p, p, None, None, None, None, None, None, p, p, p, p, p, p, None, None, None, ctypes.c_size_t(0), None]
    for bad, word in ((dict(min_commit=-1), b"min_commit"), (dict(max_commit=-2), b"max_commit"),
                      (dict(adaptive=1, alpha=0.6, beta=0.5), b"alpha"), (dict(adaptive=1, alpha=0.0, beta=0.5), b"alpha"),
                      (dict(snap_enabled=1), b"bitmap"), (dict(num_layers=2, Hkv=1, D=8, kv_dtype=1), b"layer")):
        c = lsp.CommitDesc(**{**dict(B=1, S=4, V=8, C=8), **bad})
        assert L.lsp_commit(ctypes.byref(c), *ptrs) == -1 and word in L.lsp_last_error(), bad
    # Scattered-Margin entry points
    assert L.lsp_select_scattered(None, 1, 4, None, None, None, None, None) == -1
    assert L.lsp_select_scattered(p, 1, 100000, p, p, p, p, None) == -2 and b"exceeds" in L.lsp_last_error()
    assert L.lsp_kv_gather_append(1, 1, 4, 1, 3, 8, 1, ctypes.c_int64(0), ctypes.c_int64(0), p, p, p, p, p, p, p, p, None) == -1
    assert b"multiple of 16" in L.lsp_last_error()
    assert L.lsp_kv_gather_append(1, 1, 4, 1, 8, 8, 1, ctypes.c_int64(0), ctypes.c_int64(0), p, p, p, p, p, p, p, None, None) == -1
    assert b"null pointer" in L.lsp_last_error()        # appended is a required output
    # the multi-layer attention call
    d = lsp.AttnDesc(dtype=1, B=1, S=4, Hq=2, Hkv=2, D=128, C=8)
    assert L.lsp_attn_step_layers(ctypes.byref(d), 0, p, p, p, p, p, p, p, p, None, ctypes.c_size_t(0), None) == -1
    assert b"num_layers" in L.lsp_last_error()
    tbl = (ctypes.c_void_p * 2)(ctypes.addressof(buf), 0)
    assert L.lsp_attn_step_layers(ctypes.byref(d), 2, tbl, tbl, tbl, tbl, tbl, p, p, tbl, None, ctypes.c_size_t(0), None) == -1
    assert b"layer 1" in L.lsp_last_error()
    d = lsp.AttnDesc(dtype=1, B=1, S=4, Hq=2, Hkv=2, D=128, C=8)
    rc = L.lsp_attn_step_gather(ctypes.byref(d), p, p, p, p, p, None, p, p, p, None, ctypes.c_size_t(0), None)
    assert rc == -1 and b"row index" in L.lsp_last_error()
    d = lsp.AttnDesc(dtype=1, B=1, S=4, Hq=2, Hkv=2, D=96, C=8)
    sixteen = ctypes.c_void_p((ctypes.addressof(buf) + 15) & ~15)
    args = [sixteen] * 5 + [sixteen, sixteen, sixteen, None, ctypes.c_size_t(0), None]
    assert L.lsp_attn_step(ctypes.byref(d), *args) == -2 and b"head_dim" in L.lsp_last_error()
    d = lsp.AttnDesc(dtype=1, B=1, S=4, Hq=2, Hkv=2, D=128, C=8)
    d.cache_stride[0], d.cache_stride[1], d.cache_stride[2] = 8 << 25, 1 << 25, 128
    assert L.lsp_attn_step(ctypes.byref(d), *args) == -1 and b"row strides" in L.lsp_last_error()

    # output head: dtype, K granularity, strides, workspace (all before any launch)
    i64 = ctypes.c_int64
    def lm(dtype=1, K=64, V=8, hrs=0, wrs=0, ws=sixteen, wsb=1 << 20, hid=sixteen):
        return L.lsp_lm_head_confidence(dtype, hid, sixteen, 1, 4, K, V, i64(hrs), i64(0), i64(wrs), None,
                                        p, p, p, ws, ctypes.c_size_t(wsb), None)
    assert lm(dtype=0) == -2 and b"bf16" in L.lsp_last_error()
    assert lm(K=60) == -1 and b"multiple of 8" in L.lsp_last_error()
    assert lm(V=1) == -1
    assert lm(hrs=32) == -1 and b"strides" in L.lsp_last_error()
    assert lm(wrs=68) == -1 and b"strides" in L.lsp_last_error()
    assert lm(hid=ctypes.c_void_p(sixteen.value + 2)) == -1 and b"aligned" in L.lsp_last_error()
    assert lm(ws=None) == -3 and lm(wsb=8) == -3 and b"workspace" in L.lsp_last_error()
    assert L.lsp_lm_head_confidence_workspace_bytes(2, 300, 1000) == 2 * 300 * 4 * 16


def test_measurement_helpers_and_flip_update_validate_on_the_host():
    import paper_2603_05454_amd as lsp
    L = lsp.lib()
    buf = (ctypes.c_int32 * 64)()
    p = ctypes.c_void_p((ctypes.addressof(buf) + 15) & ~15)
    assert L.lsp_bench_read(None, ctypes.c_int64(64), 1, p, None) == -1
    assert L.lsp_bench_read(p, ctypes.c_int64(48), 2, p, None) == -1 and b"evenly" in L.lsp_last_error()
    assert L.lsp_bench_mfma(None, 1, 1, p, None) == -1
    assert L.lsp_bench_mfma(p, 0, 1, p, None) == -1
    odd = ctypes.c_void_p(p.value + 4)
    assert L.lsp_bench_mfma(odd, 1, 1, p, None) == -1 and b"aligned" in L.lsp_last_error()
    assert L.lsp_flip_update(None, 1, 4, 4, p, p, p, p, p, 0, 0, None, None) == -1 and b"null" in L.lsp_last_error()
    assert L.lsp_flip_update(p, 0, 4, 4, p, p, p, p, p, 0, 0, None, None) == -1


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2603_05454_amd as lsp
    monkeypatch.setattr(lsp, "_lib", None)
    monkeypatch.setattr(lsp, "LIB_PATH", "/nonexistent/liblsp.so")
    with pytest.raises(lsp.LspError):
        lsp.lib()


def test_binding_refuses_tensors_of_the_wrong_type_or_shape(monkeypatch):
    """Element types and shapes do not cross a boundary of plain pointers: the binding checks
    what a kernel would otherwise misread (int64 lengths read as int32, a short index list,
    K and V of different element types) and raises before it touches the library.  (Host
    tensors stand in for device tensors here: the device check is switched off, and a call
    that got past the checks would fail the test by reaching the library without a GPU.)"""
    import torch
    import paper_2603_05454_amd as m
    monkeypatch.setattr(m, "_dev", lambda *ts: None)
    monkeypatch.setattr(m, "lib", lambda: pytest.fail("the call reached the library"))
    B, S, V = 2, 8, 64
    i32 = lambda *shape: torch.zeros(shape, dtype=torch.int32)
    f32 = lambda *shape: torch.zeros(shape, dtype=torch.float32)
    good_out = (i32(B, S), f32(B, S), f32(B, S))
    bm = i32(2)
    cases = [
        ("suffix_len must be torch.int32", lambda: m.confidence(f32(B, S, V), torch.zeros(B, dtype=torch.int64), out=good_out)),
        ("top1_id", lambda: m.confidence(f32(B, S, V), None, out=(torch.zeros((B, S), dtype=torch.int64), f32(B, S), f32(B, S)))),
        ("shape", lambda: m.confidence(f32(B, S, V), None, out=(i32(B, S + 1), f32(B, S), f32(B, S)))),
        ("contiguous", lambda: m.confidence(f32(B, S, V), None, out=(i32(S, B).t(), f32(B, S), f32(B, S)))),
        ("margin must be torch.float32", lambda: m.commit(f32(B, S).double(), i32(B, S), bm, V, 0.9, 4, 1, 1, i32(B), i32(B), C=16)),
        ("top1_id must be torch.int32", lambda: m.commit(f32(B, S), i32(B, S).long(), bm, V, 0.9, 4, 1, 1, i32(B), i32(B), C=16)),
        ("prefix_len must be torch.int32", lambda: m.commit(f32(B, S), i32(B, S), bm, V, 0.9, 4, 1, 1, i32(B).long(), i32(B), C=16)),
        ("bitmap holds 1 words", lambda: m.commit(f32(B, S), i32(B, S), i32(1), V, 0.9, 4, 1, 1, i32(B), i32(B), C=16)),
        ("tokens must be torch.int32", lambda: m.commit(f32(B, S), i32(B, S), bm, V, 0.9, 4, 1, 1, i32(B), i32(B),
                                                        tokens=torch.zeros((B, 16), dtype=torch.int64), C=16)),
        ("needs the cache capacity", lambda: m.commit(f32(B, S), i32(B, S), bm, V, 0.9, 4, 1, 1, i32(B), i32(B))),
        ("counters must be torch.int64", lambda: m.flip_update(i32(B, S), i32(B), i32(B), i32(B), i32(B, S), i32(4))),
        ("last_id must be torch.int32", lambda: m.flip_update(i32(B, S), i32(B), i32(B), i32(B), i32(B, S).long(),
                                                              torch.zeros(4, dtype=torch.int64))),
        ("count must be torch.int32", lambda: m.select_scattered(f32(B, S), i32(B), i32(B).long())),
        ("v_suf must be", lambda: m.attn_step(f32(B, S, 4, 64), f32(B, S, 2, 64), f32(B, S, 2, 64).bfloat16(),
                                              f32(B, 16, 2, 64), f32(B, 16, 2, 64), i32(B), i32(B))),
        ("k_cache must be", lambda: m.attn_step(f32(B, S, 4, 64), f32(B, S, 2, 64), f32(B, S, 2, 64),
                                                f32(B, 16, 1, 64), f32(B, 16, 1, 64), i32(B), i32(B))),
        ("prefix_len must be torch.int32", lambda: m.attn_step(f32(B, S, 4, 64), f32(B, S, 2, 64), f32(B, S, 2, 64),
                                                               f32(B, 16, 2, 64), f32(B, 16, 2, 64), i32(B).long(), i32(B))),
        ("weight must be", lambda: m.lm_head_confidence(f32(B, S, 32).bfloat16(), f32(V, 32))),
    ]
    for text, call in cases:
        with pytest.raises(m.LspError, match=text):
            call()

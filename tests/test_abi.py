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
    rc = L.lsp_commit(ctypes.byref(c), None, None, None, None, None, None, None, None, None, None, None,
                      None, None, None, None, None, ctypes.c_size_t(0), None)
    assert rc == -1


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2603_05454_amd as lsp
    monkeypatch.setattr(lsp, "_lib", None)
    monkeypatch.setattr(lsp, "LIB_PATH", "/nonexistent/liblsp.so")
    with pytest.raises(lsp.LspError):
        lsp.lib()

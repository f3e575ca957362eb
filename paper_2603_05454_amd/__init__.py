"""Python binding of liblsp (the LSP per-step hot path for MI355X).

Argument marshalling only: every function takes torch tensors that already
live on the GPU, passes their pointers and the current HIP stream to the C-ABI
entry point of the same name (include/lsp.h) and returns the output tensors.
There is no fallback: importing works without the built library (so that the
package can be inspected), but the first call raises if liblsp.so is missing.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblsp.so")
_lib = None

LSP_F32, LSP_BF16 = 0, 1
FLAG_CACHE_FULL, FLAG_TOKENS_FULL = 1, 2


class LspError(RuntimeError):
    pass


class AttnDesc(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("S", ctypes.c_int32),
                ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
                ("C", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride", ctypes.c_int64 * 3), ("kv_suf_stride", ctypes.c_int64 * 3),
                ("cache_stride", ctypes.c_int64 * 3), ("o_stride", ctypes.c_int64 * 3)]


class CommitDesc(ctypes.Structure):
    _fields_ = [("kv_dtype", ctypes.c_int32), ("B", ctypes.c_int32), ("S", ctypes.c_int32),
                ("V", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
                ("C", ctypes.c_int32), ("num_layers", ctypes.c_int32), ("T", ctypes.c_int32),
                ("tau", ctypes.c_float), ("window", ctypes.c_int32), ("min_commit", ctypes.c_int32),
                ("snap_enabled", ctypes.c_int32), ("suf_batch_stride", ctypes.c_int64),
                ("cache_batch_stride", ctypes.c_int64), ("adaptive", ctypes.c_int32),
                ("alpha", ctypes.c_float), ("beta", ctypes.c_float), ("max_commit", ctypes.c_int32)]


EXPORTS = ["lsp_version", "lsp_last_error", "lsp_attn_workspace_bytes", "lsp_attn_step", "lsp_attn_step_layers",
           "lsp_confidence_workspace_bytes", "lsp_confidence", "lsp_confidence_static_scratch_bytes",
           "lsp_confidence_static", "lsp_commit_workspace_bytes",
           "lsp_commit", "lsp_flip_update", "lsp_select_scattered", "lsp_kv_gather_append",
           "lsp_attn_step_gather", "lsp_lm_head_confidence_workspace_bytes", "lsp_lm_head_confidence", "lsp_bench_read", "lsp_bench_mfma"]


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises LspError when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise LspError(f"{LIB_PATH} is missing: run `python -m paper_2603_05454_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        L.lsp_version.restype = ctypes.c_char_p
        L.lsp_last_error.restype = ctypes.c_char_p
        for n in ("lsp_attn_workspace_bytes", "lsp_confidence_workspace_bytes", "lsp_commit_workspace_bytes",
                  "lsp_lm_head_confidence_workspace_bytes", "lsp_confidence_static_scratch_bytes"):
            getattr(L, n).restype = ctypes.c_size_t
        for n in ("lsp_attn_step", "lsp_attn_step_layers", "lsp_confidence", "lsp_confidence_static", "lsp_commit", "lsp_flip_update", "lsp_select_scattered",
                  "lsp_kv_gather_append", "lsp_attn_step_gather", "lsp_lm_head_confidence", "lsp_bench_read", "lsp_bench_mfma"):
            getattr(L, n).restype = ctypes.c_int32
        _lib = L
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise LspError(f"{what} failed with status {rc}: {lib().lsp_last_error().decode()}")


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _dtype(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return LSP_F32
    if t.dtype == torch.bfloat16:
        return LSP_BF16
    raise LspError(f"unsupported element type {t.dtype}")


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise LspError("liblsp takes device tensors only")


def _need(name, t, dtype, shape=None, optional=False):
    """A tensor whose element type the library cannot see through a plain pointer: the
    wrong type or shape here would make a kernel read lengths or indices that are not
    there, so it is refused before anything is launched."""
    if t is None:
        if optional:
            return
        raise LspError(f"{name} is required")
    if t.dtype != dtype and not (isinstance(dtype, tuple) and t.dtype in dtype):
        raise LspError(f"{name} must be {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise LspError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if not t.is_contiguous():
        raise LspError(f"{name} must be contiguous")


def _need_kv(q, k_suf, v_suf, k_cache, v_cache, out):
    B, S, Hq, D = q.shape
    Hkv, C = k_suf.shape[2], k_cache.shape[1]
    for name, t, shape in (("k_suf", k_suf, (B, S, Hkv, D)), ("v_suf", v_suf, (B, S, Hkv, D)),
                           ("k_cache", k_cache, (B, C, Hkv, D)), ("v_cache", v_cache, (B, C, Hkv, D)),
                           ("out", out, (B, S, Hq, D))):
        if t.dtype != q.dtype or tuple(t.shape) != shape:
            raise LspError(f"{name} must be {q.dtype} {shape}, got {t.dtype} {tuple(t.shape)}")
    if v_suf.stride() != k_suf.stride() or v_cache.stride() != k_cache.stride():
        raise LspError("K and V must share strides")


def _need_conf_out(out, B, S):
    if len(out) != 3:
        raise LspError("out must be (top1_id, top1_prob, margin)")
    _need("out[0] (top1_id)", out[0], torch.int32, (B, S))
    _need("out[1] (top1_prob)", out[1], torch.float32, (B, S))
    _need("out[2] (margin)", out[2], torch.float32, (B, S))


def version() -> str:
    return lib().lsp_version().decode()


def _strides3(t):
    if t.dim() != 4 or t.stride(3) != 1:
        raise LspError("attention operands are [batch, row, head, D] with a contiguous innermost dimension")
    return (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def attn_workspace_bytes(dtype, B, S, Hq, Hkv, D, C) -> int:
    d = AttnDesc(dtype=dtype, B=B, S=S, Hq=Hq, Hkv=Hkv, D=D, C=C)
    return lib().lsp_attn_workspace_bytes(ctypes.byref(d))


def attn_step(q, k_suf, v_suf, k_cache, v_cache, prefix_len, suffix_len, scale=0.0, out=None,
              workspace=None, cache_row_index=None):
    """lsp_attn_step: q [B,S,Hq,D], k_suf/v_suf [B,S,Hkv,D], caches [B,C,Hkv,D],
    prefix_len/suffix_len int32 [B].  Returns out [B,S,Hq,D] (same dtype as q);
    rows >= suffix_len[b] are not written.  cache_row_index int32 [B,C] selects
    lsp_attn_step_gather (key t of the prefix is cache row cache_row_index[b,t])."""
    _dev(q, k_suf, v_suf, k_cache, v_cache, prefix_len, suffix_len, cache_row_index, out)
    B, S, Hq, D = q.shape
    if out is None:
        out = torch.empty((B, S, Hq, D), dtype=q.dtype, device=q.device)
    _need_kv(q, k_suf, v_suf, k_cache, v_cache, out)
    _need("prefix_len", prefix_len, torch.int32, (B,))
    _need("suffix_len", suffix_len, torch.int32, (B,))
    d = AttnDesc(dtype=_dtype(q), B=B, S=S, Hq=Hq, Hkv=k_suf.shape[2], D=D, C=k_cache.shape[1],
                 scale=float(scale))
    d.q_stride = _strides3(q)
    d.kv_suf_stride = _strides3(k_suf)
    d.cache_stride = _strides3(k_cache)
    d.o_stride = _strides3(out)
    need = lib().lsp_attn_workspace_bytes(ctypes.byref(d))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if cache_row_index is None:
        rc = lib().lsp_attn_step(ctypes.byref(d), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_cache),
                                 _ptr(v_cache), _ptr(prefix_len), _ptr(suffix_len), _ptr(out),
                                 _ptr(workspace), ctypes.c_size_t(wb), _stream())
    else:
        _need("cache_row_index", cache_row_index, torch.int32, (B, k_cache.shape[1]))
        rc = lib().lsp_attn_step_gather(ctypes.byref(d), _ptr(q), _ptr(k_suf), _ptr(v_suf), _ptr(k_cache),
                                        _ptr(v_cache), _ptr(cache_row_index), _ptr(prefix_len),
                                        _ptr(suffix_len), _ptr(out), _ptr(workspace), ctypes.c_size_t(wb),
                                        _stream())
    _check(rc, "lsp_attn_step")
    return out


class AttnLayerTable:
    """Host arrays of per-layer device pointers for lsp_attn_step_layers, built once and
    reused (all layers must share shape, dtype and strides)."""

    def __init__(self, q, k_suf, v_suf, k_cache, v_cache, out):
        n = len(q)
        if not (len(k_suf) == len(v_suf) == len(k_cache) == len(v_cache) == len(out) == n > 0):
            raise LspError("AttnLayerTable: one tensor of each kind per layer, at least one layer")
        for lst in (q, k_suf, v_suf, k_cache, v_cache, out):
            for t in lst:
                _dev(t)
                if t.shape != lst[0].shape or t.stride() != lst[0].stride() or t.dtype != q[0].dtype:
                    raise LspError("AttnLayerTable: all layers must share shape, strides and element type")
        _need_kv(q[0], k_suf[0], v_suf[0], k_cache[0], v_cache[0], out[0])
        Arr = ctypes.c_void_p * n
        self.n = n
        self.arrays = [Arr(*[t.data_ptr() for t in lst]) for lst in (q, k_suf, v_suf, k_cache, v_cache, out)]
        self.keep = (q, k_suf, v_suf, k_cache, v_cache, out)
        B, S, Hq, D = q[0].shape
        self.desc = AttnDesc(dtype=_dtype(q[0]), B=B, S=S, Hq=Hq, Hkv=k_suf[0].shape[2], D=D, C=k_cache[0].shape[1])
        self.desc.q_stride = _strides3(q[0])
        self.desc.kv_suf_stride = _strides3(k_suf[0])
        self.desc.cache_stride = _strides3(k_cache[0])
        self.desc.o_stride = _strides3(out[0])
        self.out = out


def attn_step_layers(table: AttnLayerTable, prefix_len, suffix_len, scale=0.0, workspace=None):
    """lsp_attn_step_layers: the attention of every layer of `table` in one launch.
    Returns the list of per-layer outputs (table.out)."""
    _dev(prefix_len, suffix_len)
    _need("prefix_len", prefix_len, torch.int32, (table.desc.B,))
    _need("suffix_len", suffix_len, torch.int32, (table.desc.B,))
    table.desc.scale = float(scale)
    need = lib().lsp_attn_workspace_bytes(ctypes.byref(table.desc))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=prefix_len.device)
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a = table.arrays
    rc = lib().lsp_attn_step_layers(ctypes.byref(table.desc), table.n, a[0], a[1], a[2], a[3], a[4],
                                    _ptr(prefix_len), _ptr(suffix_len), a[5], _ptr(workspace),
                                    ctypes.c_size_t(wb), _stream())
    _check(rc, "lsp_attn_step_layers")
    return table.out


def confidence_workspace_bytes(B, S, V) -> int:
    return lib().lsp_confidence_workspace_bytes(B, S, V)


def confidence(logits, suffix_len=None, out=None, workspace=None):
    """lsp_confidence: logits [B,S,V] -> (top1_id int32, top1_prob f32, margin f32), [B,S]."""
    _dev(logits, suffix_len)
    B, S, V = logits.shape
    if logits.stride(2) != 1:
        raise LspError("logits rows must be contiguous")
    if out is None:
        out = (torch.empty((B, S), dtype=torch.int32, device=logits.device),
               torch.empty((B, S), dtype=torch.float32, device=logits.device),
               torch.empty((B, S), dtype=torch.float32, device=logits.device))
    _dev(*out)
    _need_conf_out(out, B, S)
    _need("suffix_len", suffix_len, torch.int32, (B,), optional=True)
    need = lib().lsp_confidence_workspace_bytes(B, S, V)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=logits.device)
    wb = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().lsp_confidence(_dtype(logits), _ptr(logits), B, S, V,
                              ctypes.c_int64(logits.stride(1)), ctypes.c_int64(logits.stride(0)),
                              _ptr(suffix_len), _ptr(out[0]), _ptr(out[1]), _ptr(out[2]),
                              _ptr(workspace), ctypes.c_size_t(wb), _stream())
    _check(rc, "lsp_confidence")
    return out


def confidence_static(logits, suffix_len, out):
    """lsp_confidence_static: lsp_confidence without a workspace and without any
    allocation; `out` = (top1_id int32, top1_prob f32, margin f32), [B,S], is required."""
    _dev(logits, suffix_len, *out)
    B, S, V = logits.shape
    if logits.stride(2) != 1:
        raise LspError("logits rows must be contiguous")
    _need_conf_out(out, B, S)
    _need("suffix_len", suffix_len, torch.int32, (B,), optional=True)
    rc = lib().lsp_confidence_static(_dtype(logits), _ptr(logits), B, S, V,
                                     ctypes.c_int64(logits.stride(1)), ctypes.c_int64(logits.stride(0)),
                                     _ptr(suffix_len), _ptr(out[0]), _ptr(out[1]), _ptr(out[2]), _stream())
    _check(rc, "lsp_confidence_static")
    return out


def lm_head_confidence_workspace_bytes(B, S, V) -> int:
    return lib().lsp_lm_head_confidence_workspace_bytes(B, S, V)


def lm_head_confidence(hidden, weight, suffix_len=None, out=None, workspace=None):
    """lsp_lm_head_confidence: hidden [B,S,K], weight [V,K] (bf16) ->
    (top1_id int32, top1_prob f32, margin f32), [B,S], of the logits hidden @ weight.T,
    which are never stored."""
    _dev(hidden, weight, suffix_len)
    B, S, K = hidden.shape
    V = weight.shape[0]
    if weight.dim() != 2 or weight.shape[1] != K or weight.dtype != hidden.dtype:
        raise LspError(f"weight must be {hidden.dtype} [V, {K}], got {weight.dtype} {tuple(weight.shape)}")
    if hidden.stride(2) != 1 or weight.stride(1) != 1:
        raise LspError("hidden and weight rows must be contiguous")
    if out is None:
        out = (torch.empty((B, S), dtype=torch.int32, device=hidden.device),
               torch.empty((B, S), dtype=torch.float32, device=hidden.device),
               torch.empty((B, S), dtype=torch.float32, device=hidden.device))
    _dev(*out)
    _need_conf_out(out, B, S)
    _need("suffix_len", suffix_len, torch.int32, (B,), optional=True)
    need = lib().lsp_lm_head_confidence_workspace_bytes(B, S, V)
    if workspace is None or workspace.numel() * workspace.element_size() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=hidden.device)
    wb = workspace.numel() * workspace.element_size()
    rc = lib().lsp_lm_head_confidence(_dtype(hidden), _ptr(hidden), _ptr(weight), B, S, K, V,
                                      ctypes.c_int64(hidden.stride(1)), ctypes.c_int64(hidden.stride(0)),
                                      ctypes.c_int64(weight.stride(0)),
                                      _ptr(suffix_len), _ptr(out[0]), _ptr(out[1]), _ptr(out[2]),
                                      _ptr(workspace), ctypes.c_size_t(wb), _stream())
    _check(rc, "lsp_lm_head_confidence")
    return out


class LayerTable:
    """Host arrays of per-layer device pointers, built once and reused."""

    def __init__(self, k_suf, v_suf, k_cache, v_cache):
        n = len(k_suf)
        if not (len(v_suf) == len(k_cache) == len(v_cache) == n > 0):
            raise LspError("LayerTable: one tensor of each kind per layer, at least one layer")
        for lst in (k_suf, v_suf, k_cache, v_cache):
            for t in lst:
                _dev(t)
                if t.dim() != 4 or t.dtype != k_suf[0].dtype or t.shape != lst[0].shape or t.stride() != lst[0].stride():
                    raise LspError("LayerTable: all layers must share shape, strides and element type")
                if not (t.is_contiguous() or (t.stride(3) == 1 and t.stride(2) == t.shape[3]
                                              and t.stride(1) == t.shape[2] * t.shape[3])):
                    raise LspError("LayerTable: the rows of a sequence must be dense (only the batch stride is free)")
        if k_cache[0].shape[0] != k_suf[0].shape[0] or k_cache[0].shape[2:] != k_suf[0].shape[2:]:
            raise LspError("LayerTable: caches and suffix buffers disagree on batch, heads or head size")
        Arr = ctypes.c_void_p * n
        self.n = n
        self.arrays = [Arr(*[t.data_ptr() for t in lst]) for lst in (k_suf, v_suf, k_cache, v_cache)]
        self.keep = (k_suf, v_suf, k_cache, v_cache)
        self.kv_dtype = _dtype(k_suf[0])
        self.B = k_suf[0].shape[0]
        self.S, self.Hkv, self.D = k_suf[0].shape[1:]
        self.C = k_cache[0].shape[1]
        self.suf_bs = k_suf[0].stride(0)
        self.cache_bs = k_cache[0].stride(0)


def commit(margin, top1_id, bitmap, V, tau, window, min_commit, snap_enabled,
           prefix_len, suffix_len, tokens=None, layers: LayerTable | None = None, C=None, out=None,
           adaptive=False, alpha=0.25, beta=0.5, max_commit=0):
    """lsp_commit.  Mutates tokens, prefix_len, suffix_len and the caches of
    `layers` in place.  Returns dict(stable_mask, raw_boundary, snapped_boundary,
    commit_len, status_flags, tau_used)."""
    _dev(margin, top1_id, bitmap, prefix_len, suffix_len, tokens)
    B, S = margin.shape
    dev = margin.device
    _need("margin", margin, torch.float32, (B, S))
    _need("top1_id", top1_id, torch.int32, (B, S))
    _need("bitmap", bitmap, (torch.int32, torch.uint32))     # 32 vocabulary ids per word, either way of naming the bits
    if bitmap.numel() < (int(V) + 31) // 32:
        raise LspError(f"bitmap holds {bitmap.numel()} words, V = {V} needs {(int(V) + 31) // 32}")
    _need("prefix_len", prefix_len, torch.int32, (B,))
    _need("suffix_len", suffix_len, torch.int32, (B,))
    if tokens is not None:
        _need("tokens", tokens, torch.int32, (B, tokens.shape[1]) if tokens.dim() == 2 else (B, -1))
    if out is None:
        out = {"stable_mask": torch.empty((B, S), dtype=torch.uint8, device=dev)}
        for k in ("raw_boundary", "snapped_boundary", "commit_len", "status_flags"):
            out[k] = torch.empty(B, dtype=torch.int32, device=dev)
        out["tau_used"] = torch.empty(B, dtype=torch.float32, device=dev)
    _dev(*out.values())
    _need("out['stable_mask']", out["stable_mask"], torch.uint8, (B, S))
    for k in ("raw_boundary", "snapped_boundary", "commit_len", "status_flags"):
        _need(f"out['{k}']", out[k], torch.int32, (B,))
    _need("out['tau_used']", out.get("tau_used"), torch.float32, (B,), optional=True)
    d = CommitDesc(B=B, S=S, V=V, tau=float(tau), window=int(window), min_commit=int(min_commit),
                   snap_enabled=int(snap_enabled), T=0 if tokens is None else tokens.shape[1],
                   adaptive=int(bool(adaptive)), alpha=float(alpha), beta=float(beta), max_commit=int(max_commit))
    if layers is not None:
        if layers.S != S or layers.B != B:
            raise LspError(f"layers hold [{layers.B}, {layers.S}] suffix rows, margin is [{B}, {S}]")
        d.kv_dtype, d.Hkv, d.D, d.C, d.num_layers = layers.kv_dtype, layers.Hkv, layers.D, layers.C, layers.n
        d.suf_batch_stride, d.cache_batch_stride = layers.suf_bs, layers.cache_bs
        arrs = layers.arrays
    else:
        if C is None:
            raise LspError("commit without layers needs the cache capacity C")
        d.C, d.num_layers = C, 0
        arrs = [ctypes.c_void_p(0)] * 4
    rc = lib().lsp_commit(ctypes.byref(d), _ptr(margin), _ptr(top1_id), _ptr(bitmap),
                          arrs[0], arrs[1], arrs[2], arrs[3], _ptr(tokens), _ptr(prefix_len),
                          _ptr(suffix_len), _ptr(out["stable_mask"]), _ptr(out["raw_boundary"]),
                          _ptr(out["snapped_boundary"]), _ptr(out["commit_len"]),
                          _ptr(out["status_flags"]), _ptr(out.get("tau_used")), ctypes.c_void_p(0),
                          ctypes.c_size_t(0), _stream())
    _check(rc, "lsp_commit")
    return out


def flip_update(top1_id, prefix_len, suffix_len, base_prefix_len, last_id, counters, window=None, step_counts=None):
    """lsp_flip_update: accumulate counters (int64[4]: flips, positions compared, and the
    same two for sequences whose committed count lies in window = (lo, hi), inclusive);
    step_counts int32 [B,2], when given, receives this call's per-sequence counts."""
    _dev(top1_id, prefix_len, suffix_len, base_prefix_len, last_id, counters, step_counts)
    B, S = top1_id.shape
    _need("top1_id", top1_id, torch.int32, (B, S))
    _need("prefix_len", prefix_len, torch.int32, (B,))
    _need("suffix_len", suffix_len, torch.int32, (B,))
    _need("base_prefix_len", base_prefix_len, torch.int32, (B,))
    _need("last_id", last_id, torch.int32, (B, last_id.shape[1]) if last_id.dim() == 2 else (B, -1))
    _need("counters", counters, torch.int64, (4,))
    _need("step_counts", step_counts, torch.int32, (B, 2), optional=True)
    lo, hi = (1, 0) if window is None else window
    rc = lib().lsp_flip_update(_ptr(top1_id), B, S, last_id.shape[1], _ptr(prefix_len), _ptr(suffix_len),
                               _ptr(base_prefix_len), _ptr(last_id), _ptr(counters), int(lo), int(hi),
                               _ptr(step_counts), _stream())
    _check(rc, "lsp_flip_update")


def select_scattered(margin, suffix_len, count, out=None):
    """lsp_select_scattered: the count[b] highest-margin active positions of every
    sequence.  Returns (sel_index int32 [B,S] ascending, -1 padded; sel_mask uint8 [B,S])."""
    _dev(margin, suffix_len, count)
    B, S = margin.shape
    if out is None:
        out = (torch.empty((B, S), dtype=torch.int32, device=margin.device),
               torch.empty((B, S), dtype=torch.uint8, device=margin.device))
    _dev(*out)
    _need("margin", margin, torch.float32, (B, S))
    _need("suffix_len", suffix_len, torch.int32, (B,))
    _need("count", count, torch.int32, (B,))
    _need("out[0] (sel_index)", out[0], torch.int32, (B, S))
    _need("out[1] (sel_mask)", out[1], torch.uint8, (B, S))
    rc = lib().lsp_select_scattered(_ptr(margin), B, S, _ptr(suffix_len), _ptr(count), _ptr(out[0]),
                                    _ptr(out[1]), _stream())
    _check(rc, "lsp_select_scattered")
    return out


def kv_gather_append(sel_index, count, prefix_len, layers: LayerTable, appended=None):
    """lsp_kv_gather_append: cache rows [P_b, P_b+k_b) <- suffix rows sel_index[b, :k_b]
    for every layer of `layers`; prefix_len advanced in place.  Returns appended int32 [B]."""
    _dev(sel_index, count, prefix_len, appended)
    B, S = sel_index.shape
    if layers.S != S or layers.B != B:
        raise LspError(f"layers hold [{layers.B}, {layers.S}] suffix rows, sel_index is [{B}, {S}]")
    if appended is None:
        appended = torch.empty(B, dtype=torch.int32, device=sel_index.device)
    _need("sel_index", sel_index, torch.int32, (B, S))
    _need("count", count, torch.int32, (B,))
    _need("prefix_len", prefix_len, torch.int32, (B,))
    _need("appended", appended, torch.int32, (B,))
    a = layers.arrays
    rc = lib().lsp_kv_gather_append(layers.kv_dtype, B, S, layers.Hkv, layers.D, layers.C, layers.n,
                                    ctypes.c_int64(layers.suf_bs), ctypes.c_int64(layers.cache_bs),
                                    _ptr(sel_index), _ptr(count), a[0], a[1], a[2], a[3], _ptr(prefix_len),
                                    _ptr(appended), _stream())
    _check(rc, "lsp_kv_gather_append")
    return appended


def bench_read(buffer, workgroups, out):
    """lsp_bench_read: bare streaming read of a device buffer (measurement helper)."""
    _dev(buffer, out)
    nbytes = buffer.numel() * buffer.element_size()
    rc = lib().lsp_bench_read(_ptr(buffer), ctypes.c_int64(nbytes), int(workgroups), _ptr(out), _stream())
    _check(rc, "lsp_bench_read")


MFMA_BENCH_OPERAND_BYTES = 16 * 512 * 16
MFMA_BENCH_FLOP_PER_WG_ITER = 8 * 8 * 2 * 32 * 32 * 16


def bench_mfma(operands, iters, workgroups, out):
    """lsp_bench_mfma: bare matrix-instruction loop on the given operand values (measurement helper)."""
    _dev(operands, out)
    if operands.numel() * operands.element_size() < MFMA_BENCH_OPERAND_BYTES:
        raise ValueError("bench_mfma: operands must hold 16 * 512 * 16 bytes")
    if out.numel() < int(workgroups) * 512 or out.dtype != torch.float32:
        raise ValueError("bench_mfma: out must be float32 [workgroups * 512]")
    rc = lib().lsp_bench_mfma(_ptr(operands), int(iters), int(workgroups), _ptr(out), _stream())
    _check(rc, "lsp_bench_mfma")

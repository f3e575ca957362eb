"""ctypes front end of the CPU oracle (oracle/lsp_oracle.c).

TEST INFRASTRUCTURE ONLY.  May be imported by tests/, by the smoke check and by
the benchmark's cpu_baseline leg; the product package never imports it.  It
takes CPU torch tensors (fp32 or bf16), hands their memory to the C routines
and returns fresh CPU tensors.  No arithmetic happens on the Python side.
"""
from __future__ import annotations

import ctypes
import os

import torch

from .build import LIB, build

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        _lib = ctypes.CDLL(LIB)
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for the oracle's OpenMP loops (the benchmark also times it on one thread)."""
    lib().oracle_set_num_threads(int(n))


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise TypeError(t.dtype)


def _p(t):
    if t is None:
        return ctypes.c_void_p(0)
    assert t.device.type == "cpu" and t.is_contiguous()
    return ctypes.c_void_p(t.data_ptr())


def _i32(t):
    return t.to(torch.int32).contiguous()


def attention(q, k_suf, v_suf, k_cache, v_cache, prefix_len, suffix_len, scale=None, rows=None):
    """Suffix-over-[cache || suffix] attention without mask.
    q [B,S,Hq,D], k_suf/v_suf [B,S,Hkv,D], caches [B,C,Hkv,D].
    rows=None -> out [B,S,Hq,D] fp32 (rows >= suffix_len stay NaN);
    rows=[n,3] int (b,i,h) -> out [n,D]."""
    B, S, Hq, D = q.shape
    Hkv, C = k_suf.shape[2], k_cache.shape[1]
    scale = float(scale) if scale else 1.0 / (D ** 0.5)
    pl, sl = _i32(prefix_len), _i32(suffix_len)
    args = [_dt(q), _p(q), _p(k_suf), _p(v_suf), _p(k_cache), _p(v_cache), _p(pl), _p(sl),
            B, S, Hq, Hkv, D, C, ctypes.c_double(scale)]
    if rows is None:
        out = torch.full((B, S, Hq, D), float("nan"), dtype=torch.float32)
        rc = lib().oracle_attention(*args, _p(out))
    else:
        rows = _i32(rows)
        out = torch.empty((rows.shape[0], D), dtype=torch.float32)
        rc = lib().oracle_attention_rows(*args, rows.shape[0], _p(rows), _p(out))
    assert rc == 0, rc
    return out


def confidence(logits, suffix_len=None):
    """logits [B,S,V] -> (top1_id int32, top1_prob f32, margin f32), each [B,S].
    Rows >= suffix_len[b] hold id -1 / NaN."""
    B, S, V = logits.shape
    ids = torch.full((B, S), -1, dtype=torch.int32)
    prob = torch.full((B, S), float("nan"), dtype=torch.float32)
    mar = torch.full((B, S), float("nan"), dtype=torch.float32)
    sl = None if suffix_len is None else _i32(suffix_len)
    rc = lib().oracle_confidence(_dt(logits), _p(logits), B, S, V, _p(sl), _p(ids), _p(prob), _p(mar))
    assert rc == 0, f"oracle_confidence: non-finite row maximum or NaN (rc={rc})"
    return ids, prob, mar


def lm_head_confidence(hidden, weight, suffix_len=None, return_logits=False):
    """hidden [B,S,K], weight [V,K] -> (top1_id, top1_prob, margin) of the logits
    hidden @ weight.T kept in double; with return_logits also z [B,S,V] float64."""
    B, S, K = hidden.shape
    V = weight.shape[0]
    assert weight.shape[1] == K and weight.dtype == hidden.dtype
    ids = torch.full((B, S), -1, dtype=torch.int32)
    prob = torch.full((B, S), float("nan"), dtype=torch.float32)
    mar = torch.full((B, S), float("nan"), dtype=torch.float32)
    z = torch.full((B, S, V), float("nan"), dtype=torch.float64) if return_logits else None
    sl = None if suffix_len is None else _i32(suffix_len)
    rc = lib().oracle_lm_head_confidence(_dt(hidden), _p(hidden), _p(weight), B, S, K, V, _p(sl),
                                         _p(ids), _p(prob), _p(mar), _p(z))
    assert rc == 0, f"oracle_lm_head_confidence: non-finite logits (rc={rc})"
    return (ids, prob, mar, z) if return_logits else (ids, prob, mar)


def commit(margin, top1_id, bitmap, V, tau, window, min_commit, snap_enabled,
           prefix_len, suffix_len, tokens=None, k_suf=None, v_suf=None, k_cache=None, v_cache=None,
           C=None, adaptive=False, alpha=0.25, beta=0.5, max_commit=0):
    """Boundary search + snap + commit + append.  Mutates tokens, prefix_len,
    suffix_len and the cache tensors IN PLACE (pass clones).  k_suf.. are lists
    of per-layer tensors ([B,S,Hkv,D] / [B,C,Hkv,D]) or None for scan only.
    adaptive: choose the threshold per sequence so that L' falls in
    [ceil(alpha N), floor(beta N)] (Eq. 2); max_commit > 0 caps the commit length.
    Returns dict(stable_mask, raw_boundary, snapped_boundary, commit_len, status_flags, tau_used)."""
    B, S = margin.shape
    assert margin.dtype == torch.float32 and top1_id.dtype == torch.int32
    assert prefix_len.dtype == torch.int32 and suffix_len.dtype == torch.int32
    layers = 0 if k_suf is None else len(k_suf)
    if layers:
        Hkv, D, C = k_suf[0].shape[2], k_suf[0].shape[3], k_cache[0].shape[1]
        kvdt = _dt(k_suf[0])
        PtrArr = ctypes.c_void_p * layers
        arrs = [PtrArr(*[t.data_ptr() for t in lst]) for lst in (k_suf, v_suf, k_cache, v_cache)]
        for lst in (k_suf, v_suf, k_cache, v_cache):
            for t in lst:
                assert t.is_contiguous() and t.device.type == "cpu"
    else:
        Hkv = D = 1
        kvdt = 0
        assert C is not None
        arrs = [ctypes.c_void_p(0)] * 4
    T = tokens.shape[1] if tokens is not None else 0
    if tokens is not None:
        assert tokens.dtype == torch.int32
    out = {
        "stable_mask": torch.zeros((B, S), dtype=torch.uint8),
        "raw_boundary": torch.zeros(B, dtype=torch.int32),
        "snapped_boundary": torch.zeros(B, dtype=torch.int32),
        "commit_len": torch.zeros(B, dtype=torch.int32),
        "status_flags": torch.zeros(B, dtype=torch.int32),
        "tau_used": torch.zeros(B, dtype=torch.float32),
    }
    rc = lib().oracle_commit(kvdt, B, S, V, Hkv, D, C, layers, T,
                             ctypes.c_float(tau), int(window), int(min_commit), int(snap_enabled),
                             int(bool(adaptive)), ctypes.c_float(alpha), ctypes.c_float(beta), int(max_commit),
                             _p(margin), _p(top1_id), _p(bitmap),
                             arrs[0], arrs[1], arrs[2], arrs[3],
                             _p(tokens), _p(prefix_len), _p(suffix_len),
                             _p(out["stable_mask"]), _p(out["raw_boundary"]), _p(out["snapped_boundary"]),
                             _p(out["commit_len"]), _p(out["status_flags"]), _p(out["tau_used"]))
    assert rc == 0, rc
    return out


def select_scattered(margin, suffix_len, count):
    """Scattered-Margin selection: per sequence the count[b] active positions with
    the largest margins (ties: lower position).  Returns (sel_index int32 [B,S],
    ascending, padded with -1; sel_mask uint8 [B,S])."""
    B, S = margin.shape
    assert margin.dtype == torch.float32
    sl, ct = _i32(suffix_len), _i32(count)
    idx = torch.empty((B, S), dtype=torch.int32)
    mask = torch.empty((B, S), dtype=torch.uint8)
    rc = lib().oracle_select_scattered(B, S, _p(margin), _p(sl), _p(ct), _p(idx), _p(mask))
    assert rc == 0
    return idx, mask


def gather_append(sel_index, count, prefix_len, k_suf, v_suf, k_cache, v_cache):
    """Cache rows [P_b, P_b+k_b) <- suffix rows sel_index[b, :k_b] for every layer.
    Mutates the caches and prefix_len IN PLACE."""
    layers = len(k_suf)
    B, S, Hkv, D = k_suf[0].shape
    C = k_cache[0].shape[1]
    PtrArr = ctypes.c_void_p * layers
    arrs = [PtrArr(*[t.data_ptr() for t in lst]) for lst in (k_suf, v_suf, k_cache, v_cache)]
    for lst in (k_suf, v_suf, k_cache, v_cache):
        for t in lst:
            assert t.is_contiguous() and t.device.type == "cpu"
    assert sel_index.dtype == torch.int32 and prefix_len.dtype == torch.int32
    ct = _i32(count)
    rc = lib().oracle_gather_append(_dt(k_suf[0]), B, S, Hkv, D, C, layers, _p(sel_index), _p(ct),
                                    arrs[0], arrs[1], arrs[2], arrs[3], _p(prefix_len))
    assert rc == 0

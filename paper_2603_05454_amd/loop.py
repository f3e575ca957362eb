"""Outer LSP loop (Algorithm 1 lines 3-11) on the HIP library.

Host side of the scheduler: per iteration it obtains the step's logits from
the caller (the stand-in for the denoiser), runs lsp_confidence, the flip
bookkeeping and lsp_commit, optionally lsp_attn_step per layer, and stops when
no sequence has an active position left.  The only device-to-host traffic is
the termination test, polled every `poll` steps.
"""
from __future__ import annotations

import torch

from . import (AttnLayerTable, LayerTable, LspError, attn_step_layers, commit, confidence, flip_update, lm_head_confidence,
               lm_head_confidence_workspace_bytes)


def decode_loop(logits_fn, bitmap, V, tau, window, min_commit, snap_enabled,
                prefix_len, suffix_len, tokens, kv_layers=None, gen_len=None, run_attention=False,
                poll=1, max_steps=100000, stop_after=None, observer=None, timed=False, commit_kw=None,
                graph=False, lm_head_weight=None, flip_window=None, flip_trace=False, state=None):
    """logits_fn(step, prefix_len) -> device logits [B,S,V].  prefix_len,
    suffix_len, tokens and the caches in kv_layers (list of dicts q?, k_suf,
    v_suf, k_cache, v_cache) are updated in place.
    commit_kw: extra keyword arguments of commit() (adaptive, alpha, beta, max_commit).
    stop_after: leave the loop after that many steps even if positions remain.
    observer(step, logits, conf, commit_out): called after every step's commit
    (the tensors are reused by the next step: copy what is to be kept).
    timed: bracket every step's library calls with HIP events on the current
    stream and return their sum as lsp_ms (the logits callback is outside).
    lm_head_weight [V,K] (bf16): logits_fn then returns the step's HIDDEN states
    [B,S,K] and lsp_lm_head_confidence takes the place of lsp_confidence (the
    logits are never stored).
    graph: launch every step after the first from ONE captured HIP graph (all
    sequence state lives in device memory and no entry point reads it on the
    host, so the same graph serves every step); the first step runs eagerly.
    The step's logits must then sit at one address: a tensor that logits_fn
    returns elsewhere is copied there (outside the timed region).
    flip_window: (lo, hi) committed positions of a sequence, inclusive, inside which its
    flips also count towards the mid-generation window of Section 4.3.4 (default: 25 %-75 %
    of the generation length).  flip_trace: keep every step's per-sequence counts.
    state: the dict an earlier call returned under "state" (one that stop_after ended, or
    whose tensors were saved and loaded back): the call then continues that generation -
    same generation start, last-seen ids and flip counters, step numbers going on from
    where it stopped - so that stopping and resuming walks exactly like one uninterrupted
    call.  The sequence state itself (lengths, tokens, caches) is the caller's as always.
    A sequence that still has active positions but commits nothing (min_commit = 0, or its
    cache / token buffer is full) would never finish: the loop raises LspError instead.
    Returns dict(steps, flips, flip_denominator, window_flips, window_denominator, committed,
    state[, flip_trace: int32 [steps,B,2]][, lsp_ms, lsp_ms_steps]); steps, the flip counts
    and committed are totals since the generation began (earlier calls included)."""
    dev = prefix_len.device
    B = prefix_len.shape[0]
    G = int(gen_len if gen_len is not None else suffix_len.max().item())
    if state is None:
        base = prefix_len.clone()
        last_id = torch.full((B, G), -1, dtype=torch.int32, device=dev)
        counters = torch.zeros(4, dtype=torch.int64, device=dev)
        steps = 0
    else:
        base, last_id, counters, steps = state["base"], state["last_id"], state["counters"], int(state["steps"])
        if (tuple(base.shape) != (B,) or base.dtype != prefix_len.dtype or tuple(last_id.shape) != (B, G)
                or last_id.dtype != torch.int32 or tuple(counters.shape) != (4,) or counters.dtype != torch.int64
                or any(t.device != dev for t in (base, last_id, counters)) or steps < 0):
            raise LspError("decode_loop: state does not belong to this batch (shapes, dtypes or device differ)")
    first = steps
    if flip_window is None:
        flip_window = (-(-G // 4), (3 * G) // 4)
    step_counts = torch.zeros((B, 2), dtype=torch.int32, device=dev) if flip_trace else None
    trace = []
    if min_commit < 1 and stop_after is None:
        raise LspError("decode_loop needs min_commit >= 1 (Section 3.2: at least one token per iteration) "
                       "unless stop_after bounds the number of steps")
    table = None
    if kv_layers is not None:
        table = LayerTable([L["k_suf"] for L in kv_layers], [L["v_suf"] for L in kv_layers],
                           [L["k_cache"] for L in kv_layers], [L["v_cache"] for L in kv_layers])
    out = conf = None
    attn_out = None
    events = []
    zbuf = step_graph = None
    lm_ws = None   # workspace of the fused output head: allocated by the first (eager) step, then reused

    def one_step(z):
        nonlocal out, conf, attn_out, lm_ws
        if run_attention and kv_layers is not None:
            if attn_out is None:     # one output per layer (a denoiser consumes each of them), allocated once
                attn_out = AttnLayerTable(*[[L[k] for L in kv_layers] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")],
                                          [torch.empty_like(L["q"]) for L in kv_layers])
            attn_step_layers(attn_out, prefix_len, suffix_len)     # every layer in one launch
        if lm_head_weight is None:
            conf = confidence(z, suffix_len, out=conf)
        else:
            if lm_ws is None:
                lm_ws = torch.empty(lm_head_confidence_workspace_bytes(z.shape[0], z.shape[1], V), dtype=torch.uint8, device=dev)
            conf = lm_head_confidence(z, lm_head_weight, suffix_len, out=conf, workspace=lm_ws)
        flip_update(conf[0], prefix_len, suffix_len, base, last_id, counters, window=flip_window,
                    step_counts=step_counts)
        out = commit(conf[2], conf[0], bitmap, V, tau, window, min_commit, snap_enabled,
                     prefix_len, suffix_len, tokens=tokens, layers=table, C=tokens.shape[1], out=out,
                     **(commit_kw or {}))

    while True:
        if (steps - first) % poll == 0:
            if out is None:
                left, stalled = int(suffix_len.max().item()), 0
            else:   # one transfer: positions left, and whether a sequence that has some committed nothing
                left, stalled = torch.stack([suffix_len.max(), ((out["commit_len"] == 0) & (suffix_len > 0)).any().to(torch.int32)]).tolist()
            if left == 0:
                break
            if stalled and min_commit >= 1:
                raise LspError(f"decode_loop: a sequence with active positions committed nothing at step {steps - 1} "
                               f"(status_flags {out['status_flags'].tolist()}): cache or token buffer full")
        if stop_after is not None and steps - first >= stop_after:
            break
        assert steps < max_steps
        z = logits_fn(steps, prefix_len)
        if graph:
            if zbuf is None:
                zbuf = z
            elif z.data_ptr() != zbuf.data_ptr():
                zbuf.copy_(z)
                z = zbuf
        if graph and steps - first >= 1 and step_graph is None:   # one-time set-up, not part of a step
            step_graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(step_graph):
                one_step(zbuf)
        if timed:
            events.append((torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)))
            events[-1][0].record()
        if graph and steps - first >= 1:
            step_graph.replay()
        else:
            one_step(z)
        if timed:
            events[-1][1].record()
        if step_counts is not None:
            trace.append(step_counts.clone())
        if observer is not None:
            observer(steps, z, conf, out)
        steps += 1
    c = counters.tolist()
    committed = int((prefix_len - base).sum().item())
    res = dict(steps=steps, flips=c[0], flip_denominator=c[1], window_flips=c[2], window_denominator=c[3],
               committed=committed, state=dict(base=base, last_id=last_id, counters=counters, steps=steps))
    if flip_trace:
        res["flip_trace"] = torch.stack(trace).cpu() if trace else torch.zeros((0, B, 2), dtype=torch.int32)
    if timed:
        torch.cuda.synchronize()
        res["lsp_ms_steps"] = [a.elapsed_time(b) for a, b in events]
        res["lsp_ms"] = sum(res["lsp_ms_steps"])
    return res

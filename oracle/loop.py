"""Outer LSP loop (Algorithm 1 lines 3-11) on the CPU oracle.  TEST
INFRASTRUCTURE ONLY (see oracle/lsp_oracle.c).

Each iteration asks the caller for this step's logits over the still-active
rows, takes id / margin (Eq. 1), finds and snaps the boundary, commits and
appends, until no sequence has an active position left.  It also counts top-1
flips (Section 4.3.4): positions that are still active at step k and whose
top-1 id differs from the one they had at step k-1, in total and restricted to
the mid-stage of generation (a sequence counts towards the window while the
number of its positions already committed lies in [window_lo, window_hi],
25 %-75 % of its generation length by default).
"""
from __future__ import annotations

import torch

from . import commit, confidence, lm_head_confidence


def decode_loop(logits_fn, bitmap, V, tau, window, min_commit, snap_enabled,
                prefix_len, suffix_len, tokens, kv_layers=None, max_steps=100000, trace=False,
                commit_kw=None, lm_head_weight=None, window_lo=None, window_hi=None):
    """logits_fn(step, prefix_len) -> [B,S,V] CPU tensor (row u = u-th active position).
    prefix_len / suffix_len / tokens / kv_layers (list of dicts with k_suf,
    v_suf [B,S,Hkv,D], row u = u-th active position, reused unchanged by every
    step, and k_cache, v_cache) are updated in place.
    commit_kw: extra keyword arguments of oracle.commit (adaptive, alpha, beta, max_commit).
    lm_head_weight [V,K]: logits_fn then returns the step's HIDDEN states [B,S,K] and
    the logits are hidden @ weight.T kept in double (Algorithm 1 lines 4-5 together).
    window_lo / window_hi: bounds (in committed positions of a sequence, inclusive) of the
    mid-generation window of Section 4.3.4; default ceil(G/4) and floor(3G/4).
    Returns dict(steps, flips, flip_denominator, window_flips, window_denominator, committed,
    flip_trace=[per step: (flips, positions compared), each a [B] tensor], per_step=[...])."""
    B = prefix_len.shape[0]
    P0 = prefix_len.clone()
    G = int(suffix_len.max())
    prev = torch.full((B, G), -1, dtype=torch.int64)
    steps = flips = denom = committed = 0
    wflips = wdenom = 0
    if window_lo is None:
        window_lo = -(-G // 4)
    if window_hi is None:
        window_hi = (3 * G) // 4
    per_step = []
    flip_trace = []
    while int(suffix_len.max()) > 0:
        assert steps < max_steps
        z = logits_fn(steps, prefix_len)
        if lm_head_weight is None:
            ids, prob, mar = confidence(z, suffix_len)
        else:
            ids, prob, mar = lm_head_confidence(z, lm_head_weight, suffix_len)
        done = (prefix_len - P0).long()
        f_step = torch.zeros(B, dtype=torch.int64)
        d_step = torch.zeros(B, dtype=torch.int64)
        for b in range(B):
            n = int(suffix_len[b])
            cur = ids[b, :n].long()
            old = prev[b, done[b]:done[b] + n]
            seen = old >= 0
            f_step[b] = int(((cur != old) & seen).sum())
            d_step[b] = int(seen.sum())
            prev[b, done[b]:done[b] + n] = cur
            if window_lo <= int(done[b]) <= window_hi:
                wflips += int(f_step[b])
                wdenom += int(d_step[b])
        flips += int(f_step.sum())
        denom += int(d_step.sum())
        flip_trace.append((f_step, d_step))
        kw = dict(commit_kw or {})
        if kv_layers is not None:
            kw.update(k_suf=[L["k_suf"] for L in kv_layers], v_suf=[L["v_suf"] for L in kv_layers],
                      k_cache=[L["k_cache"] for L in kv_layers], v_cache=[L["v_cache"] for L in kv_layers])
        out = commit(mar, ids, bitmap, V, tau, window, min_commit, snap_enabled,
                     prefix_len, suffix_len, tokens=tokens, C=tokens.shape[1], **kw)
        committed += int(out["commit_len"].sum())
        if trace:
            per_step.append({k: v.clone() for k, v in out.items()} | {"ids": ids, "margin": mar, "prob": prob})
        steps += 1
    return dict(steps=steps, flips=flips, flip_denominator=denom, window_flips=wflips, window_denominator=wdenom,
                committed=committed, flip_trace=flip_trace, per_step=per_step)

"""Seeded synthetic inputs for the LSP per-step hot path.

This module only *draws data*: random tensors with the shapes, value
distributions and planted structure of the workloads the method runs on.  It
holds none of the method's arithmetic (no arg-max, margin, soft-max, boundary
search or cache append) and is imported neither by the CPU oracle nor by the
HIP library; tests and the benchmark call it once and hand the same tensors to
both sides.

Shapes follow the two public model families the paper evaluates (Section 4.1):
an LLaDA-8B-like decoder (32 layers, 32 heads of 128, vocab 126464) and a
Dream-7B-like decoder (28 query heads / 4 KV heads of 128, vocab 152064).
Hyper-parameters default to the paper's (Section 4.1: L_min = 1, W = 16).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16": storage type of Q/K/V/logits
    B: int                # sequences
    layers: int
    Hq: int
    Hkv: int
    D: int
    P: int                # committed-prefix rows already in the cache
    S: int                # active-suffix rows (suffix buffer height)
    C: int                # cache capacity (positions)
    V: int                # vocabulary
    tau: float            # margin threshold (logit units)
    n_delim: int
    delim_frac: float     # fraction of positions whose planted id is a delimiter
    boost: float = 0.0    # planted-argmax boost amplitude A
    decay: float = 1.0    # boost decays as A * exp(-i / decay)
    window: int = 16      # snap look-back W
    min_commit: int = 1   # L_min
    seed: int = 1000
    plant: str = "decay"  # "decay" | "stable_len" | "process"
    gen_len: int = 0      # loop workloads: positions to generate (= S at step 0)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


# The five configurations the benchmark contract names, plus reduced copies the
# CPU oracle can finish in seconds (same structure, fewer/lower dimensions).
C1 = Workload("c1_tiny_f32", "f32", 1, 1, 4, 4, 64, 128, 64, 256, 1024, 0.9, 16, 0.10,
              boost=8.0, decay=16.0, seed=1001)
C2 = Workload("c2_llada8b_layer", "bf16", 1, 1, 32, 32, 128, 512, 256, 2048, 126464, 0.9, 64, 0.08,
              boost=16.0, decay=128.0, seed=1002)
C3 = Workload("c3_dream7b_gqa", "bf16", 4, 1, 28, 4, 128, 1024, 512, 2048, 152064, 0.85, 64, 0.08,
              boost=12.0, seed=1003, plant="stable_len")
C4 = Workload("c4_llada8b_long", "bf16", 8, 32, 32, 32, 128, 4096, 1024, 8192, 126464, 0.9, 64, 0.08,
              boost=12.0, decay=256.0, seed=1004)
C5 = Workload("c5_llada8b_loop", "bf16", 16, 32, 32, 32, 128, 512, 1024, 1536, 126464, 0.9, 64, 0.08,
              seed=1005, plant="process", gen_len=1024)

CONFIGS = {w.name: w for w in (C1, C2, C3, C4, C5)}


def scaled(w: Workload, **kw) -> Workload:
    """A reduced copy of a workload (tests): same structure, overridden sizes."""
    return replace(w, **kw)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def _randn(shape, g, device, dtype):
    """N(0,1) drawn in fp32 then rounded once to the storage type."""
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


# --------------------------------------------------------------------------- #
# attention operands
# --------------------------------------------------------------------------- #
POISON_F32 = -768.0      # exactly representable in bf16 as well


def make_layer_kv(w: Workload, layer: int, device="cpu", prefix_len=None):
    """One layer's attention operands.

    Returns dict(q, k_suf, v_suf: [B,S,H,D]; k_cache, v_cache: [B,C,Hkv,D]).
    Cache rows at and beyond each sequence's prefix length hold a poison value
    so that a test can tell an untouched row from a written one.
    """
    g = _gen(w.seed * 1000 + 17 * layer + 1, device)
    dt = w.torch_dtype
    out = {
        "q": _randn((w.B, w.S, w.Hq, w.D), g, device, dt),
        "k_suf": _randn((w.B, w.S, w.Hkv, w.D), g, device, dt),
        "v_suf": _randn((w.B, w.S, w.Hkv, w.D), g, device, dt),
    }
    for name in ("k_cache", "v_cache"):
        c = torch.full((w.B, w.C, w.Hkv, w.D), POISON_F32, device=device, dtype=dt)
        if prefix_len is None:
            c[:, : w.P] = _randn((w.B, w.P, w.Hkv, w.D), g, device, dt)
        else:
            pmax = int(max(prefix_len))
            fresh = _randn((w.B, pmax, w.Hkv, w.D), g, device, dt)
            for b in range(w.B):
                c[b, : int(prefix_len[b])] = fresh[b, : int(prefix_len[b])]
        out[name] = c
    return out


def make_lengths(w: Workload, device="cpu", ragged=False):
    """prefix_len[B], suffix_len[B] (int32).  ragged=True draws per-sequence
    lengths (with one empty suffix when B > 2) the way a decode loop leaves
    them after a few commits."""
    if not ragged:
        p = torch.full((w.B,), w.P, dtype=torch.int32)
        n = torch.full((w.B,), w.S, dtype=torch.int32)
    else:
        g = _gen(w.seed + 77, "cpu")
        n = torch.randint(1, w.S + 1, (w.B,), generator=g, dtype=torch.int32)
        p = torch.randint(0, w.P + 1, (w.B,), generator=g, dtype=torch.int32)
        if w.B > 2:
            n[1] = 0
        if w.B > 1:
            p[0] = 0
    return p.to(device), n.to(device)


# --------------------------------------------------------------------------- #
# delimiters, tokens
# --------------------------------------------------------------------------- #
def make_delimiters(w: Workload):
    """Seeded delimiter id set D (sorted int64 tensor) and its bitmap over the
    vocabulary (uint32 words held in an int32 tensor, bit v%32 of word v//32)."""
    g = _gen(w.seed + 5, "cpu")
    ids = torch.randperm(w.V, generator=g)[: w.n_delim].sort().values
    words = torch.zeros((w.V + 31) // 32, dtype=torch.int64)
    for v in ids.tolist():
        words[v // 32] |= 1 << (v % 32)
    words = torch.where(words >= 2**31, words - 2**32, words).to(torch.int32)
    return ids, words


def make_tokens(w: Workload, T: int, mask_id: int = -1):
    """[B,T] int32 token buffer: seeded prompt ids in [0,P), mask_id after."""
    g = _gen(w.seed + 9, "cpu")
    t = torch.full((w.B, T), mask_id, dtype=torch.int32)
    t[:, : w.P] = torch.randint(0, w.V, (w.B, w.P), generator=g, dtype=torch.int32)
    return t


# --------------------------------------------------------------------------- #
# logits
# --------------------------------------------------------------------------- #
def _planted_ids(w: Workload, delim_ids, shape, g, device):
    """Per position: a delimiter id with probability delim_frac, otherwise a
    seeded id outside the delimiter set."""
    is_d = torch.rand(shape, generator=g, device=device) < w.delim_frac
    pick = torch.randint(0, len(delim_ids), shape, generator=g, device=device)
    d = delim_ids.to(device)[pick]
    other = torch.randint(0, w.V, shape, generator=g, device=device)
    # push an accidental delimiter hit to a neighbouring id that is not one
    dset = torch.zeros(w.V + 1, dtype=torch.bool, device=device)
    dset[delim_ids.to(device)] = True
    for _ in range(4):
        other = torch.where(dset[other], (other + 1) % w.V, other)
    return torch.where(is_d, d, other)


def make_logits(w: Workload, device="cpu", step: int = 0, prefix_len=None, stable_len=None):
    """Logits [B,S,V] in the workload's storage type, plus what was planted.

    plant == "decay":      N(0,1) background; entry t_i of row i gets
                           + boost * exp(-i / decay) before rounding.
    plant == "stable_len": per sequence a seeded length l_b in [0,S]; rows
                           i < l_b get +boost at t_i; row l_b gets two equal
                           entries of 6.0 (margin 0); rows beyond are boosted
                           with probability 1/2.
    plant == "process":    see make_process_logits.
    Returns (logits, info) with info = dict(planted_id [B,S], stable_len [B] or None).
    """
    if w.plant == "process":
        return make_process_logits(w, device, step, prefix_len)
    g = _gen(w.seed + 31 + 7919 * step, device)
    delim_ids, _ = make_delimiters(w)
    z = torch.randn((w.B, w.S, w.V), generator=g, device=device, dtype=torch.float32)
    tid = _planted_ids(w, delim_ids, (w.B, w.S), g, device)
    pos = torch.arange(w.S, device=device, dtype=torch.float32)
    info = {"planted_id": tid, "stable_len": None}
    if w.plant == "decay":
        add = (w.boost * torch.exp(-pos / w.decay)).expand(w.B, w.S)
    else:
        if stable_len is None:
            gl = _gen(w.seed + 41, "cpu")
            stable_len = torch.randint(0, w.S + 1, (w.B,), generator=gl)
        sl = stable_len.to(device).view(w.B, 1)
        coin = torch.rand((w.B, w.S), generator=g, device=device) < 0.5
        i = pos.view(1, w.S)
        on = (i < sl) | ((i > sl) & coin)
        add = torch.where(on, torch.full_like(i, w.boost).expand(w.B, w.S), torch.zeros((), device=device))
        info["stable_len"] = stable_len.clone()
    z.scatter_add_(2, tid.unsqueeze(-1), add.unsqueeze(-1).contiguous())
    if w.plant == "stable_len":
        for b in range(w.B):
            lb = int(stable_len[b])
            if lb < w.S:
                a = int(tid[b, lb])
                z[b, lb, a] = 6.0
                z[b, lb, (a + 1) % w.V] = 6.0
    return z.to(w.torch_dtype), info


def make_lm_head(w: Workload, K: int, device="cpu", step: int = 0):
    """Operands of the output head for the workload's rows: weight [V,K] ~
    N(0, 1/K) and hidden [B,S,K] ~ N(0,1), both rounded to the storage type, so
    that the logits hidden @ weight.T are ~ N(0,1) like make_logits' background.
    Row i additionally gets boost * exp(-i/decay) (plant "decay") or boost (any
    other plant) times weight[t_i] / |weight[t_i]|^2 added to its hidden state,
    which lifts the logit of the planted id t_i by that amount.
    Returns (hidden, weight, info) with info = dict(planted_id [B,S])."""
    g = _gen(w.seed + 57 + 7919 * step, device)
    delim_ids, _ = make_delimiters(w)
    weight = (torch.randn((w.V, K), generator=g, device=device, dtype=torch.float32) / math.sqrt(K)).to(w.torch_dtype)
    hidden = torch.randn((w.B, w.S, K), generator=g, device=device, dtype=torch.float32)
    tid = _planted_ids(w, delim_ids, (w.B, w.S), g, device)
    pos = torch.arange(w.S, device=device, dtype=torch.float32)
    amp = w.boost * torch.exp(-pos / w.decay) if w.plant == "decay" else torch.full_like(pos, w.boost)
    wt = weight[tid.reshape(-1)].float().view(w.B, w.S, K)
    hidden += amp.view(1, w.S, 1) * wt / (wt * wt).sum(-1, keepdim=True)
    return hidden.to(w.torch_dtype), weight, {"planted_id": tid}


def make_process_logits(w: Workload, device, step: int, prefix_len):
    """Config-5 style synthetic denoising process.

    Row u of sequence b stands for absolute generation position
    j = prefix_len[b] - P + u (u-th still-active position).  Its confidence is
        c = 1 - exp(-(step+1) / (1 + u/64)) + N(0, 0.5^2)
    The background is N(0,1) clipped to <= 4 with one seeded runner-up entry
    set to exactly 4, so the row's background maximum is 4 by construction;
    the planted entry is 4 + |c|.  The planted id is the position's fixed
    target token when c > 0 and a fixed alternative otherwise (this is what
    produces top-1 flips between steps).  Rows at or beyond the sequence's
    remaining length are left as plain background.
    Returns (logits [B,S,V], info(planted_id, conf, target, alt)).
    """
    assert prefix_len is not None
    G = w.gen_len or w.S
    g = _gen(w.seed + 31 + 7919 * step, device)
    gfix = _gen(w.seed + 43, "cpu")
    delim_ids, _ = make_delimiters(w)
    # fixed per absolute position: target / alternative / runner-up ids
    target = _planted_ids(w, delim_ids, (w.B, G), gfix, "cpu")
    alt = (target + 1 + torch.randint(0, w.V - 2, (w.B, G), generator=gfix)) % w.V
    runner = (target + 1 + torch.randint(0, w.V - 2, (w.B, G), generator=gfix)) % w.V
    runner = torch.where(runner == alt, (runner + 1) % w.V, runner)
    runner = torch.where(runner == target, (runner + 1) % w.V, runner)
    done = (prefix_len.to("cpu").to(torch.int64) - w.P).clamp(0, G)          # committed so far
    u = torch.arange(w.S).view(1, w.S)
    j = (done.view(w.B, 1) + u).clamp(max=G - 1)                              # absolute position
    active = (done.view(w.B, 1) + u) < G
    tgt_u, alt_u, run_u = (t.gather(1, j).to(device) for t in (target, alt, runner))
    z = torch.randn((w.B, w.S, w.V), generator=g, device=device, dtype=torch.float32).clamp_(max=4.0)
    noise = 0.5 * torch.randn((w.B, w.S), generator=g, device=device, dtype=torch.float32)
    uu = u.to(device=device, dtype=torch.float32)
    conf = 1.0 - torch.exp(-(step + 1.0) / (1.0 + uu / 64.0)) + noise
    tid = torch.where(conf > 0, tgt_u, alt_u)
    z.scatter_(2, run_u.unsqueeze(-1), torch.full((w.B, w.S, 1), 4.0, device=device))
    top = (4.0 + conf.abs()).unsqueeze(-1)
    act = active.to(device)
    cur = z.gather(2, tid.unsqueeze(-1))
    z.scatter_(2, tid.unsqueeze(-1), torch.where(act.unsqueeze(-1), top, cur))
    return z.to(w.torch_dtype), {"planted_id": tid, "conf": conf, "target": target, "alt": alt, "active": act}


def attn_flops(w: Workload, prefix_len=None, suffix_len=None) -> float:
    """4 * sum_b Hq * N_b * (P_b + N_b) * D (QK^T and PV, multiply-add = 2)."""
    if prefix_len is None:
        return 4.0 * w.B * w.Hq * w.S * (w.P + w.S) * w.D
    tot = 0.0
    for p, n in zip(prefix_len.tolist(), suffix_len.tolist()):
        tot += 4.0 * w.Hq * n * (p + n) * w.D
    return tot


def elem_bytes(w: Workload) -> int:
    return 4 if w.dtype == "f32" else 2

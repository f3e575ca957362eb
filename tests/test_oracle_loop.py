"""Pins for the loop oracle (Algorithm 1 lines 3-11): closed-form step counts
(Table 2's one-token row, the Full baseline's T_max = generation length of
Section 4.1), single-step completion, conservation, restart equivalence."""
import os

import pytest
import torch

import workloads as W
from oracle.loop import decode_loop

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as f:
    for line in f:
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            GOLD[k] = float(v)


def _setup(G, B=2, V=512, P=4):
    w = W.scaled(W.C5, B=B, S=G, V=V, P=P, gen_len=G, C=P + G, layers=1, Hq=2, Hkv=2, D=8)
    _, bm = W.make_delimiters(w)
    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, P + G)
    fn = lambda step, p: W.make_logits(w, step=step, prefix_len=p)[0]
    return w, bm, pl, sl, tokens, fn


def test_tau_inf_takes_one_token_per_step_table2(oracle):
    """tau = +inf: nothing is ever stable, L_min = 1 commits one token per step, so a
    budget of G tokens takes G steps: Table 2's 'Fixed Prefix (1 tokens)' row."""
    G = int(GOLD["fixed_prefix_steps_k1"])
    w, bm, pl, sl, tokens, fn = _setup(G)
    r = decode_loop(fn, bm, w.V, float("inf"), int(GOLD["W"]), int(GOLD["L_min"]), 1, pl, sl, tokens)
    assert r["steps"] == G == 128 and r["committed"] == 2 * G
    assert torch.all(sl == 0) and torch.all(pl == w.P + G)


@pytest.mark.parametrize("k", [2, 4, 8])
def test_fixed_prefix_k_tokens_table2(oracle, k):
    """L_min = k with tau = +inf commits exactly k per step: ceil(G/k) steps."""
    G = 128
    w, bm, pl, sl, tokens, fn = _setup(G)
    r = decode_loop(fn, bm, w.V, float("inf"), 16, k, 1, pl, sl, tokens)
    assert r["steps"] == int(GOLD[f"fixed_prefix_steps_k{k}"])


def test_tau_minus_inf_no_snap_single_step(oracle):
    w, bm, pl, sl, tokens, fn = _setup(40)
    r = decode_loop(fn, bm, w.V, -float("inf"), 16, 1, 0, pl, sl, tokens)
    assert r["steps"] == 1 and r["committed"] == 80 and r["flips"] == 0


def test_conservation_monotone_prefix_and_tokens(oracle):
    G = 96
    w, bm, pl, sl, tokens, fn = _setup(G, B=3)
    r = decode_loop(fn, bm, w.V, w.tau, w.window, 1, 1, pl, sl, tokens, trace=True)
    tot = sum(s["commit_len"] for s in r["per_step"])
    assert tot.tolist() == [G] * 3
    assert 1 < r["steps"] < G                       # the process does commit multi-token blocks
    assert r["flips"] > 0 and r["flip_denominator"] >= r["flips"]
    # every step commits at least one token per unfinished sequence (monotone progress)
    left = torch.full((3,), G)
    for s in r["per_step"]:
        assert torch.all((s["commit_len"] >= 1) | (left == 0))
        assert torch.all(s["snapped_boundary"] <= s["raw_boundary"])
        left = left - s["commit_len"]
    # the token buffer holds, position by position, the id that was top-1 when it was committed
    pos = torch.full((3,), w.P)
    for s in r["per_step"]:
        for b in range(3):
            L = int(s["commit_len"][b])
            assert tokens[b, pos[b]:pos[b] + L].tolist() == s["ids"][b, :L].tolist()
            pos[b] += L
    assert torch.all(tokens[:, w.P:] >= 0)


def test_restart_from_snapshot(oracle):
    G = 64
    w, bm, pl, sl, tokens, fn = _setup(G)
    full = decode_loop(fn, bm, w.V, w.tau, w.window, 1, 1, pl, sl, tokens, trace=True)
    # replay 3 steps by hand, snapshot, continue with a loop whose step index is offset
    w, bm, pl2, sl2, tok2, fn = _setup(G)
    for k in range(3):
        ids, p, m = oracle.confidence(fn(k, pl2), sl2)
        oracle.commit(m, ids, bm, w.V, w.tau, w.window, 1, 1, pl2, sl2, tokens=tok2, C=w.P + G)
    rest = decode_loop(lambda s, p: fn(s + 3, p), bm, w.V, w.tau, w.window, 1, 1, pl2, sl2, tok2)
    assert rest["steps"] + 3 == full["steps"]
    assert torch.equal(tok2, tokens)


def test_loop_on_hidden_states_equals_loop_on_their_logits(oracle):
    """lm_head_weight mode: with operands whose logits are exact in fp32 the loop
    fed hidden states must walk exactly like the loop fed the logits themselves."""
    import workloads as W
    from oracle.loop import decode_loop
    G, K = 40, 16
    w = W.scaled(W.C5, B=2, S=G, V=300, P=4, gen_len=G, C=4 + G, layers=1, Hq=2, Hkv=2, D=64)
    _, bm = W.make_delimiters(w)
    weight = torch.randint(-3, 4, (w.V, K), generator=torch.Generator().manual_seed(1)).float()

    def hidden_fn(step, p):
        return torch.randint(-3, 4, (w.B, w.S, K), generator=torch.Generator().manual_seed(50 + step)).float()

    runs = []
    for mode in ("hidden", "logits"):
        pl, sl = W.make_lengths(w)
        tokens = W.make_tokens(w, w.C)
        if mode == "hidden":
            r = decode_loop(hidden_fn, bm, w.V, 0.5, w.window, 1, 1, pl, sl, tokens, lm_head_weight=weight)
        else:
            r = decode_loop(lambda s, p: hidden_fn(s, p) @ weight.T, bm, w.V, 0.5, w.window, 1, 1, pl, sl, tokens)
        runs.append((r["steps"], r["flips"], r["flip_denominator"], r["committed"], tokens.clone(), pl.clone()))
    assert runs[0][:4] == runs[1][:4] and runs[0][0] > 2
    assert torch.equal(runs[0][4], runs[1][4]) and torch.equal(runs[0][5], runs[1][5])

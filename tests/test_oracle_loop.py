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


# --------------------------------------------------------------------------- #
# The flip statistic of Section 4.3.4, pinned by a trace counted by hand
# --------------------------------------------------------------------------- #
def _scripted_logits(script, S, V=16):
    """logits_fn for a hand-written trace.  script[step][b] lists, for the rows
    u = 0.. of sequence b (its still-active positions, in order), pairs
    (top-1 id, stable?).  A stable row gets margin 10, an unstable one 0.25
    (tau is 1).  Rows beyond the listed ones are filled with id 15 at margin 10:
    if the loop ever looked at an inactive row, counts and commits would change."""
    def fn(step, prefix_len):
        B = len(script[step])
        z = torch.zeros((B, S, V))
        z[:, :, 15] = 10.0
        for b, rows in enumerate(script[step]):
            for u, (tid, stable) in enumerate(rows):
                z[b, u] = 0.0
                z[b, u, tid] = 10.0 if stable else 0.25
        return z
    return fn


def test_flip_counts_of_a_hand_worked_trace(oracle):
    """Two sequences, five generation positions each, tau = 1, no snapping, L_min = 1.
    Absolute generation positions are written p0..p4.

    Sequence 0                                   top-1 ids          committed    compared  flips
      step 0: active p0..p4 (first prediction)   3 4 5 6 7          p0 (1 stable)    0       0
      step 1: active p1..p4, before: 4 5 6 7     4 1 6 2            p1 p2 (2 stable) 4       2  (p2 5->1, p4 7->2)
      step 2: active p3 p4,  before: 6 2         6 7                p3 (L_min)       2       1  (p4 2->7)
      step 3: active p4,     before: 7           7                  p4               1       0
    Sequence 1
      step 0: active p0..p4                      1 1 1 1 1          p0 p1 p2         0       0
      step 1: active p3 p4,  before: 1 1         2 1                p3 p4            2       1  (p3 1->2)
      steps 2, 3: nothing active                                                     0       0
    Totals: 4 steps, compared 4+2+1+2 = 9, flips 2+1+0+1 = 4.

    A comparison that forgets the positions already committed (row u against the
    previous step's row u instead of position done+u) would see, for sequence 0,
    step 1: 4 1 6 2 against 3 4 5 6 = 4 flips, and so a different total.

    Window [2, 3] committed positions (40 %-60 % of five): sequence 0 is inside at step 2
    (3 committed) only; at step 1 it has 1, at step 3 it has 4.  Sequence 1 is inside at
    step 1 (3 committed).  Window: compared 2 + 2 = 4, flips 1 + 1 = 2."""
    S = 5
    script = [
        [[(3, True), (4, False), (5, True), (6, True), (7, True)], [(1, True), (1, True), (1, True), (1, False), (1, False)]],
        [[(4, True), (1, True), (6, False), (2, True)], [(2, True), (1, True)]],
        [[(6, False), (7, True)], []],
        [[(7, True)], []],
    ]
    bm = torch.zeros(1, dtype=torch.int32)
    pl = torch.tensor([2, 0], dtype=torch.int32)          # different prompt lengths: positions are relative to them
    sl = torch.tensor([S, S], dtype=torch.int32)
    tokens = torch.full((2, 2 + S), -1, dtype=torch.int32)
    r = decode_loop(_scripted_logits(script, S), bm, 16, 1.0, 16, 1, 0, pl, sl, tokens, trace=True,
                    window_lo=2, window_hi=3)
    assert [s["commit_len"].tolist() for s in r["per_step"]] == [[1, 3], [2, 2], [1, 0], [1, 0]]
    assert r["steps"] == 4 and r["committed"] == 10
    assert (r["flips"], r["flip_denominator"]) == (4, 9)
    assert (r["window_flips"], r["window_denominator"]) == (2, 4)
    assert [(f.tolist(), d.tolist()) for f, d in r["flip_trace"]] == [
        ([0, 0], [0, 0]), ([2, 1], [4, 2]), ([1, 0], [2, 0]), ([0, 0], [1, 0])]
    assert tokens[0, 2:].tolist() == [3, 4, 1, 6, 7] and tokens[1, :S].tolist() == [1, 1, 1, 2, 1]


def test_flip_counts_do_not_depend_on_how_much_is_committed_elsewhere(oracle):
    """The same id history at the same absolute positions gives the same flips whether the
    positions in front of them were committed one at a time or all at once (an indexing
    mistake by the committed count would not survive this)."""
    S, V = 6, 16
    hist = {0: [1, 2, 3, 4, 5, 6], 1: [1, 2, 3, 9, 5, 8], 2: [1, 2, 3, 9, 7, 8]}   # ids of p0..p5 at steps 0, 1, 2

    def run(stable_len_by_step):
        def fn(step, prefix_len):
            done = int(prefix_len[0])
            z = torch.zeros((1, S, V))
            for u in range(S - done):
                tid = hist[min(step, 2)][done + u]
                z[0, u, tid] = 10.0 if u < stable_len_by_step[min(step, len(stable_len_by_step) - 1)] else 0.25
            return z
        pl, sl = torch.zeros(1, dtype=torch.int32), torch.full((1,), S, dtype=torch.int32)
        tok = torch.full((1, S), -1, dtype=torch.int32)
        return decode_loop(fn, torch.zeros(1, dtype=torch.int32), V, 1.0, 16, 1, 0, pl, sl, tok, trace=True)

    a = run([1, 1, 4])     # commits p0, then p1, then the rest: step 1 compares p1..p5, step 2 compares p2..p5
    b = run([3, 0, 3])     # commits p0..p2 at once, then p3 (L_min), then the rest: step 1 compares p3..p5, step 2 p4, p5
    # step 0 -> 1 changes p3 (4->9) and p5 (6->8); step 1 -> 2 changes p4 (5->7)
    assert [f.tolist() for f, _ in a["flip_trace"]] == [[0], [2], [1]]
    assert [d.tolist() for _, d in a["flip_trace"]] == [[0], [5], [4]]
    assert [f.tolist() for f, _ in b["flip_trace"]] == [[0], [2], [1]]
    assert [d.tolist() for _, d in b["flip_trace"]] == [[0], [3], [2]]

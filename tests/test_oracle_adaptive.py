"""Pins for the adaptive threshold of the commit oracle (Section 3.2 "targeted
block sizing", Eq. 2; Algorithm 1 line 6) and for the commit cap (the
fixed-prefix rows of Table 2): exhaustive enumeration of thresholds on small
inputs, closed forms, and loop-level step counts."""
import itertools
import math
import os

import pytest
import torch

import workloads as W
from oracle.loop import decode_loop

V = 64
OTHER = 9
NO_DELIM = torch.zeros(2, dtype=torch.int32)
GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")) as f:
    for line in f:
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            GOLD[k] = float(v)


def _run_len(mg, t):
    """L'(t) from the text: longest run from the left whose margins all exceed t."""
    n = 0
    while n < len(mg) and mg[n] > t:
        n += 1
    return n


def _by_threshold_enumeration(mg, tau0, alpha, beta):
    """Eq. 2 solved by trying every threshold that can change L': each margin value
    and -inf (between two neighbouring values L' is constant).  Returns the chosen
    length and whether any threshold puts L' inside the interval."""
    N = len(mg)
    lo = min(N, max(0, math.ceil(alpha * N)))
    hi = max(lo, min(N, math.floor(beta * N)))
    L0 = _run_len(mg, tau0)
    if lo <= L0 <= hi:
        return L0, True, lo, hi
    reach = {_run_len(mg, t) for t in list(mg) + [-math.inf]}
    inside = sorted(a for a in reach if lo <= a <= hi)
    if not inside:
        return (lo if L0 < lo else hi), False, lo, hi
    return (inside[0] if L0 < lo else inside[-1]), True, lo, hi


@pytest.mark.parametrize("alpha,beta", [(0.25, 0.5), (0.5, 0.5), (0.2, 1.0), (0.75, 0.75)])
def test_every_small_margin_vector_against_threshold_enumeration(oracle, alpha, beta):
    N = 5
    vals = [1.0, 2.0, 3.0, 4.0]
    cases = [(list(mg), tau0) for mg in itertools.product(vals, repeat=N) for tau0 in (0.5, 2.0, 2.5, 4.0)]
    B = len(cases)
    margin = torch.tensor([c[0] for c in cases], dtype=torch.float32)
    ids = torch.full((B, N), OTHER, dtype=torch.int32)
    # one tau per call: group by tau0
    for tau0 in (0.5, 2.0, 2.5, 4.0):
        sel = [i for i, c in enumerate(cases) if c[1] == tau0]
        m = margin[sel].contiguous()
        pl = torch.zeros(len(sel), dtype=torch.int32)
        sl = torch.full((len(sel),), N, dtype=torch.int32)
        out = oracle.commit(m, ids[sel].contiguous(), NO_DELIM, V, tau0, 16, 0, 0, pl, sl, C=64,
                            adaptive=True, alpha=alpha, beta=beta)
        for k, i in enumerate(sel):
            mg = cases[i][0]
            want, ok, lo, hi = _by_threshold_enumeration(mg, tau0, alpha, beta)
            got = int(out["raw_boundary"][k])
            assert got == want, (mg, tau0, got, want)
            assert lo <= got <= hi                                   # Eq. 2
            tk = float(out["tau_used"][k])
            if ok:
                assert not math.isnan(tk) and _run_len(mg, tk) == got   # the reported threshold gives that length
                assert not (int(out["status_flags"][k]) & 4)
            else:
                assert math.isnan(tk) and (int(out["status_flags"][k]) & 4)
            # the mask output stays relative to the caller's threshold
            assert out["stable_mask"][k].tolist() == [int(x > tau0) for x in mg]


def test_closed_forms(oracle):
    N = 16
    ids = torch.full((1, N), OTHER, dtype=torch.int32)
    st = lambda: (torch.zeros(1, dtype=torch.int32), torch.full((1,), N, dtype=torch.int32))
    dec = torch.arange(N, 0, -1, dtype=torch.float32).view(1, N)       # strictly decreasing: every length reachable
    o = oracle.commit(dec, ids, NO_DELIM, V, float("inf"), 16, 0, 0, *st(), C=64, adaptive=True, alpha=0.25, beta=0.5)
    assert int(o["raw_boundary"]) == 4 and float(o["tau_used"]) == float(dec[0, 4])     # ceil(alpha N), lowered just enough
    o = oracle.commit(dec, ids, NO_DELIM, V, -float("inf"), 16, 0, 0, *st(), C=64, adaptive=True, alpha=0.25, beta=0.5)
    assert int(o["raw_boundary"]) == 8 and float(o["tau_used"]) == float(dec[0, 8])     # floor(beta N), raised just enough
    o = oracle.commit(dec, ids, NO_DELIM, V, 10.5, 16, 0, 0, *st(), C=64, adaptive=True, alpha=0.25, beta=0.5)
    assert int(o["raw_boundary"]) == 6 and float(o["tau_used"]) == 10.5                 # already inside: untouched
    const = torch.full((1, N), 3.0)                                    # only lengths 0 and N are reachable
    o = oracle.commit(const, ids, NO_DELIM, V, 1.0, 16, 0, 0, *st(), C=64, adaptive=True, alpha=0.25, beta=0.5)
    assert int(o["raw_boundary"]) == 8 and int(o["status_flags"]) & 4 and math.isnan(float(o["tau_used"]))
    o = oracle.commit(const, ids, NO_DELIM, V, 3.0, 16, 0, 0, *st(), C=64, adaptive=True, alpha=0.25, beta=0.5)
    assert int(o["raw_boundary"]) == 4 and int(o["status_flags"]) & 4
    o = oracle.commit(const, ids, NO_DELIM, V, 3.0, 16, 0, 0, *st(), C=64, adaptive=True, alpha=1.0, beta=1.0)
    assert int(o["raw_boundary"]) == N and float(o["tau_used"]) == -float("inf") and not int(o["status_flags"]) & 4
    # adaptive off: the same inputs give the plain fixed-threshold answer
    o = oracle.commit(dec, ids, NO_DELIM, V, 10.5, 16, 0, 0, *st(), C=64)
    assert int(o["raw_boundary"]) == 6 and float(o["tau_used"]) == 10.5


def test_commit_cap(oracle):
    N = 12
    margin = torch.full((1, N), 5.0)
    ids = torch.full((1, N), OTHER, dtype=torch.int32)
    for cap, want in [(0, 12), (5, 5), (12, 12), (40, 12)]:
        pl, sl = torch.zeros(1, dtype=torch.int32), torch.full((1,), N, dtype=torch.int32)
        o = oracle.commit(margin, ids, NO_DELIM, V, 1.0, 16, 1, 0, pl, sl, C=64, max_commit=cap)
        assert int(o["commit_len"]) == want and int(o["raw_boundary"]) == 12 and int(pl) == want


def _loop(G, fn, tau, Lmin, **kw):
    w = W.scaled(W.C5, B=2, S=G, V=32, P=4, gen_len=G, C=4 + G, layers=1, Hq=2, Hkv=2, D=8)
    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, 4 + G)
    return decode_loop(fn, NO_DELIM[:1], 32, tau, 16, Lmin, 0, pl, sl, tokens, trace=True, commit_kw=kw)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_fixed_prefix_of_k_tokens_via_the_cap_table2(oracle, k):
    """Everything stable (tau = -inf) and a cap of k tokens commits exactly k per
    step: the 'Fixed Prefix (k tokens)' rows of Table 2, 128 / 64 / 32 / 16 steps."""
    G = 128
    fn = lambda step, p: torch.randn((2, G, 32), generator=torch.Generator().manual_seed(step))
    r = _loop(G, fn, -float("inf"), 1, max_commit=k)
    assert r["steps"] == int(GOLD[f"fixed_prefix_steps_k{k}"]) == G // k


def test_geometric_decay_with_alpha_equal_beta(oracle):
    """alpha = beta = 1/4 on margins that fall strictly along the suffix: every
    length is reachable, so each step commits exactly ceil(N/4) and the suffix
    shrinks geometrically (Section 3.2): 128 -> 96 -> 72 -> 54 -> 40 -> ... -> 0."""
    G = 128

    def fn(step, p):
        z = torch.zeros((2, G, 32))
        z[:, :, 3] = 10.0 - 0.01 * torch.arange(G).view(1, G)          # margin of row u = 10 - 0.01 u
        return z

    r = _loop(G, fn, float("inf"), 0, adaptive=True, alpha=0.25, beta=0.25)
    lens = [int(s["commit_len"][0]) for s in r["per_step"]]
    assert lens == [32, 24, 18, 14, 10, 8, 6, 4, 3, 3, 2, 1, 1, 1, 1]
    n = G
    for k, L in enumerate(lens):
        assert L == math.ceil(n / 4)
        n -= L
        assert n <= G * 0.75 ** (k + 1)
    assert r["steps"] == 15

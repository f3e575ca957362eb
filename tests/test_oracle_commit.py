"""Pins for the commit oracle (Section 3.2: L'(tau), the snap equation, the
fallback; Algorithm 1 lines 7-10): brute force over every mask and delimiter
placement against the set-form definition, invariants, closed forms, append."""
import itertools

import pytest
import torch

import workloads as W

V = 64
DELIM = 5          # the one delimiter id used by the enumeration
OTHER = 9


def _bitmap(ids, V=V):
    words = torch.zeros((V + 31) // 32, dtype=torch.int64)
    for v in ids:
        words[v // 32] |= 1 << (v % 32)
    return torch.where(words >= 2**31, words - 2**32, words).to(torch.int32)


def _definition(mask, is_d, N, Wn, Lmin, snap=True):
    """Set form, written from the text: L' = length of the longest all-stable
    run from the left; candidates = {j in 1..L' : token j is a delimiter and
    L'-j <= W}; snapped = max(candidates) or L' when empty; L = max(L_min, snapped)
    limited by the N positions that exist."""
    Lp = 0
    while Lp < N and mask[Lp]:
        Lp += 1
    cand = {j for j in range(1, Lp + 1) if is_d[j - 1] and (Wn < 0 or Lp - j <= Wn)}
    Ls = max(cand) if (cand and snap) else Lp
    return Lp, Ls, min(N, max(Lmin, Ls))


@pytest.mark.parametrize("Wn", [0, 1, 3, -1])
@pytest.mark.parametrize("Lmin", [0, 1, 2])
def test_brute_force_all_masks_and_delimiters(oracle, Wn, Lmin):
    N = 6
    cases = list(itertools.product(itertools.product([0, 1], repeat=N), itertools.product([0, 1], repeat=N)))
    B = len(cases)
    margin = torch.tensor([[2.0 if m else 0.5 for m in mk] for mk, _ in cases], dtype=torch.float32)
    ids = torch.tensor([[DELIM if d else OTHER for d in dl] for _, dl in cases], dtype=torch.int32)
    pl = torch.zeros(B, dtype=torch.int32)
    sl = torch.full((B,), N, dtype=torch.int32)
    out = oracle.commit(margin, ids, _bitmap([DELIM]), V, 1.0, Wn, Lmin, 1, pl, sl, C=64)
    for b, (mk, dl) in enumerate(cases):
        Lp, Ls, L = _definition(mk, dl, N, Wn, Lmin)
        assert (out["raw_boundary"][b], out["snapped_boundary"][b], out["commit_len"][b]) == (Lp, Ls, L), (mk, dl)
        assert out["stable_mask"][b].tolist() == list(mk)
        assert pl[b] == L and sl[b] == N - L
        # invariants: snapped <= raw; snapped ends on a delimiter or equals raw
        assert Ls <= Lp and (Ls == Lp or dl[Ls - 1])


def test_ragged_suffix_lengths_and_snap_off(oracle):
    N = 5
    cases = list(itertools.product(itertools.product([0, 1], repeat=N), itertools.product([0, 1], repeat=N)))
    B = len(cases)
    Ns = [(b % (N + 1)) for b in range(B)]            # includes empty suffixes
    margin = torch.tensor([[2.0 if m else 0.5 for m in mk] for mk, _ in cases], dtype=torch.float32)
    ids = torch.tensor([[DELIM if d else OTHER for d in dl] for _, dl in cases], dtype=torch.int32)
    for snap in (0, 1):
        pl = torch.full((B,), 3, dtype=torch.int32)
        sl = torch.tensor(Ns, dtype=torch.int32)
        out = oracle.commit(margin, ids, _bitmap([DELIM]), V, 1.0, 2, 1, snap, pl, sl, C=64)
        for b, (mk, dl) in enumerate(cases):
            Lp, Ls, L = _definition(mk, dl, Ns[b], 2, 1, snap=bool(snap))
            assert (out["raw_boundary"][b], out["snapped_boundary"][b], out["commit_len"][b]) == (Lp, Ls, L)
            assert out["stable_mask"][b].tolist() == [int(m and i < Ns[b]) for i, m in enumerate(mk)]
            assert pl[b] == 3 + L and sl[b] == Ns[b] - L


def test_threshold_is_strict_and_closed_forms(oracle):
    margin = torch.tensor([[1.0, 1.0, 1.0, 1.0]], dtype=torch.float32)
    ids = torch.full((1, 4), OTHER, dtype=torch.int32)
    bm = _bitmap([])
    mk = lambda: (torch.zeros(1, dtype=torch.int32), torch.full((1,), 4, dtype=torch.int32))
    # margin == tau is NOT stable
    o = oracle.commit(margin, ids, bm, V, 1.0, 16, 1, 1, *mk(), C=8)
    assert o["raw_boundary"].item() == 0 and o["commit_len"].item() == 1
    # tau = +inf: nothing stable, exactly L_min committed
    o = oracle.commit(margin, ids, bm, V, float("inf"), 16, 2, 1, *mk(), C=8)
    assert o["raw_boundary"].item() == 0 and o["commit_len"].item() == 2
    # tau = -inf and no delimiters: everything committed
    o = oracle.commit(margin, ids, bm, V, -float("inf"), 16, 1, 1, *mk(), C=8)
    assert o["raw_boundary"].item() == 4 and o["commit_len"].item() == 4
    # L_min = 0 with nothing stable commits nothing
    o = oracle.commit(margin, ids, bm, V, 5.0, 16, 0, 1, *mk(), C=8)
    assert o["commit_len"].item() == 0


def test_delimiter_is_last_committed_token(oracle):
    """Table 4 shows committed blocks that end WITH the delimiter: the snapped
    length includes it."""
    margin = torch.full((1, 8), 3.0)
    ids = torch.tensor([[9, 9, DELIM, 9, 9, DELIM, 9, 9]], dtype=torch.int32)
    tokens = torch.full((1, 12), -1, dtype=torch.int32)
    pl = torch.tensor([2], dtype=torch.int32)
    sl = torch.tensor([8], dtype=torch.int32)
    o = oracle.commit(margin, ids, _bitmap([DELIM]), V, 0.9, 16, 1, 1, pl, sl, tokens=tokens, C=12)
    assert o["raw_boundary"].item() == 8 and o["snapped_boundary"].item() == 6
    assert tokens[0].tolist() == [-1, -1, 9, 9, DELIM, 9, 9, DELIM, -1, -1, -1, -1]
    assert pl.item() == 8 and sl.item() == 2


def test_window_excludes_far_delimiters(oracle):
    margin = torch.full((1, 10), 3.0)
    ids = torch.full((1, 10), OTHER, dtype=torch.int32)
    ids[0, 2] = DELIM                       # j = 3; L' = 10; distance 7
    for Wn, want in [(6, 10), (7, 3), (-1, 3), (0, 10)]:
        o = oracle.commit(margin, ids, _bitmap([DELIM]), V, 0.9, Wn, 1, 1,
                          torch.zeros(1, dtype=torch.int32), torch.full((1,), 10, dtype=torch.int32), C=16)
        assert o["snapped_boundary"].item() == want, Wn


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_append_copies_exact_rows_and_leaves_the_rest(oracle, dtype):
    w = W.scaled(W.C1, B=3, S=6, P=4, C=12, Hq=2, Hkv=2, D=8, V=V, layers=2, dtype="f32" if dtype == torch.float32 else "bf16")
    pl0 = torch.tensor([4, 0, 9], dtype=torch.int32)
    sl0 = torch.tensor([6, 5, 6], dtype=torch.int32)
    layers = [W.make_layer_kv(w, l, prefix_len=pl0) for l in range(2)]
    before = [{k: v.clone() for k, v in L.items()} for L in layers]
    margin = torch.tensor([[3, 3, 3, 0, 3, 3], [0, 3, 3, 3, 3, 3], [3, 3, 3, 3, 3, 3]], dtype=torch.float32)
    ids = torch.full((3, 6), OTHER, dtype=torch.int32)
    pl, sl = pl0.clone(), sl0.clone()
    o = oracle.commit(margin, ids, _bitmap([]), V, 0.9, 16, 1, 1, pl, sl,
                      k_suf=[L["k_suf"] for L in layers], v_suf=[L["v_suf"] for L in layers],
                      k_cache=[L["k_cache"] for L in layers], v_cache=[L["v_cache"] for L in layers])
    # sequence 2 has room for only 3 rows (C - P = 12 - 9): clamped and flagged
    assert o["commit_len"].tolist() == [3, 1, 3] and o["status_flags"].tolist() == [0, 0, 1]
    for l in range(2):
        for name, src in (("k_cache", "k_suf"), ("v_cache", "v_suf")):
            for b in range(3):
                P, Lc = int(pl0[b]), int(o["commit_len"][b])
                got = layers[l][name][b]
                assert torch.equal(got[P:P + Lc], before[l][src][b, :Lc])
                assert torch.equal(got[:P], before[l][name][b, :P])
                assert torch.equal(got[P + Lc:], before[l][name][b, P + Lc:])   # poison intact
                assert torch.all(got[P + Lc:].float() == W.POISON_F32)


def test_planted_stable_length_workload(oracle):
    """Config-3 style plant: raw boundary equals the planted stable length."""
    w = W.scaled(W.C3, B=4, S=40, V=2048, P=8, C=64)
    sl_plant = torch.tensor([0, 17, 40, 39])
    z, info = W.make_logits(w, stable_len=sl_plant)
    ids, p, m = oracle.confidence(z)
    _, bm = W.make_delimiters(w)
    pl, sl = W.make_lengths(w)
    o = oracle.commit(m, ids, bm, w.V, w.tau, w.window, 1, 1, pl, sl, C=w.C)
    assert o["raw_boundary"].tolist() == sl_plant.tolist()
    delim_ids, _ = W.make_delimiters(w)
    dset = set(delim_ids.tolist())
    for b in range(4):
        Lp, Ls = int(o["raw_boundary"][b]), int(o["snapped_boundary"][b])
        assert Ls <= Lp and (Ls == Lp or int(ids[b, Ls - 1]) in dset) and Lp - Ls <= w.window

"""Pins for the Scattered-Margin oracle (Section 4.3.3): selection against a
library sort and against exhaustive subset enumeration, invariants, and the
gathered cache append against plain tensor indexing."""
import itertools

import numpy as np
import torch

import workloads as W


def test_selection_against_stable_sort(oracle):
    g = torch.Generator().manual_seed(0)
    B, S = 40, 37
    margin = (torch.rand((B, S), generator=g) * 6).round() / 2          # quantised: many ties
    sl = torch.randint(0, S + 1, (B,), generator=g, dtype=torch.int32)
    ct = torch.randint(0, S + 3, (B,), generator=g, dtype=torch.int32)
    idx, mask = oracle.select_scattered(margin, sl, ct)
    for b in range(B):
        n, k = int(sl[b]), min(int(ct[b]), int(sl[b]))
        order = np.argsort(-margin[b, :n].numpy(), kind="stable")        # largest first, ties by position
        want = sorted(order[:k].tolist())
        assert idx[b, :k].tolist() == want and torch.all(idx[b, k:] == -1)
        assert mask[b].tolist() == [int(i in set(want)) for i in range(S)]


def test_selection_maximises_the_margin_sum_over_all_subsets(oracle):
    """Tiny rows, distinct margins: the selected set is THE subset of size k with
    the largest total margin (checked against every subset)."""
    g = torch.Generator().manual_seed(1)
    N = 7
    margin = torch.randperm(N, generator=g).float().view(1, N) * 0.5
    for k in range(N + 1):
        idx, mask = oracle.select_scattered(margin, torch.tensor([N], dtype=torch.int32), torch.tensor([k], dtype=torch.int32))
        best = max(itertools.combinations(range(N), k), key=lambda c: sum(float(margin[0, i]) for i in c))
        assert idx[0, :k].tolist() == sorted(best)


def test_selection_edge_cases(oracle):
    margin = torch.tensor([[1.0, 1.0, 1.0, 1.0, 9.0]])
    one = lambda n, k: oracle.select_scattered(margin, torch.tensor([n], dtype=torch.int32), torch.tensor([k], dtype=torch.int32))
    assert one(5, 0)[0].tolist() == [[-1] * 5]
    assert one(5, 5)[0].tolist() == [[0, 1, 2, 3, 4]]
    assert one(5, 2)[0][0, :2].tolist() == [0, 4]              # the 9, then the lowest-position 1
    assert one(4, 2)[0][0, :2].tolist() == [0, 1]              # position 4 is not active
    assert one(0, 3)[1].sum() == 0
    # every selected margin >= every unselected active margin
    g = torch.Generator().manual_seed(2)
    m = torch.rand((6, 50), generator=g)
    sl = torch.full((6,), 50, dtype=torch.int32)
    idx, mask = oracle.select_scattered(m, sl, torch.tensor([0, 1, 10, 25, 49, 50], dtype=torch.int32))
    for b in range(6):
        s, u = m[b][mask[b] == 1], m[b][mask[b] == 0]
        assert s.numel() == 0 or u.numel() == 0 or s.min() >= u.max()


def test_gather_append_against_tensor_indexing(oracle):
    w = W.scaled(W.C1, B=3, S=20, P=5, C=32, Hq=2, Hkv=2, D=8, V=64, layers=2, dtype="bf16")
    layers = [W.make_layer_kv(w, l) for l in range(2)]
    before = [{k: v.clone() for k, v in L.items()} for L in layers]
    g = torch.Generator().manual_seed(3)
    margin = torch.rand((3, 20), generator=g)
    sl = torch.tensor([20, 11, 0], dtype=torch.int32)
    ct = torch.tensor([30, 4, 2], dtype=torch.int32)             # seq 0 wants more rows than the cache has room for
    pl = torch.tensor([5, 5, 5], dtype=torch.int32)
    idx, _ = oracle.select_scattered(margin, sl, ct)
    cnt = torch.minimum(ct, sl)
    oracle.gather_append(idx, cnt, pl, [L["k_suf"] for L in layers], [L["v_suf"] for L in layers],
                         [L["k_cache"] for L in layers], [L["v_cache"] for L in layers])
    assert pl.tolist() == [5 + 20, 5 + 4, 5]
    for L, L0 in zip(layers, before):
        for b in range(3):
            k = int(pl[b]) - 5
            rows = idx[b, :k].long()
            for name, suf in (("k_cache", "k_suf"), ("v_cache", "v_suf")):
                assert torch.equal(L[name][b, 5:5 + k], L0[suf][b][rows])               # gathered rows, in order
                assert torch.equal(L[name][b, :5], L0[name][b, :5])                     # prefix untouched
                assert torch.equal(L[name][b, 5 + k:], L0[name][b, 5 + k:])             # rest untouched (poison)


def test_gather_append_stops_where_the_selection_list_ends(oracle):
    """count[b] larger than the number of active positions: the selection holds N_b entries
    and is padded with -1; only those N_b rows are appended and the prefix advances by N_b
    (no more positions can be committed than exist)."""
    w = W.scaled(W.C1, B=3, S=12, P=3, C=40, Hq=2, Hkv=2, D=8, V=64, layers=2, dtype="f32")
    layers = [W.make_layer_kv(w, l) for l in range(2)]
    before = [{k: v.clone() for k, v in L.items()} for L in layers]
    margin = torch.rand((3, 12), generator=torch.Generator().manual_seed(8))
    sl = torch.tensor([12, 4, 0], dtype=torch.int32)
    ct = torch.tensor([5, 9, 3], dtype=torch.int32)               # sequences 1 and 2 ask for more than they have
    pl = torch.tensor([3, 3, 3], dtype=torch.int32)
    idx, _ = oracle.select_scattered(margin, sl, ct)
    assert (idx[1] >= 0).sum() == 4 and (idx[2] >= 0).sum() == 0
    oracle.gather_append(idx, ct, pl, [L["k_suf"] for L in layers], [L["v_suf"] for L in layers],
                         [L["k_cache"] for L in layers], [L["v_cache"] for L in layers])
    assert pl.tolist() == [3 + 5, 3 + 4, 3]
    for L, L0 in zip(layers, before):
        for b, k in enumerate([5, 4, 0]):
            rows = idx[b, :k].long()
            assert torch.equal(L["k_cache"][b, 3:3 + k], L0["k_suf"][b][rows])
            assert torch.equal(L["v_cache"][b, 3:3 + k], L0["v_suf"][b][rows])
            assert torch.equal(L["k_cache"][b, 3 + k:], L0["k_cache"][b, 3 + k:])       # nothing beyond

"""GPU parity for the Scattered-Margin pieces (Section 4.3.3): selection and
gathered append bit-exact against the oracle; attention over an index-addressed
cache against the oracle run on the gathered rows."""
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


@pytest.mark.parametrize("S", [5, 64, 257, 1024, 1500])
def test_selection_matches_oracle(lsp, oracle, S):
    g = torch.Generator().manual_seed(S)
    B = 9
    margin = torch.rand((B, S), generator=g)
    margin[1] = (margin[1] * 4).floor() / 4                      # heavy ties
    margin[2] = 1.0                                              # all equal: the first k positions
    sl = torch.tensor([S, S, S, max(S - 3, 0), 1, 0, S // 2, S, S], dtype=torch.int32)
    ct = torch.tensor([S // 3, S // 2, 7, S, 1, 4, S // 2 + 5, 0, S], dtype=torch.int32)
    ri, rm = oracle.select_scattered(margin, sl, ct)
    gi, gm = lsp.select_scattered(margin.cuda(), sl.cuda(), ct.cuda())
    torch.cuda.synchronize()
    assert torch.equal(gi.cpu(), ri) and torch.equal(gm.cpu(), rm)


def test_selection_at_config_shapes(lsp, oracle):
    """Margins of the config-3 logits (four sequences of 512) and the block sizes LSP
    itself commits there."""
    w = W.C3
    z, _ = W.make_logits(w, device="cuda")
    ids, p, m = lsp.confidence(z)
    _, bm = W.make_delimiters(w)
    pl, sl = (t.cuda() for t in W.make_lengths(w))
    out = lsp.commit(m, ids, bm.cuda(), w.V, w.tau, w.window, 1, 1, pl.clone(), sl.clone(), C=w.C)
    gi, gm = lsp.select_scattered(m, sl, out["commit_len"])
    torch.cuda.synchronize()
    ri, rm = oracle.select_scattered(m.cpu(), sl.cpu(), out["commit_len"].cpu())
    assert torch.equal(gi.cpu(), ri) and torch.equal(gm.cpu(), rm)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gather_append_matches_oracle(lsp, oracle, dtype):
    w = W.scaled(W.C1, B=4, S=40, P=10, C=64, Hq=2, Hkv=2, D=64, V=64, layers=3, dtype=dtype)
    pl = torch.tensor([10, 0, 50, 64], dtype=torch.int32)         # seq 2 nearly full, seq 3 full
    sl = torch.tensor([40, 33, 40, 5], dtype=torch.int32)
    ct = torch.tensor([12, 33, 30, 3], dtype=torch.int32)
    layers = [W.make_layer_kv(w, l, prefix_len=pl) for l in range(3)]
    margin = torch.rand((4, 40), generator=torch.Generator().manual_seed(5))
    idx, _ = oracle.select_scattered(margin, sl, ct)
    cnt = torch.minimum(ct, sl)
    ref = [{k: v.clone() for k, v in L.items()} for L in layers]
    pl_r = pl.clone()
    oracle.gather_append(idx, cnt, pl_r, [L["k_suf"] for L in ref], [L["v_suf"] for L in ref],
                         [L["k_cache"] for L in ref], [L["v_cache"] for L in ref])
    dev = [{k: v.cuda() for k, v in L.items()} for L in layers]
    table = lsp.LayerTable([L["k_suf"] for L in dev], [L["v_suf"] for L in dev], [L["k_cache"] for L in dev], [L["v_cache"] for L in dev])
    pl_g = pl.cuda()
    app = lsp.kv_gather_append(idx.cuda(), cnt.cuda(), pl_g, table)
    torch.cuda.synchronize()
    assert torch.equal(pl_g.cpu(), pl_r) and app.cpu().tolist() == (pl_r - pl).tolist()
    view = torch.int16 if dtype == "bf16" else torch.int32
    for Lg, Lr in zip(dev, ref):
        for name in ("k_cache", "v_cache"):
            assert torch.equal(Lg[name].cpu().view(view), Lr[name].view(view)), name


@pytest.mark.parametrize("cfg", ["small_f32", "short_bf16", "long_bf16"])
def test_attention_over_index_addressed_cache(lsp, oracle, cfg):
    """The prefix keys live in shuffled cache rows; the kernel reads them through the
    row index.  Reference: the oracle on a cache whose rows were put back in order."""
    if cfg == "small_f32":
        w = W.scaled(W.C1, B=2, S=40, P=70, C=128, Hq=4, Hkv=2, D=64)
    elif cfg == "short_bf16":
        w = W.scaled(W.C2, B=2, S=100, P=300, C=512, Hq=4, Hkv=4, D=128, seed=3)
    else:
        w = W.scaled(W.C2, B=3, S=520, P=300, C=512, Hq=24, Hkv=8, D=128, seed=4)     # shared-tile launch shape
    pl = torch.full((w.B,), w.P, dtype=torch.int32)
    pl[0] = w.P - 37
    sl = torch.full((w.B,), w.S, dtype=torch.int32)
    sl[-1] = w.S - 9
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    g = torch.Generator().manual_seed(8)
    rows = torch.stack([torch.randperm(w.C, generator=g) for _ in range(w.B)]).to(torch.int32)   # logical t -> physical row
    shuffled = {k: v.clone() for k, v in kv.items()}
    for name in ("k_cache", "v_cache"):
        for b in range(w.B):
            p = int(pl[b])
            shuffled[name][b] = W.POISON_F32
            shuffled[name][b][rows[b, :p].long()] = kv[name][b, :p]
    d = {k: v.cuda() for k, v in shuffled.items()}
    out = lsp.attn_step(d["q"], d["k_suf"], d["v_suf"], d["k_cache"], d["v_cache"], pl.cuda(), sl.cuda(),
                        cache_row_index=rows.cuda())
    torch.cuda.synchronize()
    n = 48
    pick = torch.stack([torch.randint(0, w.B, (n,), generator=g), torch.zeros(n, dtype=torch.int64),
                        torch.randint(0, w.Hq, (n,), generator=g)], 1)
    for r in range(n):
        pick[r, 1] = int(torch.randint(0, int(sl[pick[r, 0]]), (1,), generator=g))
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=pick.to(torch.int32))
    got = out[pick[:, 0].cuda(), pick[:, 1].cuda(), pick[:, 2].cuda()].float().cpu()
    tol = 1e-5 if w.dtype == "f32" else 2e-2
    assert (got - ref).abs().max().item() <= tol


def test_gather_append_with_count_above_the_active_positions(lsp, oracle):
    """count[b] > N_b: the selection is padded with -1 and the append stops at the padding
    on both sides (rows appended = N_b, nothing written beyond them)."""
    w = W.scaled(W.C1, B=4, S=300, P=10, C=400, Hq=2, Hkv=2, D=64, V=64, layers=2, dtype="bf16")
    pl = torch.tensor([10, 0, 395, 20], dtype=torch.int32)        # sequence 2: room for 5 rows only
    sl = torch.tensor([300, 7, 40, 0], dtype=torch.int32)
    ct = torch.tensor([290, 300, 30, 12], dtype=torch.int32)      # 1 and 3 ask for more than they have
    layers = [W.make_layer_kv(w, l, prefix_len=pl) for l in range(2)]
    margin = torch.rand((4, 300), generator=torch.Generator().manual_seed(6))
    ref = [{k: v.clone() for k, v in L.items()} for L in layers]
    pl_r = pl.clone()
    idx_r, _ = oracle.select_scattered(margin, sl, ct)
    oracle.gather_append(idx_r, ct, pl_r, [L["k_suf"] for L in ref], [L["v_suf"] for L in ref],
                         [L["k_cache"] for L in ref], [L["v_cache"] for L in ref])
    assert (pl_r - pl).tolist() == [290, 7, 5, 0]
    dev = [{k: v.cuda() for k, v in L.items()} for L in layers]
    table = lsp.LayerTable([L["k_suf"] for L in dev], [L["v_suf"] for L in dev], [L["k_cache"] for L in dev], [L["v_cache"] for L in dev])
    pl_g = pl.cuda()
    idx_g, _ = lsp.select_scattered(margin.cuda(), sl.cuda(), ct.cuda())
    assert torch.equal(idx_g.cpu(), idx_r)
    app = lsp.kv_gather_append(idx_g, ct.cuda(), pl_g, table)
    torch.cuda.synchronize()
    assert torch.equal(pl_g.cpu(), pl_r) and app.cpu().tolist() == (pl_r - pl).tolist()
    for Lg, Lr in zip(dev, ref):
        for name in ("k_cache", "v_cache"):
            assert torch.equal(Lg[name].cpu().view(torch.int16), Lr[name].view(torch.int16)), name

"""GPU parity: lsp_commit against the CPU oracle (Section 3.2; Algorithm 1
lines 7-10).  Everything is integer / byte work: bit-exact."""
import itertools

import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu
V = 64
DELIM, OTHER = 5, 9


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


def _bitmap(ids, V=V):
    words = torch.zeros((V + 31) // 32, dtype=torch.int64)
    for v in ids:
        words[v // 32] |= 1 << (v % 32)
    return torch.where(words >= 2**31, words - 2**32, words).to(torch.int32)


def _same(a, b):
    """Bit-for-bit equal; NaN (the 'no threshold' marker of tau_used) equals NaN."""
    if a.dtype.is_floating_point:
        return torch.equal(torch.isnan(a), torch.isnan(b)) and torch.equal(a[~torch.isnan(a)], b[~torch.isnan(b)])
    return torch.equal(a, b)


def _both(lsp, oracle, margin, ids, bm, Vv, tau, Wn, Lmin, snap, pl, sl, tokens=None, layers=None, C=None, **sizing):
    """Run oracle (CPU clones) and HIP (GPU clones); compare every output.
    sizing: adaptive / alpha / beta / max_commit, passed to both sides."""
    pl_r, sl_r = pl.clone(), sl.clone()
    tok_r = None if tokens is None else tokens.clone()
    kw = {}
    lay_r = None
    if layers is not None:
        lay_r = [{k: v.clone() for k, v in L.items()} for L in layers]
        kw = dict(k_suf=[L["k_suf"] for L in lay_r], v_suf=[L["v_suf"] for L in lay_r],
                  k_cache=[L["k_cache"] for L in lay_r], v_cache=[L["v_cache"] for L in lay_r])
    ref = oracle.commit(margin, ids, bm, Vv, tau, Wn, Lmin, snap, pl_r, sl_r, tokens=tok_r, C=C, **kw, **sizing)
    pl_g, sl_g = pl.cuda(), sl.cuda()
    tok_g = None if tokens is None else tokens.cuda()
    table = None
    lay_g = None
    if layers is not None:
        lay_g = [{k: v.cuda() for k, v in L.items()} for L in layers]
        table = lsp.LayerTable([L["k_suf"] for L in lay_g], [L["v_suf"] for L in lay_g],
                               [L["k_cache"] for L in lay_g], [L["v_cache"] for L in lay_g])
    got = lsp.commit(margin.cuda(), ids.cuda(), bm.cuda(), Vv, tau, Wn, Lmin, snap, pl_g, sl_g,
                     tokens=tok_g, layers=table, C=C, **sizing)
    torch.cuda.synchronize()
    for k in ref:
        assert _same(got[k].cpu(), ref[k]), k
    assert torch.equal(pl_g.cpu(), pl_r) and torch.equal(sl_g.cpu(), sl_r)
    if tokens is not None:
        assert torch.equal(tok_g.cpu(), tok_r)
    if layers is not None:
        for Lg, Lr in zip(lay_g, lay_r):
            for name in ("k_cache", "v_cache"):
                assert torch.equal(Lg[name].cpu().view(torch.int16 if Lr[name].dtype == torch.bfloat16 else torch.int32),
                                   Lr[name].view(torch.int16 if Lr[name].dtype == torch.bfloat16 else torch.int32)), name
    return ref


@pytest.mark.parametrize("Wn,Lmin,snap", [(0, 0, 1), (1, 1, 1), (3, 2, 1), (-1, 1, 1), (16, 1, 0)])
def test_every_mask_and_delimiter_placement(lsp, oracle, Wn, Lmin, snap):
    N = 6
    cases = list(itertools.product(itertools.product([0, 1], repeat=N), itertools.product([0, 1], repeat=N)))
    B = len(cases)
    margin = torch.tensor([[2.0 if m else 0.5 for m in mk] + [9.0] for mk, _ in cases], dtype=torch.float32)
    ids = torch.tensor([[DELIM if d else OTHER for d in dl] + [DELIM] for _, dl in cases], dtype=torch.int32)
    pl = torch.full((B,), 2, dtype=torch.int32)
    sl = torch.tensor([N - (b % 3 == 0) * (b % 5) for b in range(B)], dtype=torch.int32).clamp(min=0)
    tokens = torch.full((B, 12), -1, dtype=torch.int32)
    _both(lsp, oracle, margin, ids, _bitmap([DELIM]), V, 1.0, Wn, Lmin, snap, pl, sl, tokens=tokens, C=12)


def test_long_rows_many_waves(lsp, oracle):
    """S spans several 256-position chunks; first unstable position placed in
    every wave/chunk; unlimited and bounded windows."""
    S = 1100
    firsts = [0, 1, 63, 64, 65, 255, 256, 257, 511, 700, 1023, 1024, 1099, 1100]
    B = len(firsts)
    g = torch.Generator().manual_seed(0)
    margin = 1.0 + torch.rand((B, S), generator=g)
    for b, f in enumerate(firsts):
        if f < S:
            margin[b, f] = 0.25
            margin[b, min(f + 7, S - 1)] = 0.1       # a later unstable position must not win
    ids = torch.randint(0, 4096, (B, S), generator=g, dtype=torch.int32)
    dl = torch.randperm(4096, generator=g)[:200]
    bm = _bitmap(dl.tolist(), 4096)
    for Wn in (16, -1, 0, 300):
        pl = torch.zeros(B, dtype=torch.int32)
        sl = torch.full((B,), S, dtype=torch.int32)
        tokens = torch.full((B, S), -1, dtype=torch.int32)
        ref = _both(lsp, oracle, margin, ids, bm, 4096, 0.9, Wn, 1, 1, pl, sl, tokens=tokens, C=4096)
        assert ref["raw_boundary"].tolist() == firsts


def test_thresholds_inf_and_strictness(lsp, oracle):
    margin = torch.tensor([[1.0, 1.0, 1.0, 1.0]] * 4, dtype=torch.float32)
    ids = torch.full((4, 4), OTHER, dtype=torch.int32)
    for tau, Lmin in [(1.0, 1), (float("inf"), 2), (-float("inf"), 1), (5.0, 0)]:
        pl = torch.zeros(4, dtype=torch.int32)
        sl = torch.tensor([4, 3, 1, 0], dtype=torch.int32)
        _both(lsp, oracle, margin, ids, _bitmap([]), V, tau, 16, Lmin, 1, pl, sl, C=8)


def test_out_of_range_ids_are_not_delimiters(lsp):
    margin = torch.full((1, 4), 3.0).cuda()
    ids = torch.tensor([[-5, 1 << 30, 63, 5]], dtype=torch.int32).cuda()
    pl, sl = torch.zeros(1, dtype=torch.int32).cuda(), torch.full((1,), 4, dtype=torch.int32).cuda()
    out = lsp.commit(margin, ids, _bitmap([63]).cuda(), V, 0.9, -1, 1, 1, pl, sl, C=8)
    torch.cuda.synchronize()
    assert out["snapped_boundary"].item() == 3


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_rows_flags_and_poison(lsp, oracle, dtype):
    w = W.scaled(W.C1, B=4, S=40, P=10, C=64, Hq=2, Hkv=2, D=64, V=V, layers=3, dtype=dtype)
    pl = torch.tensor([10, 0, 50, 64], dtype=torch.int32)       # seq 2 nearly full, seq 3 full
    sl = torch.tensor([40, 33, 40, 5], dtype=torch.int32)
    layers = [W.make_layer_kv(w, l, prefix_len=pl) for l in range(3)]
    g = torch.Generator().manual_seed(1)
    margin = 2 * torch.rand((4, 40), generator=g)
    margin[:, :20] += 1.0
    ids = torch.randint(0, V, (4, 40), generator=g, dtype=torch.int32)
    tokens = torch.full((4, 60), -1, dtype=torch.int32)         # T < C: token room clamps too
    ref = _both(lsp, oracle, margin, ids, _bitmap([5, 6, 7, 8]), V, 0.9, 16, 1, 1, pl, sl, tokens=tokens, layers=layers)
    assert ref["status_flags"][2].item() & 1 and ref["status_flags"][3].item() & 1
    assert ref["commit_len"][3].item() == 0


def test_scan_only_without_tokens(lsp, oracle):
    margin = torch.full((2, 8), 3.0)
    ids = torch.full((2, 8), OTHER, dtype=torch.int32)
    pl = torch.tensor([1, 2], dtype=torch.int32)
    sl = torch.tensor([8, 5], dtype=torch.int32)
    _both(lsp, oracle, margin, ids, _bitmap([DELIM]), V, 0.9, 16, 1, 1, pl, sl, C=32)


@pytest.mark.parametrize("cfg", ["c2", "c3"])
def test_full_config_shapes(lsp, oracle, cfg):
    """Configs 2 and 3 at full size: confidence by the oracle feeds both sides."""
    w = W.C2 if cfg == "c2" else W.C3
    z, info = W.make_logits(w, device="cuda")
    # margins/ids for the commit come from the HIP confidence (already parity-tested) to keep this fast
    ids, p, m = lsp.confidence(z)
    torch.cuda.synchronize()
    _, bm = W.make_delimiters(w)
    pl, sl = W.make_lengths(w)
    layers = [W.make_layer_kv(w, 0)]
    tokens = W.make_tokens(w, w.C)
    ref = _both(lsp, oracle, m.cpu(), ids.cpu(), bm, w.V, w.tau, w.window, 1, 1, pl, sl, tokens=tokens, layers=layers)
    if cfg == "c3":
        assert ref["raw_boundary"].tolist() == info["stable_len"].tolist()
    assert torch.all(ref["snapped_boundary"] <= ref["raw_boundary"])


@pytest.mark.parametrize("cfg", ["c2", "c3"])
def test_confidence_then_commit_each_side_on_its_own(lsp, oracle, cfg):
    """Configs 2 and 3 at full size with NOTHING passed between the two sides: the oracle's
    commit consumes the oracle's ids and margins (all rows), the library's commit consumes
    the library's; every output of the pair of calls is then compared (Algorithm 1 lines
    5 and 7-10 chained)."""
    w = W.C2 if cfg == "c2" else W.C3
    z, info = W.make_logits(w)
    _, bm = W.make_delimiters(w)
    pl, sl = W.make_lengths(w)
    layers = [W.make_layer_kv(w, 0)]
    tokens = W.make_tokens(w, w.C)
    # oracle side
    ids_r, p_r, m_r = oracle.confidence(z, sl)
    lay_r = [{k: v.clone() for k, v in L.items()} for L in layers]
    pl_r, sl_r, tok_r = pl.clone(), sl.clone(), tokens.clone()
    ref = oracle.commit(m_r, ids_r, bm, w.V, w.tau, w.window, 1, 1, pl_r, sl_r, tokens=tok_r,
                        k_suf=[L["k_suf"] for L in lay_r], v_suf=[L["v_suf"] for L in lay_r],
                        k_cache=[L["k_cache"] for L in lay_r], v_cache=[L["v_cache"] for L in lay_r])
    # library side
    lay_g = [{k: v.cuda() for k, v in L.items()} for L in layers]
    table = lsp.LayerTable([L["k_suf"] for L in lay_g], [L["v_suf"] for L in lay_g],
                           [L["k_cache"] for L in lay_g], [L["v_cache"] for L in lay_g])
    pl_g, sl_g, tok_g = pl.cuda(), sl.cuda(), tokens.cuda()
    ids_g, p_g, m_g = lsp.confidence(z.cuda(), sl_g)
    got = lsp.commit(m_g, ids_g, bm.cuda(), w.V, w.tau, w.window, 1, 1, pl_g, sl_g, tokens=tok_g, layers=table)
    torch.cuda.synchronize()
    act = torch.arange(w.S)[None, :] < sl[:, None]
    assert torch.equal(ids_g.cpu()[act], ids_r[act]) and torch.equal(m_g.cpu()[act], m_r[act])
    assert (p_g.cpu()[act] - p_r[act]).abs().max().item() <= 2e-2
    for k in ref:
        assert _same(got[k].cpu(), ref[k]), k
    assert torch.equal(pl_g.cpu(), pl_r) and torch.equal(sl_g.cpu(), sl_r) and torch.equal(tok_g.cpu(), tok_r)
    for name in ("k_cache", "v_cache"):
        assert torch.equal(lay_g[0][name].cpu().view(torch.int16), lay_r[0][name].view(torch.int16)), name
    assert int(ref["commit_len"].sum()) > 0


def test_c4_shape_two_layers(lsp, oracle):
    """Config-4 cache geometry (B=8, C=8192, rows of 8 KB), two layers, worst-case
    commit length (tau = -inf, no snap => L = S = 1024 rows per sequence)."""
    w = W.scaled(W.C4, layers=2)
    layers = [W.make_layer_kv(w, l) for l in range(2)]
    margin = torch.ones((w.B, w.S))
    ids = torch.randint(0, w.V, (w.B, w.S), generator=torch.Generator().manual_seed(3), dtype=torch.int32)
    _, bm = W.make_delimiters(w)
    pl, sl = W.make_lengths(w)
    ref = _both(lsp, oracle, margin, ids, bm, w.V, -float("inf"), 16, 1, 0, pl, sl, layers=layers)
    assert ref["commit_len"].tolist() == [w.S] * w.B


def test_many_layers_more_than_one_launch(lsp, oracle):
    w = W.scaled(W.C1, B=2, S=16, P=4, C=32, Hq=1, Hkv=1, D=64, V=V, layers=70, dtype="bf16")
    pl, sl = W.make_lengths(w)
    layers = [W.make_layer_kv(w, l) for l in range(70)]
    margin = torch.full((2, 16), 3.0)
    margin[0, 9] = 0
    ids = torch.full((2, 16), OTHER, dtype=torch.int32)
    _both(lsp, oracle, margin, ids, _bitmap([]), V, 0.9, 16, 1, 1, pl, sl, layers=layers)


# ---- adaptive threshold (Section 3.2 targeted block sizing, Eq. 2) and commit cap (Table 2) ----
@pytest.mark.parametrize("alpha,beta", [(0.25, 0.5), (0.5, 0.5), (0.2, 1.0), (0.75, 0.75)])
def test_adaptive_every_small_margin_vector(lsp, oracle, alpha, beta):
    N = 5
    vals = [1.0, 2.0, 3.0, 4.0]
    rows = list(itertools.product(vals, repeat=N))
    margin = torch.tensor(rows, dtype=torch.float32)
    B = len(rows)
    ids = torch.tensor([[DELIM if (b >> i) & 1 else OTHER for i in range(N)] for b in range(B)], dtype=torch.int32)
    for tau0 in (0.5, 2.0, 2.5, 4.0):
        pl = torch.zeros(B, dtype=torch.int32)
        sl = torch.tensor([N - (b % 7 == 0) * (b % 4) for b in range(B)], dtype=torch.int32)
        _both(lsp, oracle, margin, ids, _bitmap([DELIM]), V, tau0, 2, 1, 1, pl, sl, C=16,
              adaptive=True, alpha=alpha, beta=beta)


@pytest.mark.parametrize("tau0", [-float("inf"), 0.3, 0.9, float("inf")])
def test_adaptive_long_ragged_rows(lsp, oracle, tau0):
    """Rows longer than one position per thread, lengths that end inside chunks,
    quantised margins (ties), an empty suffix; three acceptance intervals."""
    S = 1500
    g = torch.Generator().manual_seed(4)
    B = 12
    margin = torch.rand((B, S), generator=g)
    margin[0] = torch.linspace(3.0, 1.0, S)                          # strictly decreasing: every length reachable
    margin[1] = 2.0                                                  # constant: only 0 and N reachable
    margin[2] = (margin[2] * 8).floor() / 8                          # heavy ties
    margin[3, :700] += 1.0
    margin[4, 0] = 0.0                                               # unstable at once
    ids = torch.randint(0, 4096, (B, S), generator=g, dtype=torch.int32)
    bm = _bitmap(torch.randperm(4096, generator=g)[:300].tolist(), 4096)
    sl0 = torch.tensor([1500, 1500, 1499, 1024, 1500, 1, 2, 257, 0, 777, 1300, 64], dtype=torch.int32)
    for alpha, beta in [(0.25, 0.5), (0.1, 0.1), (0.6, 1.0)]:
        pl = torch.zeros(B, dtype=torch.int32)
        ref = _both(lsp, oracle, margin, ids, bm, 4096, tau0, 16, 1, 1, pl, sl0.clone(), C=4096,
                    adaptive=True, alpha=alpha, beta=beta)
        for b in range(B):
            n = int(sl0[b])
            if n:
                lo = min(n, int(torch.ceil(torch.tensor(alpha, dtype=torch.float32) * n)))
                hi = max(lo, min(n, int(torch.floor(torch.tensor(beta, dtype=torch.float32) * n))))
                assert lo <= int(ref["raw_boundary"][b]) <= hi                 # Eq. 2 holds for every sequence


def test_commit_cap_and_adaptive_with_append(lsp, oracle):
    w = W.scaled(W.C1, B=3, S=48, P=8, C=64, Hq=2, Hkv=2, D=64, V=V, layers=2, dtype="bf16")
    pl, sl = W.make_lengths(w)
    layers = [W.make_layer_kv(w, l) for l in range(2)]
    g = torch.Generator().manual_seed(2)
    margin = 3.0 * torch.rand((3, 48), generator=g)
    ids = torch.randint(0, V, (3, 48), generator=g, dtype=torch.int32)
    tokens = torch.full((3, 64), -1, dtype=torch.int32)
    for kw in (dict(max_commit=5), dict(adaptive=True, alpha=0.25, beta=0.5), dict(adaptive=True, alpha=0.25, beta=0.5, max_commit=7)):
        _both(lsp, oracle, margin, ids, _bitmap([5, 6, 7]), V, 0.9, 16, 1, 1, pl.clone(), sl.clone(), tokens=tokens.clone(),
              layers=[{k: v.clone() for k, v in L.items()} for L in layers], **kw)

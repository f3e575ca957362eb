"""GPU parity: lsp_lm_head_confidence (output head fused with Eq. 1, Algorithm 1
lines 4-5) against the CPU oracle, which keeps the logits in double.

The kernel sums bf16 products in fp32 in its own order, so:
  * operands whose logits are exact in fp32 (small integers) must match the
    oracle BIT-exactly, ties included;
  * otherwise the margin is within MARGIN_TOL and the probability within
    PROB_TOL of the oracle, the id equals the oracle's wherever the oracle's
    margin exceeds MARGIN_TOL, and elsewhere it names an entry whose exact logit
    is within MARGIN_TOL of the maximum.
Tolerances: K <= 4096 products of magnitude ~ |h||w| <= 1 summed in fp32 carry an
error of about sqrt(K) * 2^-24 * |z| <= 1e-5 for |z| <= 20; a margin is a
difference of two such sums, a probability a ratio of sums of their exponentials."""
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu
MARGIN_TOL = 1e-4
PROB_TOL = 5e-5


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


def _run(lsp, hidden_gpu, weight_gpu, sl=None):
    B, S, _ = hidden_gpu.shape
    out = (torch.full((B, S), -7, dtype=torch.int32, device="cuda"),
           torch.full((B, S), -7.0, device="cuda"), torch.full((B, S), -7.0, device="cuda"))
    ids, p, m = lsp.lm_head_confidence(hidden_gpu, weight_gpu, None if sl is None else sl.cuda(), out=out)
    torch.cuda.synchronize()
    return ids.cpu(), p.cpu(), m.cpu()


def _compare(got, ref, z, exact=False):
    ids, p, m = got
    ids_r, p_r, m_r = ref
    act = ids_r >= 0
    assert torch.all(ids[~act] == -7) and torch.all(m[~act] == -7.0) and torch.all(p[~act] == -7.0)
    if exact:
        assert torch.equal(ids[act], ids_r[act]) and torch.equal(m[act], m_r[act])
    else:
        clear = act & (m_r > MARGIN_TOL)
        assert torch.equal(ids[clear], ids_r[clear])
        assert (m[act] - m_r[act]).abs().max().item() <= MARGIN_TOL
        if z is not None:  # an id in a near-tie must still name a near-maximal entry
            zmax = z.max(dim=-1).values
            zid = z.gather(-1, ids.clamp(min=0).long().unsqueeze(-1)).squeeze(-1)
            assert ((zmax - zid)[act] <= MARGIN_TOL).all()
    assert (p[act] - p_r[act]).abs().max().item() <= PROB_TOL
    assert (ids[act] >= 0).all() and (ids[act] < (z.shape[-1] if z is not None else 1 << 30)).all()


@pytest.mark.parametrize("B,S,K,V", [(2, 150, 200, 700), (1, 64, 64, 256), (3, 257, 72, 513), (1, 5, 8, 2),
                                      (1, 300, 136, 1031)])
def test_random_operands_several_tiles_and_ragged_edges(lsp, oracle, B, S, K, V):
    """Rows, vocabulary and K each span several tiles with ragged ends (K = 200 is
    three 64-steps plus one 8-element piece; V = 2 a single nearly empty tile)."""
    w = W.scaled(W.C2, B=B, S=S, V=V, n_delim=min(64, max(1, V // 4)), seed=2000 + V)
    hidden, weight, _ = W.make_lm_head(w, K)
    ref = oracle.lm_head_confidence(hidden, weight, return_logits=True)
    got = _run(lsp, hidden.cuda(), weight.cuda())
    _compare(got, ref[:3], ref[3])


def test_exact_integer_logits_bitwise_with_ties(lsp, oracle):
    g = torch.Generator().manual_seed(7)
    h = torch.randint(-3, 4, (2, 130, 96), generator=g).to(torch.bfloat16)
    w = torch.randint(-3, 4, (777, 96), generator=g).to(torch.bfloat16)
    # duplicated vocabulary entries at several distances: same lane, other half, other wave, other tile
    for a, b in [(5, 6), (10, 14), (40, 200), (100, 600), (300, 301), (0, 776)]:
        w[b] = w[a]
    ref = oracle.lm_head_confidence(h, w, return_logits=True)
    assert (ref[2] == 0).any()
    got = _run(lsp, h.cuda(), w.cuda())
    _compare(got, ref[:3], ref[3], exact=True)


def test_inactive_rows_and_whole_inactive_tiles(lsp, oracle):
    w = W.scaled(W.C2, B=3, S=300, V=520, seed=2101)
    hidden, weight, _ = W.make_lm_head(w, 128)
    sl = torch.tensor([300, 0, 17], dtype=torch.int32)
    ref = oracle.lm_head_confidence(hidden, weight, suffix_len=sl)
    got = _run(lsp, hidden.cuda(), weight.cuda(), sl)
    _compare(got, ref, None)


def test_strided_hidden_and_weight_views(lsp, oracle):
    g = torch.Generator().manual_seed(9)
    K = 96
    hbig = torch.randn((2, 70, 2 * K), generator=g).to(torch.bfloat16)
    wbig = (torch.randn((300, K + 24), generator=g) / 10).to(torch.bfloat16)
    hv, wv = hbig[:, :, K:], wbig[:, 8:8 + K]
    ref = oracle.lm_head_confidence(hv.contiguous(), wv.contiguous(), return_logits=True)
    got = _run(lsp, hbig.cuda()[:, :, K:], wbig.cuda()[:, 8:8 + K])
    _compare(got, ref[:3], ref[3])


def test_c2_shape_sampled_rows(lsp, oracle):
    """Full config-2 shape (256 rows, K = 4096, V = 126464) in the launch shape the
    benchmark times; the oracle evaluates a sample of rows."""
    w = W.C2
    hidden, weight, info = W.make_lm_head(w, 4096, device="cuda")
    got = _run(lsp, hidden, weight)
    rows = torch.tensor([0, 1, 37, 100, 128, 200, 255])
    ref = oracle.lm_head_confidence(hidden[:, rows].cpu(), weight.cpu(), return_logits=True)
    sub = tuple(t[:, rows] for t in got)
    _compare(sub, ref[:3], ref[3])
    # planted ids of the strongly boosted early rows come out (a property that holds at any size)
    assert torch.equal(got[0][0, :32].long(), info["planted_id"][0, :32].cpu())


def test_c4_shape_sampled_rows_and_tile_invariants(lsp, oracle):
    """Config-4 rows (8 x 1024) in the launch shape the benchmark times (four-wave
    tiles, 32 row tiles): the oracle evaluates sampled rows from first, middle and
    last row tiles; every row must also satisfy what holds at any size."""
    w = W.C4
    hidden, weight, info = W.make_lm_head(w, 4096, device="cuda")
    sl = torch.tensor([1024, 1000, 1, 0, 512, 1024, 257, 1024], dtype=torch.int32)
    got = _run(lsp, hidden, weight, sl)
    ids, p, m = got
    act = torch.arange(w.S).view(1, -1) < sl.view(-1, 1)
    assert torch.all(ids[~act] == -7) and torch.all(m[~act] == -7.0)
    assert ((ids[act] >= 0) & (ids[act] < w.V)).all() and (m[act] >= 0).all()
    assert ((p[act] > 0) & (p[act] <= 1.0 + 1e-6)).all()
    # a probability above one half needs a positive margin: exp(-margin) <= (1 - p) / p
    assert (torch.exp(-m[act].double()) <= (1 - p[act].double()) / p[act].double() + 1e-4).all()
    weight_cpu = weight.cpu()
    for b, rows in ((0, [0, 255, 256, 1023]), (2, [0]), (6, [100, 256])):
        r = torch.tensor(rows)
        ref = oracle.lm_head_confidence(hidden[b:b + 1, r].cpu(), weight_cpu, return_logits=True)
        _compare(tuple(t[b:b + 1, r] for t in got), ref[:3], ref[3])

"""GPU parity on tensors of more than 2**31 elements (more than 2**32 bytes): the shapes a
288 GB device holds once the batch or the cache grows past the workload sizes.  Element
and byte offsets of the later sequences no longer fit 32 bits, so any index arithmetic
done in int would read or write the wrong rows: sampled outputs are compared with the
oracle, and the structure planted by the input generator is checked on every row."""
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


def test_confidence_on_logits_beyond_2_31_elements(lsp, oracle):
    """20 x 1024 x 126464 bf16 logits (2.59e9 elements, 5.2 GB).  Eq. 1 on rows at both ends,
    on the rows either side of the 2**31-element and 2**32-byte marks, and on a seeded sample."""
    w = W.scaled(W.C4, B=20)
    z, info = W.make_logits(w, device="cuda")
    assert z.numel() > 2**31
    ids, p, m = lsp.confidence(z)
    torch.cuda.synchronize()
    R = w.B * w.S
    marks = [2**31 // w.V, 2**32 // (2 * w.V), 2**32 // w.V]
    g = torch.Generator().manual_seed(11)
    rows = torch.cat([torch.tensor([0, R - 1] + [r + d for r in marks for d in (-1, 0, 1) if r + d < R]),
                      torch.randint(R // 2, R, (100,), generator=g)])
    zs = z.view(-1, w.V)[rows.cuda()].cpu().unsqueeze(0)
    ids_r, p_r, m_r = oracle.confidence(zs)
    assert torch.equal(ids.view(-1)[rows.cuda()].cpu(), ids_r[0])
    assert torch.equal(m.view(-1)[rows.cuda()].cpu(), m_r[0])
    assert (p.view(-1)[rows.cuda()].cpu() - p_r[0]).abs().max().item() <= 2e-2
    # every sequence, also those stored beyond the marks: the planted token wins where the boost is large
    assert torch.equal(ids[:, :32].long(), info["planted_id"][:, :32])
    assert torch.all(m >= 0) and torch.all(p <= 1.0 + 1e-6) and torch.all(p >= 1.0 / w.V)


def test_commit_appends_into_caches_beyond_2_31_elements(lsp, oracle):
    """One layer whose K and V cache hold 8 x 73728 x 32 x 128 bf16 (2.4e9 elements, 4.8 GB each), every
    sequence's prefix close to the end of its slab: boundaries, tokens, lengths and the WHOLE caches
    bit-exact against the oracle (a stray row anywhere in the 9.6 GB would show)."""
    B, S, C, Hkv, D, Vv = 8, 1024, 73728, 32, 128, 4096
    assert B * C * Hkv * D > 2**31
    w = W.scaled(W.C4, B=B, S=S, C=C, P=C - S, Hkv=Hkv, D=D, seed=77)
    src = W.make_layer_kv(W.scaled(w, C=1, P=1), 0)          # suffix K/V from the generator; the caches start at zero
    g = torch.Generator().manual_seed(3)
    margin = 1.0 + torch.rand((B, S), generator=g)
    firsts = [0, 1, 63, 500, 777, 1000, 1023, 1024]
    for b, f in enumerate(firsts):
        if f < S:
            margin[b, f] = 0.25
    ids = torch.randint(0, Vv, (B, S), generator=g, dtype=torch.int32)
    bm = torch.zeros(Vv // 32, dtype=torch.int32)             # no delimiters: the boundary is the first unstable row
    pl = torch.tensor([C - S - 3 * b for b in range(B)], dtype=torch.int32)
    sl = torch.full((B,), S, dtype=torch.int32)
    tokens = torch.full((B, C), -1, dtype=torch.int32)

    pl_r, sl_r, tok_r = pl.clone(), sl.clone(), tokens.clone()
    kc_r = torch.zeros((B, C, Hkv, D), dtype=torch.bfloat16)
    vc_r = torch.zeros((B, C, Hkv, D), dtype=torch.bfloat16)
    ref = oracle.commit(margin, ids, bm, Vv, 0.9, 0, 1, 0, pl_r, sl_r, tokens=tok_r,
                        k_suf=[src["k_suf"]], v_suf=[src["v_suf"]], k_cache=[kc_r], v_cache=[vc_r])
    assert ref["commit_len"].tolist() == [max(f, 1) for f in firsts]

    pl_g, sl_g, tok_g = pl.cuda(), sl.cuda(), tokens.cuda()
    kc_g = torch.zeros((B, C, Hkv, D), dtype=torch.bfloat16, device="cuda")
    vc_g = torch.zeros((B, C, Hkv, D), dtype=torch.bfloat16, device="cuda")
    table = lsp.LayerTable([src["k_suf"].cuda()], [src["v_suf"].cuda()], [kc_g], [vc_g])
    got = lsp.commit(margin.cuda(), ids.cuda(), bm.cuda(), Vv, 0.9, 0, 1, 0, pl_g, sl_g, tokens=tok_g, layers=table, C=C)
    torch.cuda.synchronize()
    for k in ("raw_boundary", "snapped_boundary", "commit_len", "status_flags", "stable_mask"):
        assert torch.equal(got[k].cpu(), ref[k]), k
    assert torch.equal(pl_g.cpu(), pl_r) and torch.equal(sl_g.cpu(), sl_r) and torch.equal(tok_g.cpu(), tok_r)
    for got_c, ref_c, name in ((kc_g, kc_r, "k_cache"), (vc_g, vc_r, "v_cache")):
        host = got_c.cpu()
        for b in range(B):                                    # sequence by sequence: a failure names its slab
            assert torch.equal(host[b].view(torch.int16), ref_c[b].view(torch.int16)), (name, b)
        del host


@pytest.mark.parametrize("S", [48, 300])
def test_attention_over_caches_beyond_2_31_elements(lsp, oracle, S):
    """17 sequences of 131072 cache rows x 8 KV heads x 128 (2.28e9 elements, 4.6 GB per cache tensor):
    the last sequences' keys start beyond the 2**31-element mark.  S = 48 takes the short-suffix launch,
    S = 300 the long-suffix one.  Oracle on sampled (sequence, row, head) of the first and last sequences,
    each given to it as a batch of one."""
    B, C, Hkv, Hq, D = 17, 131072, 8, 16, 128
    assert B * C * Hkv * D > 2**31
    w = W.scaled(W.C2, B=B, S=S, P=C, C=C, Hq=Hq, Hkv=Hkv, D=D, seed=515)
    pl = torch.tensor([130000 - 4099 * b for b in range(B)], dtype=torch.int32)
    sl = torch.tensor([S - (b % 3) for b in range(B)], dtype=torch.int32)
    kv = W.make_layer_kv(w, 0, device="cuda", prefix_len=pl)
    out = torch.full((B, S, Hq, D), 123.0, dtype=torch.bfloat16, device="cuda")
    lsp.attn_step(kv["q"], kv["k_suf"], kv["v_suf"], kv["k_cache"], kv["v_cache"], pl.cuda(), sl.cuda(), out=out)
    torch.cuda.synchronize()
    worst = 0.0
    for b in (0, B - 2, B - 1):
        n = int(sl[b])
        one = {k: v[b:b + 1].cpu() for k, v in kv.items()}
        rows = torch.tensor([[0, i, h] for i in (0, n // 2, n - 1) for h in (0, 7, Hq - 1)], dtype=torch.int32)
        ref = oracle.attention(**one, prefix_len=pl[b:b + 1], suffix_len=sl[b:b + 1], rows=rows)
        sel = out[b, rows[:, 1].long().cuda(), rows[:, 2].long().cuda()].float().cpu()
        worst = max(worst, (sel - ref).abs().max().item())
        assert torch.all(out[b, n:].float() == 123.0) and not torch.isnan(out[b, :n].float()).any()
    assert worst <= 2e-2, worst

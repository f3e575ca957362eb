"""The whole step (lsp_attn_step, lsp_confidence, lsp_commit) captured in a HIP
graph, the way bench.py launches it: every replay - with eager work and
synchronisations between replays - must reproduce the eager result bit for bit."""
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


@pytest.mark.parametrize("cfg", ["split_rows", "many_rows", "long_suffix"])
def test_graph_replays_match_eager(lsp, cfg):
    if cfg == "split_rows":      # few rows: confidence splits rows over workgroups and uses its workspace
        w = W.scaled(W.C2, B=2, S=24, P=40, C=96, Hq=4, Hkv=2, D=128, V=70001, layers=2)
    elif cfg == "long_suffix":   # enough (sequence, head, row) triples for the long-suffix attention kernel
        w = W.scaled(W.C3, B=8, S=160, P=200, C=512, Hq=32, Hkv=8, D=128, V=4099, layers=2)
    else:
        w = W.scaled(W.C3, B=3, S=300, P=200, C=512, Hq=8, Hkv=2, D=128, V=4099, layers=2)
    dev = "cuda"
    _, bm = W.make_delimiters(w)
    bm = bm.to(dev)
    z, _ = W.make_logits(w, device=dev)
    layers = [W.make_layer_kv(w, l, device=dev) for l in range(w.layers)]
    cache0 = [(L["k_cache"].clone(), L["v_cache"].clone()) for L in layers]
    table = lsp.LayerTable([L["k_suf"] for L in layers], [L["v_suf"] for L in layers],
                           [L["k_cache"] for L in layers], [L["v_cache"] for L in layers])
    pl0, sl0 = (t.to(dev) for t in W.make_lengths(w, ragged=True))
    tok0 = W.make_tokens(w, w.C).to(dev)
    pl, sl, tok = pl0.clone(), sl0.clone(), tok0.clone()
    attn_out = [torch.zeros_like(L["q"]) for L in layers]
    conf = (torch.zeros((w.B, w.S), dtype=torch.int32, device=dev), torch.zeros((w.B, w.S), device=dev),
            torch.zeros((w.B, w.S), device=dev))
    ws = torch.empty(max(lsp.confidence_workspace_bytes(w.B, w.S, w.V), 256), dtype=torch.uint8, device=dev)
    out = lsp.commit(conf[2], conf[0], bm, w.V, w.tau, w.window, 1, 1, pl.clone(), sl.clone(), C=w.C)  # allocates the outputs

    def reset():
        pl.copy_(pl0); sl.copy_(sl0); tok.copy_(tok0)
        for L, (k, v) in zip(layers, cache0):
            L["k_cache"].copy_(k); L["v_cache"].copy_(v)
        for o in attn_out:
            o.zero_()
        for t in conf:
            t.zero_()
        for t in out.values():
            t.zero_()

    def step():
        for L, o in zip(layers, attn_out):
            lsp.attn_step(L["q"], L["k_suf"], L["v_suf"], L["k_cache"], L["v_cache"], pl, sl, out=o)
        lsp.confidence(z, sl, out=conf, workspace=ws)
        lsp.commit(conf[2], conf[0], bm, w.V, w.tau, w.window, 1, 1, pl, sl, tokens=tok, layers=table, out=out)

    def snapshot():
        torch.cuda.synchronize()
        items = [pl, sl, tok, *attn_out, conf[0], conf[2], *out.values()] + [L[n] for L in layers for n in ("k_cache", "v_cache")]
        snap = [t.clone() for t in items]
        return snap, conf[1].clone()

    reset()
    step()
    want, want_prob = snapshot()
    assert int(out["commit_len"].sum()) > 0

    reset()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph):
            step()
    torch.cuda.synchronize()
    for replay in range(4):
        reset()
        torch.cuda.synchronize()
        (z.float().sum() + replay).item()            # unrelated eager work and a sync between replays
        graph.replay()
        got, got_prob = snapshot()
        for i, (a, b) in enumerate(zip(got, want)):
            ab = a.view(torch.int16) if a.dtype == torch.bfloat16 else a
            bb = b.view(torch.int16) if b.dtype == torch.bfloat16 else b
            same = torch.equal(torch.nan_to_num(ab), torch.nan_to_num(bb)) if ab.dtype.is_floating_point else torch.equal(ab, bb)
            assert same, (replay, i)
        assert torch.equal(got_prob, want_prob), replay

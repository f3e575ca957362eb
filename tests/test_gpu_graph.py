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


@pytest.mark.parametrize("cfg", ["split_rows", "long_suffix"])
def test_graph_of_two_steps_with_the_one_launch_attention_and_the_allocation_free_confidence(lsp, cfg):
    """Two consecutive scheduler steps in ONE graph, launched the way a serving loop that cannot
    allocate would: lsp_attn_step_layers (all layers, one launch), lsp_confidence_static (its
    scratch lives in the library image), lsp_flip_update with the mid-stage window and the per-step
    trace, lsp_commit.  The second step sees the lengths, cache and previous ids the first one left.
    Every replay must reproduce the eager result bit for bit."""
    if cfg == "split_rows":
        w = W.scaled(W.C2, B=2, S=24, P=40, C=96, Hq=4, Hkv=2, D=128, V=70001, layers=3)
    else:
        w = W.scaled(W.C3, B=8, S=160, P=200, C=512, Hq=32, Hkv=8, D=128, V=4099, layers=2)
    dev = "cuda"
    _, bm = W.make_delimiters(w)
    bm = bm.to(dev)
    z = [W.make_logits(W.scaled(w, seed=w.seed + 7 * k), device=dev)[0] for k in range(2)]      # one logits tensor per step
    layers = [W.make_layer_kv(w, l, device=dev) for l in range(w.layers)]
    cache0 = [(L["k_cache"].clone(), L["v_cache"].clone()) for L in layers]
    table = lsp.LayerTable([L["k_suf"] for L in layers], [L["v_suf"] for L in layers],
                           [L["k_cache"] for L in layers], [L["v_cache"] for L in layers])
    attn_out = [[torch.zeros_like(L["q"]) for L in layers] for _ in range(2)]
    atab = [lsp.AttnLayerTable(*[[L[k] for L in layers] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")], attn_out[k])
            for k in range(2)]
    pl0, sl0 = (t.to(dev) for t in W.make_lengths(w, ragged=True))
    tok0 = W.make_tokens(w, w.C).to(dev)
    pl, sl, tok = pl0.clone(), sl0.clone(), tok0.clone()
    base = pl0.clone()
    G = w.S
    conf = [(torch.zeros((w.B, w.S), dtype=torch.int32, device=dev), torch.zeros((w.B, w.S), device=dev),
             torch.zeros((w.B, w.S), device=dev)) for _ in range(2)]
    last_id = torch.full((w.B, G), -1, dtype=torch.int32, device=dev)
    counters = torch.zeros(4, dtype=torch.int64, device=dev)
    trace = [torch.zeros((w.B, 2), dtype=torch.int32, device=dev) for _ in range(2)]
    outs = [lsp.commit(conf[0][2], conf[0][0], bm, w.V, w.tau, w.window, 1, 1, pl.clone(), sl.clone(), C=w.C) for _ in range(2)]

    def reset():
        pl.copy_(pl0); sl.copy_(sl0); tok.copy_(tok0)
        last_id.fill_(-1); counters.zero_()
        for L, (k, v) in zip(layers, cache0):
            L["k_cache"].copy_(k); L["v_cache"].copy_(v)
        for k in range(2):
            for o in attn_out[k]:
                o.zero_()
            for t in conf[k]:
                t.zero_()
            for t in outs[k].values():
                t.zero_()
            trace[k].zero_()

    def two_steps():
        for k in range(2):
            lsp.attn_step_layers(atab[k], pl, sl)
            lsp.confidence_static(z[k], sl, conf[k])
            lsp.flip_update(conf[k][0], pl, sl, base, last_id, counters, window=(0, G), step_counts=trace[k])
            lsp.commit(conf[k][2], conf[k][0], bm, w.V, w.tau, w.window, 1, 1, pl, sl, tokens=tok, layers=table, out=outs[k])

    def snapshot():
        torch.cuda.synchronize()
        items = [pl, sl, tok, last_id, counters, *trace]
        for k in range(2):
            items += [*attn_out[k], conf[k][0], conf[k][1], conf[k][2], *outs[k].values()]
        items += [L[n] for L in layers for n in ("k_cache", "v_cache")]
        return [t.clone() for t in items]

    reset()
    two_steps()
    want = snapshot()
    assert int(outs[0]["commit_len"].sum()) > 0 and int(counters[1]) > 0      # the second step compared positions

    reset()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(torch.cuda.Stream()):
        with torch.cuda.graph(graph):
            two_steps()
    torch.cuda.synchronize()
    for replay in range(3):
        reset()
        torch.cuda.synchronize()
        (z[0].float().sum() + replay).item()              # unrelated eager work and a sync between replays
        graph.replay()
        got = snapshot()
        for i, (a, b) in enumerate(zip(got, want)):
            ab = a.view(torch.int16) if a.dtype == torch.bfloat16 else a
            bb = b.view(torch.int16) if b.dtype == torch.bfloat16 else b
            same = torch.equal(torch.nan_to_num(ab), torch.nan_to_num(bb)) if ab.dtype.is_floating_point else torch.equal(ab, bb)
            assert same, (replay, i)

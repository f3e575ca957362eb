"""GPU parity: the whole step chained in a decode loop (Algorithm 1 lines 3-11)
against the oracle loop - steps, flips, tokens, lengths and cache contents
bit-exact; attention outputs to tolerance at sampled steps."""
import pytest
import torch

import workloads as W
from oracle.loop import decode_loop

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


KEYS = ("steps", "flips", "flip_denominator", "window_flips", "window_denominator", "committed")


def _same_counts(got, ref):
    """Step, flip and window counts of the two loops, and the per-step, per-sequence flip trace."""
    assert tuple(got[k] for k in KEYS) == tuple(ref[k] for k in KEYS), ([got[k] for k in KEYS], [ref[k] for k in KEYS])
    if "flip_trace" in got:
        want = torch.stack([torch.stack([f, d], 1) for f, d in ref["flip_trace"]]).to(torch.int32)
        assert torch.equal(got["flip_trace"], want)


@pytest.mark.parametrize("graph", [False, True])
@pytest.mark.parametrize("tau,Lmin,sizing", [(0.9, 1, {}), (float("inf"), 3, {}),
                                             (0.9, 1, dict(adaptive=True, alpha=0.25, beta=0.5)),
                                             (-float("inf"), 1, dict(max_commit=8))])
def test_small_loop_matches_oracle(lsp, oracle, tau, Lmin, sizing, graph):
    """graph=True: every step after the first is a replay of ONE captured HIP graph
    (with this loop's own eager work - the logits generator, the copy into the
    captured buffer, the termination poll - between the replays)."""
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    G = 96
    w = W.scaled(W.C5, B=3, S=G, V=4096, P=16, gen_len=G, C=16 + G, layers=2, Hq=2, Hkv=2, D=64)
    _, bm = W.make_delimiters(w)
    fn = lambda step, p: W.make_logits(w, step=step, prefix_len=p.cpu())[0]
    # oracle
    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, w.C)
    lay = [W.make_layer_kv(w, l) for l in range(2)]
    ref = decode_loop(fn, bm, w.V, tau, w.window, Lmin, 1, pl, sl, tokens, kv_layers=lay, commit_kw=sizing)
    # HIP
    pl_g, sl_g = (t.cuda() for t in W.make_lengths(w))
    tok_g = W.make_tokens(w, w.C).cuda()
    lay_g = [{k: v.cuda() for k, v in W.make_layer_kv(w, l).items()} for l in range(2)]
    got = gpu_loop(lambda s, p: fn(s, p).cuda(), bm.cuda(), w.V, tau, w.window, Lmin, 1, pl_g, sl_g, tok_g,
                   kv_layers=lay_g, gen_len=G, commit_kw=sizing, run_attention=graph, graph=graph, flip_trace=True)
    _same_counts(got, ref)
    assert torch.equal(tok_g.cpu(), tokens) and torch.equal(pl_g.cpu(), pl) and torch.equal(sl_g.cpu(), sl)
    for Lg, Lr in zip(lay_g, lay):
        assert torch.equal(Lg["k_cache"].cpu().view(torch.int16), Lr["k_cache"].view(torch.int16))
        assert torch.equal(Lg["v_cache"].cpu().view(torch.int16), Lr["v_cache"].view(torch.int16))


@pytest.mark.parametrize("graph", [False, True])
def test_loop_driven_by_the_fused_output_head(lsp, oracle, graph):
    """The loop with lsp_lm_head_confidence in the place of lsp_confidence: the
    step's input is a hidden state, the logits are never stored.  Small-integer
    operands make every logit exact in fp32, so the whole loop - ids, margins,
    boundaries, tokens, steps, flips - must match the oracle loop bit for bit
    (tied maxima, margin 0, occur in nearly every step)."""
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    G, K = 80, 64
    w = W.scaled(W.C5, B=3, S=G, V=1000, P=8, gen_len=G, C=8 + G, layers=1, Hq=2, Hkv=2, D=64)
    _, bm = W.make_delimiters(w)
    gw = torch.Generator().manual_seed(5)
    weight = torch.randint(-3, 4, (w.V, K), generator=gw).to(torch.bfloat16)

    def hidden_fn(step, p):
        g = torch.Generator().manual_seed(100 + step)
        return torch.randint(-3, 4, (w.B, w.S, K), generator=g).to(torch.bfloat16)

    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, w.C)
    ref = decode_loop(hidden_fn, bm, w.V, 0.5, w.window, 1, 1, pl, sl, tokens, lm_head_weight=weight)
    pl_g, sl_g = (t.cuda() for t in W.make_lengths(w))
    tok_g = W.make_tokens(w, w.C).cuda()
    got = gpu_loop(lambda s, p: hidden_fn(s, p).cuda(), bm.cuda(), w.V, 0.5, w.window, 1, 1, pl_g, sl_g, tok_g,
                   gen_len=G, lm_head_weight=weight.cuda(), graph=graph)
    _same_counts(got, ref)
    assert ref["steps"] > 3
    assert torch.equal(tok_g.cpu(), tokens) and torch.equal(pl_g.cpu(), pl) and torch.equal(sl_g.cpu(), sl)


def test_c5_full_size_first_steps_sampled(lsp, oracle):
    """Config 5 at its full shape (batch 16, 32 layers, 1024 active rows, vocab
    126464), first steps of the loop in the launch configuration bench.py uses.
    Per step: the boundary outputs of every sequence against the oracle's commit
    run on the step's (margin, id); sampled logits rows against the oracle's
    confidence; sampled attention rows of one layer; the appended cache rows of
    sampled layers equal the suffix rows they were copied from and the row after
    them is untouched."""
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    w = W.scaled(W.C5, layers=3)          # 3 of the 32 layers keep the test at a few GB
    dev = "cuda"
    _, bm = W.make_delimiters(w)
    layers = [W.make_layer_kv(w, l, device=dev) for l in range(w.layers)]
    pl, sl = (t.to(dev) for t in W.make_lengths(w))
    tokens = W.make_tokens(w, w.C).to(dev)
    fn = lambda step, p: W.make_process_logits(w, dev, step, p)[0]
    g = torch.Generator().manual_seed(11)
    seen = {"steps": 0, "total": torch.zeros(w.B, dtype=torch.int64)}

    def observer(step, z, conf, out):
        ids, prob, mar = (t.cpu() for t in conf)
        L = out["commit_len"].cpu()
        p_after, n_after = pl.cpu(), sl.cpu()
        p0, n0 = p_after - L, n_after + L
        # commit: oracle on the same (margin, id), state before the step
        pr, nr = p0.clone(), n0.clone()
        ref = oracle.commit(mar, ids, bm, w.V, w.tau, w.window, w.min_commit, 1, pr, nr, C=w.C)
        for k in ref:
            assert torch.equal(out[k].cpu(), ref[k]), (step, k)
        assert torch.equal(pr, p_after) and torch.equal(nr, n_after)
        # confidence: sampled active rows
        for _ in range(6):
            b = int(torch.randint(0, w.B, (1,), generator=g))
            if int(n0[b]) == 0:
                continue
            i = int(torch.randint(0, int(n0[b]), (1,), generator=g))
            ri, rp, rm = oracle.confidence(z[b, i].cpu().view(1, 1, -1))
            assert int(ri) == int(ids[b, i]) and float(rm) == float(mar[b, i]), (step, b, i)
            assert abs(float(rp) - float(prob[b, i])) <= 2e-2
        # append: committed rows of every layer equal the suffix rows; the next row is still poison
        for Lr in layers:
            for b in range(w.B):
                l = int(L[b])
                if l:
                    assert torch.equal(Lr["k_cache"][b, int(p0[b]): int(p_after[b])], Lr["k_suf"][b, :l])
                    assert torch.equal(Lr["v_cache"][b, int(p0[b]): int(p_after[b])], Lr["v_suf"][b, :l])
                if int(p_after[b]) < w.C:
                    assert torch.all(Lr["k_cache"][b, int(p_after[b])].float() == W.POISON_F32)
        seen["steps"] += 1
        seen["total"] += L.long()

    r = gpu_loop(fn, bm.to(dev), w.V, w.tau, w.window, w.min_commit, 1, pl, sl, tokens, kv_layers=layers,
                 gen_len=w.gen_len, run_attention=True, stop_after=6, observer=observer)
    assert r["steps"] == seen["steps"] == 6 and r["committed"] == int(seen["total"].sum())
    # attention at the state the loop stopped in: sampled rows of layer 1 against the oracle
    Lr = layers[1]
    out = lsp.attn_step(Lr["q"], Lr["k_suf"], Lr["v_suf"], Lr["k_cache"], Lr["v_cache"], pl, sl)
    torch.cuda.synchronize()
    plc, slc = pl.cpu(), sl.cpu()
    rows = []
    for _ in range(24):
        b = int(torch.randint(0, w.B, (1,), generator=g))
        rows.append([b, int(torch.randint(0, int(slc[b]), (1,), generator=g)), int(torch.randint(0, w.Hq, (1,), generator=g))])
    rows = torch.tensor(rows, dtype=torch.int32)
    ref = oracle.attention(**{k: v.cpu() for k, v in Lr.items()}, prefix_len=plc, suffix_len=slc, rows=rows)
    got = out[rows[:, 0].long().cuda(), rows[:, 1].long().cuda(), rows[:, 2].long().cuda()].float().cpu()
    assert (got - ref).abs().max().item() <= 2e-2


def _c5_loop_against_oracle(oracle, w, tau, sizing):
    """Config-5 loop to termination on both sides.  The step's logits come from the seeded
    process on the GPU for both (the generator is a function of step and prefix lengths
    only); the oracle loop receives its own state's logits as a host copy of the rows that
    are still active.  Everything the loop produces is compared bit for bit."""
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    dev = "cuda"
    _, bm = W.make_delimiters(w)
    G = w.gen_len
    # HIP
    lay_g = [W.make_layer_kv(w, l, device=dev) for l in range(w.layers)]
    pl_g, sl_g = (t.to(dev) for t in W.make_lengths(w))
    tok_g = W.make_tokens(w, w.C).to(dev)
    got = gpu_loop(lambda s, p: W.make_process_logits(w, dev, s, p)[0], bm.to(dev), w.V, tau, w.window, w.min_commit, 1,
                   pl_g, sl_g, tok_g, kv_layers=lay_g, gen_len=G, run_attention=True, commit_kw=sizing, flip_trace=True)
    torch.cuda.synchronize()
    # oracle, on host copies of the same operands
    lay = [{k: v.cpu() for k, v in W.make_layer_kv(w, l, device=dev).items() if k != "q"} for l in range(w.layers)]
    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, w.C)
    buf = torch.zeros((w.B, w.S, w.V), dtype=torch.bfloat16).pin_memory()

    def cpu_fn(step, p):
        z = W.make_process_logits(w, dev, step, p)[0]
        nmax = int((G - (p.long() - w.P)).max())          # rows at and beyond a sequence's remaining length are not read
        buf[:, :nmax].copy_(z[:, :nmax])
        return buf

    ref = decode_loop(cpu_fn, bm, w.V, tau, w.window, w.min_commit, 1, pl, sl, tokens, kv_layers=lay, commit_kw=sizing)
    _same_counts(got, ref)
    assert got["committed"] == w.B * G and torch.all(sl_g == 0)
    assert torch.equal(tok_g.cpu(), tokens) and torch.equal(pl_g.cpu(), pl) and torch.equal(sl_g.cpu(), sl)
    for Lg, Lr in zip(lay_g, lay):
        assert torch.equal(Lg["k_cache"].cpu().view(torch.int16), Lr["k_cache"].view(torch.int16))
        assert torch.equal(Lg["v_cache"].cpu().view(torch.int16), Lr["v_cache"].view(torch.int16))
    return got


@pytest.mark.timeout(300)
def test_c5_full_shape_adaptive_loop_to_termination(lsp, oracle):
    """Config 5 at its full shape (batch 16, 1024 generated positions, vocabulary 126464;
    2 of the 32 layers) with the adaptive threshold of Eq. 2, [alpha, beta] = [0.25, 0.5]:
    the whole loop (about 25 steps) against the oracle loop."""
    got = _c5_loop_against_oracle(oracle, W.scaled(W.C5, layers=2), W.C5.tau, dict(adaptive=True, alpha=0.25, beta=0.5))
    assert 15 <= got["steps"] <= 40


@pytest.mark.timeout(600)
def test_c5_fixed_threshold_loop_to_termination_two_sequences(lsp, oracle):
    """Config 5's fixed-threshold loop (tau = 0.9) to termination, several hundred steps,
    on two of its sixteen sequences at full vocabulary and generation length (the oracle
    reads every active logits row of every step: about 80 G elements)."""
    got = _c5_loop_against_oracle(oracle, W.scaled(W.C5, B=2, layers=2), W.C5.tau, {})
    assert got["steps"] > 200


@pytest.mark.parametrize("graph", [False, True])
@pytest.mark.parametrize("cut", [1, 4])
def test_stopped_and_resumed_loop_walks_like_an_uninterrupted_one(lsp, oracle, tmp_path, cut, graph):
    """Checkpoint and resume: the loop is stopped after `cut` steps, everything it owns
    (lengths, tokens, caches, and the flip bookkeeping it returns as "state") goes through
    a file on the host into NEW device tensors, and a second call continues from there.
    Steps, flip and window counts, tokens, lengths and caches must equal the oracle's
    single uninterrupted run; the two calls' flip traces, put end to end, its trace."""
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    G = 96
    w = W.scaled(W.C5, B=3, S=G, V=4096, P=16, gen_len=G, C=16 + G, layers=2, Hq=2, Hkv=2, D=64)
    _, bm = W.make_delimiters(w)
    fn = lambda step, p: W.make_logits(w, step=step, prefix_len=p.cpu())[0]
    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, w.C)
    lay = [W.make_layer_kv(w, l) for l in range(2)]
    ref = decode_loop(fn, bm, w.V, 0.9, w.window, 1, 1, pl, sl, tokens, kv_layers=lay)
    assert ref["steps"] > cut + 2

    pl_g, sl_g = (t.cuda() for t in W.make_lengths(w))
    tok_g = W.make_tokens(w, w.C).cuda()
    lay_g = [{k: v.cuda() for k, v in W.make_layer_kv(w, l).items()} for l in range(2)]
    kw = dict(kv_layers=lay_g, gen_len=G, run_attention=graph, graph=graph, flip_trace=True)
    part = gpu_loop(lambda s, p: fn(s, p).cuda(), bm.cuda(), w.V, 0.9, w.window, 1, 1, pl_g, sl_g, tok_g,
                    stop_after=cut, **kw)
    assert part["steps"] == cut and int(sl_g.max()) > 0
    torch.save(dict(pl=pl_g, sl=sl_g, tok=tok_g, lay=lay_g, state=part["state"]), tmp_path / "ckpt.pt")
    del pl_g, sl_g, tok_g, lay_g
    ck = torch.load(tmp_path / "ckpt.pt", map_location="cpu", weights_only=True)
    pl_g, sl_g, tok_g = ck["pl"].cuda(), ck["sl"].cuda(), ck["tok"].cuda()
    lay_g = [{k: v.cuda() for k, v in L.items()} for L in ck["lay"]]
    state = {k: (v.cuda() if torch.is_tensor(v) else v) for k, v in ck["state"].items()}
    kw["kv_layers"] = lay_g
    got = gpu_loop(lambda s, p: fn(s, p).cuda(), bm.cuda(), w.V, 0.9, w.window, 1, 1, pl_g, sl_g, tok_g,
                   state=state, **kw)
    got["flip_trace"] = torch.cat([part["flip_trace"], got["flip_trace"]])
    _same_counts(got, ref)
    assert torch.equal(tok_g.cpu(), tokens) and torch.equal(pl_g.cpu(), pl) and torch.equal(sl_g.cpu(), sl)
    for Lg, Lr in zip(lay_g, lay):
        assert torch.equal(Lg["k_cache"].cpu().view(torch.int16), Lr["k_cache"].view(torch.int16))
        assert torch.equal(Lg["v_cache"].cpu().view(torch.int16), Lr["v_cache"].view(torch.int16))


def test_state_of_another_batch_is_refused(lsp):
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    G = 32
    w = W.scaled(W.C5, B=2, S=G, V=512, P=4, gen_len=G, C=4 + G, layers=1, Hq=2, Hkv=2, D=64)
    _, bm = W.make_delimiters(w)
    pl_g, sl_g = (t.cuda() for t in W.make_lengths(w))
    tok_g = W.make_tokens(w, w.C).cuda()
    bad = dict(base=pl_g.clone(), last_id=torch.full((w.B, G + 1), -1, dtype=torch.int32, device="cuda"),
               counters=torch.zeros(4, dtype=torch.int64, device="cuda"), steps=0)
    with pytest.raises(lsp.LspError, match="state does not belong"):
        gpu_loop(lambda s, p: None, bm.cuda(), w.V, 0.9, w.window, 1, 1, pl_g, sl_g, tok_g, gen_len=G, state=bad)

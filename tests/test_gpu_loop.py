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


@pytest.mark.parametrize("tau,Lmin", [(0.9, 1), (float("inf"), 3)])
def test_small_loop_matches_oracle(lsp, oracle, tau, Lmin):
    from paper_2603_05454_amd.loop import decode_loop as gpu_loop
    G = 96
    w = W.scaled(W.C5, B=3, S=G, V=4096, P=16, gen_len=G, C=16 + G, layers=2, Hq=2, Hkv=2, D=64)
    _, bm = W.make_delimiters(w)
    fn = lambda step, p: W.make_logits(w, step=step, prefix_len=p.cpu())[0]
    # oracle
    pl, sl = W.make_lengths(w)
    tokens = W.make_tokens(w, w.C)
    lay = [W.make_layer_kv(w, l) for l in range(2)]
    ref = decode_loop(fn, bm, w.V, tau, w.window, Lmin, 1, pl, sl, tokens, kv_layers=lay)
    # HIP
    pl_g, sl_g = (t.cuda() for t in W.make_lengths(w))
    tok_g = W.make_tokens(w, w.C).cuda()
    lay_g = [{k: v.cuda() for k, v in W.make_layer_kv(w, l).items()} for l in range(2)]
    got = gpu_loop(lambda s, p: fn(s, p).cuda(), bm.cuda(), w.V, tau, w.window, Lmin, 1, pl_g, sl_g, tok_g,
                   kv_layers=lay_g, gen_len=G)
    assert (got["steps"], got["flips"], got["flip_denominator"], got["committed"]) == \
           (ref["steps"], ref["flips"], ref["flip_denominator"], ref["committed"])
    assert torch.equal(tok_g.cpu(), tokens) and torch.equal(pl_g.cpu(), pl) and torch.equal(sl_g.cpu(), sl)
    for Lg, Lr in zip(lay_g, lay):
        assert torch.equal(Lg["k_cache"].cpu().view(torch.int16), Lr["k_cache"].view(torch.int16))
        assert torch.equal(Lg["v_cache"].cpu().view(torch.int16), Lr["v_cache"].view(torch.int16))

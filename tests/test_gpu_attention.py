"""GPU parity: lsp_attn_step against the CPU oracle (Algorithm 1 line 4;
Section 3.2).  Max abs error <= 1e-5 (fp32) / 2e-2 (bf16)."""
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu
TOL = {"f32": 1e-5, "bf16": 2e-2}


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


def _run(lsp, kv, pl, sl, scale=0.0):
    g = {k: v.cuda() for k, v in kv.items()}
    out = torch.full(g["q"].shape, 123.0, dtype=g["q"].dtype, device="cuda")
    lsp.attn_step(g["q"], g["k_suf"], g["v_suf"], g["k_cache"], g["v_cache"], pl.cuda(), sl.cuda(),
                  scale=scale, out=out)
    torch.cuda.synchronize()
    return out.float().cpu()


def _check_full(lsp, oracle, w, pl, sl, scale=0.0, layer=0):
    kv = W.make_layer_kv(w, layer, prefix_len=pl)
    got = _run(lsp, kv, pl, sl, scale)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, scale=scale or None)
    act = ~torch.isnan(ref)
    err = (got[act] - ref[act]).abs().max().item() if act.any() else 0.0
    assert err <= TOL[w.dtype], err
    assert torch.all(got[~act] == 123.0)          # rows >= suffix_len untouched
    return err


def test_c1_tiny_fp32(lsp, oracle):
    pl, sl = W.make_lengths(W.C1)
    _check_full(lsp, oracle, W.C1, pl, sl)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (6, 2), (7, 1)])
def test_ragged_lengths_gqa(lsp, oracle, dtype, D, Hq, Hkv):
    """Per-sequence lengths as a decode loop leaves them: an empty suffix, an
    empty prefix, lengths that are not multiples of any tile."""
    w = W.scaled(W.C2, dtype=dtype, B=4, S=150, P=200, C=256, Hq=Hq, Hkv=Hkv, D=D, seed=7 + D + Hq)
    pl = torch.tensor([200, 0, 77, 131], dtype=torch.int32)
    sl = torch.tensor([150, 129, 0, 1], dtype=torch.int32)
    _check_full(lsp, oracle, w, pl, sl)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_key_and_tile_edges(lsp, oracle, dtype):
    w = W.scaled(W.C2, dtype=dtype, B=6, S=130, P=70, C=128, Hq=2, Hkv=2, D=128, seed=21)
    pl = torch.tensor([0, 63, 64, 65, 128, 0], dtype=torch.int32)
    sl = torch.tensor([1, 1, 64, 63, 128, 130], dtype=torch.int32)
    _check_full(lsp, oracle, w, pl, sl)


@pytest.mark.parametrize("dtype,B,Hq,S", [("f32", 2, 2, 150), ("bf16", 2, 2, 150), ("bf16", 8, 16, 320)])
def test_large_scores_and_moving_maximum(lsp, oracle, dtype, B, Hq, S):
    """Scores spanning hundreds of units whose maximum keeps rising along the key
    axis (the soft-max reference has to move again and again), rows where a single
    key takes all the weight, and rows whose large scores are all negative; at the
    short-suffix and at the long-suffix launch shape (one sequence there is short
    enough for the key-split mode)."""
    w = W.scaled(W.C2, dtype=dtype, B=B, S=S, P=200, C=256, Hq=Hq, Hkv=2, D=128, seed=91)
    pl = torch.full((B,), 200, dtype=torch.int32)
    sl = torch.full((B,), S, dtype=torch.int32)
    sl[-1] = 30
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    dt = kv["q"].dtype
    ramp = torch.linspace(0.2, 6.0, 200).view(1, 200, 1, 1)
    kv["k_cache"][:, :200] = (kv["k_cache"][:, :200].float() * ramp).to(dt)     # later keys score higher
    kv["k_suf"] = (kv["k_suf"].float() * 6.0).to(dt)
    kv["q"] = (kv["q"].float() * 3.0).to(dt)
    kv["q"][0, 5] = (-kv["k_suf"][0, 7, :1].float() * 2.0).expand(Hq, -1).to(dt)  # all large scores negative but one direction
    kv["q"][0, 6] = (kv["k_cache"][0, 150, :1].float() * 4.0).expand(Hq, -1).to(dt)  # one key takes everything
    got = _run(lsp, kv, pl, sl)
    rows = torch.tensor([[b, i, h] for b in range(B) for i in range(int(sl[b])) for h in (0, Hq - 1)
                         if i < 8 or i % 37 == 0 or i >= int(sl[b]) - 2], dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
    assert not torch.isnan(sel).any()
    # fp32: a score of magnitude ~300 summed over 128 products in fp32 is off by ~1e-5 of
    # itself, and that absolute error is the relative error of its exponential: 1e-4, not the
    # 1e-5 that holds for unit-scale scores.  bf16: the usual bound.
    err = (sel - ref).abs().max().item()
    assert err <= (1e-4 if dtype == "f32" else TOL[dtype]), err


def test_explicit_scale(lsp, oracle):
    w = W.scaled(W.C2, B=1, S=64, P=64, C=64, Hq=2, Hkv=1, D=128, seed=5)
    pl, sl = W.make_lengths(w)
    _check_full(lsp, oracle, w, pl, sl, scale=0.05)


def test_cache_rows_beyond_prefix_are_never_read(lsp):
    """Poison (and NaN) beyond prefix_len must not reach the output."""
    w = W.scaled(W.C2, B=2, S=96, P=100, C=256, Hq=2, Hkv=2, D=128, seed=9)
    pl = torch.tensor([100, 37], dtype=torch.int32)
    sl = torch.tensor([96, 50], dtype=torch.int32)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    a = _run(lsp, kv, pl, sl)
    kv["k_cache"][0, 100:] = float("nan")
    kv["v_cache"][1, 37:] = float("nan")
    kv["k_suf"][1, 50:] = float("nan")
    kv["v_suf"][1, 50:] = float("nan")
    b = _run(lsp, kv, pl, sl)
    assert torch.equal(a, b) and not torch.isnan(b).any()


def test_strided_views(lsp, oracle):
    """Q/K/V sliced out of a fused [B,S,3H,D] projection buffer."""
    w = W.scaled(W.C2, B=2, S=70, P=40, C=64, Hq=4, Hkv=4, D=128, seed=13)
    pl, sl = W.make_lengths(w)
    kv = W.make_layer_kv(w, 0)
    fused = torch.cat([kv["q"], kv["k_suf"], kv["v_suf"]], dim=2).cuda()
    q, k, v = fused[:, :, 0:4], fused[:, :, 4:8], fused[:, :, 8:12]
    out = lsp.attn_step(q, k, v, kv["k_cache"].cuda(), kv["v_cache"].cuda(), pl.cuda(), sl.cuda())
    torch.cuda.synchronize()
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl)
    assert (out.float().cpu() - ref).abs().max().item() <= 2e-2


def test_c2_full_size(lsp, oracle):
    pl, sl = W.make_lengths(W.C2)
    err = _check_full(lsp, oracle, W.C2, pl, sl)
    print("c2 attention max abs err", err)


def _sampled(lsp, oracle, w, n=96, seed=3, layer=0, heads=None, rows_per_head=0):
    kv = W.make_layer_kv(w, layer, device="cuda")
    pl, sl = W.make_lengths(w)
    out = lsp.attn_step(kv["q"], kv["k_suf"], kv["v_suf"], kv["k_cache"], kv["v_cache"], pl.cuda(), sl.cuda())
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(seed)
    if heads is None:
        rows = torch.stack([torch.randint(0, w.B, (n,), generator=g), torch.randint(0, w.S, (n,), generator=g),
                            torch.randint(0, w.Hq, (n,), generator=g)], dim=1).to(torch.int32)
    else:   # the named heads of every sequence, seeded rows of each (first and last row among them)
        rows = torch.tensor([[b, i, h] for b in range(w.B) for h in heads
                             for i in [0, w.S - 1] + torch.randint(0, w.S, (rows_per_head - 2,), generator=g).tolist()],
                            dtype=torch.int32)
    rows[0] = torch.tensor([0, 0, 0]); rows[1] = torch.tensor([w.B - 1, w.S - 1, w.Hq - 1])
    ref = oracle.attention(**{k: v.cpu() for k, v in kv.items()}, prefix_len=pl, suffix_len=sl, rows=rows)
    got = out[rows[:, 0].long().cuda(), rows[:, 1].long().cuda(), rows[:, 2].long().cuda()].float().cpu()
    err = (got - ref).abs().max().item()
    assert err <= 2e-2, err
    # property on every row: outputs are convex combinations of V rows
    vmax = max(kv["v_suf"].float().abs().max().item(), kv["v_cache"][:, : w.P].float().abs().max().item())
    assert out.float().abs().max().item() <= vmax and not torch.isnan(out.float()).any()
    return err


def test_c3_gqa_sampled(lsp, oracle):
    _sampled(lsp, oracle, W.C3)


def test_c4_shape_one_layer_sampled(lsp, oracle):
    _sampled(lsp, oracle, W.C4, n=64, layer=5)


@pytest.mark.parametrize("layer", [0, 15, 31])
def test_c4_shape_first_middle_last_layer_heads_0_13_31(lsp, oracle, layer):
    """Config 4's first, middle and last layer (their own seeded operands): heads 0, 13 and
    31 of every sequence, 12 seeded query rows each, all 5120 keys, against the oracle."""
    _sampled(lsp, oracle, W.C4, layer=layer, seed=40 + layer, heads=(0, 13, 31), rows_per_head=12)


@pytest.mark.parametrize("D,Hq,Hkv,S", [(128, 16, 4, 600), (64, 16, 16, 520), (128, 72, 8, 100)])
def test_many_rows_ragged_lengths_sampled(lsp, oracle, D, Hq, Hkv, S):
    """Enough (sequence, head, row) triples to take the long-suffix launch shape,
    with per-sequence lengths that end inside tiles: sampled rows against the
    oracle, every inactive row untouched."""
    w = W.scaled(W.C2, B=5, S=S, P=300, C=384, Hq=Hq, Hkv=Hkv, D=D, seed=31 + D + S)
    pl = torch.tensor([300, 0, 77, 131, 384], dtype=torch.int32)
    sl = torch.tensor([S, S - 71, 0, 1, 257 if S > 257 else S - 3], dtype=torch.int32)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    got = _run(lsp, kv, pl, sl)
    g = torch.Generator().manual_seed(5)
    rows = []
    for b in range(w.B):
        n = int(sl[b])
        if n == 0:
            continue
        ii = torch.randint(0, n, (24,), generator=g).tolist() + [0, n - 1]
        hh = torch.randint(0, Hq, (26,), generator=g).tolist()
        rows += [[b, i, h] for i, h in zip(ii, hh)]
    rows = torch.tensor(rows, dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
    err = (sel - ref).abs().max().item()
    assert err <= 2e-2, err
    for b in range(w.B):
        assert torch.all(got[b, int(sl[b]):] == 123.0)
        assert not torch.isnan(got[b, : int(sl[b])]).any()


def test_mixed_short_and_long_suffixes_in_one_call(lsp, oracle):
    """At the long-suffix launch shape the workgroups of a sequence whose suffix is
    down to a few rows switch to the key-split mode: lengths on both sides of that
    switch, in one call, sampled active rows against the oracle."""
    w = W.scaled(W.C2, B=8, S=320, P=200, C=256, Hq=16, Hkv=4, D=128, seed=77)
    pl = torch.tensor([200, 256, 0, 31, 200, 97, 256, 5], dtype=torch.int32)
    sl = torch.tensor([0, 1, 33, 64, 65, 32, 320, 31], dtype=torch.int32)    # the switch sits at 32 / 33 (contiguous cache)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    got = _run(lsp, kv, pl, sl)
    rows = torch.tensor([[b, i, h] for b in range(w.B) for i in range(int(sl[b])) for h in (0, 5, 15)
                         if i < 3 or i >= int(sl[b]) - 3 or i % 29 == 0], dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
    assert (sel - ref).abs().max().item() <= 2e-2
    for b in range(w.B):
        assert torch.all(got[b, int(sl[b]):] == 123.0)
        assert not torch.isnan(got[b, : int(sl[b])]).any()


@pytest.mark.parametrize("indexed", [False, True])
def test_long_suffix_key_block_counts(lsp, oracle, indexed):
    """Head_dim-128 long-suffix kernels (eight-stage ring; the hand-scheduled loop
    with a barrier every second key block for a contiguous cache, the compiler-
    scheduled one with a barrier every fourth for an indexed cache): per-sequence
    key counts from 3 to 15 blocks, i.e. fewer blocks than the prefetch depth,
    every remainder modulo the barrier period, ragged last blocks, and a
    cache/suffix boundary inside a block; with the cache addressed directly and
    through a shuffled row index."""
    w = W.scaled(W.C2, B=8, S=160, P=320, C=320, Hq=32, Hkv=8, D=128, seed=123)
    pl = torch.tensor([0, 1, 31, 33, 96, 100, 224, 320], dtype=torch.int32)
    sl = torch.tensor([160, 95, 129, 130, 97, 160, 65, 160], dtype=torch.int32)   # all above the key-split switch
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    g = {k: v.cuda() for k, v in kv.items()}
    index = None
    if indexed:
        gen = torch.Generator().manual_seed(5)
        index = torch.stack([torch.randperm(w.C, generator=gen) for _ in range(w.B)]).to(torch.int32)
        for name in ("k_cache", "v_cache"):
            sh = torch.full_like(kv[name], float("nan"))
            for b in range(w.B):
                sh[b][index[b, : int(pl[b])].long()] = kv[name][b, : int(pl[b])]
            g[name] = sh.cuda()
    out = torch.full(g["q"].shape, 123.0, dtype=g["q"].dtype, device="cuda")
    lsp.attn_step(g["q"], g["k_suf"], g["v_suf"], g["k_cache"], g["v_cache"], pl.cuda(), sl.cuda(), out=out,
                  cache_row_index=None if index is None else index.cuda())
    torch.cuda.synchronize()
    got = out.float().cpu()
    rows = torch.tensor([[b, i, h] for b in range(w.B) for i in range(int(sl[b])) for h in (0, 13, 31)
                         if i < 2 or i >= int(sl[b]) - 2 or i % 31 == 0], dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
    assert (sel - ref).abs().max().item() <= TOL["bf16"]
    for b in range(w.B):
        assert torch.all(got[b, int(sl[b]):] == 123.0)
        assert not torch.isnan(got[b, : int(sl[b])]).any()


@pytest.mark.parametrize("S,tail", [(160, 0), (160, 17), (192, 31)])
def test_long_suffix_every_cache_to_suffix_switch_position(lsp, oracle, S, tail):
    """The hand-scheduled loop steps from the cache stream to the suffix stream at a
    block index that differs per sequence: 0 to 19 full cache blocks (more than two
    turns of the eight-stage ring, both parities of the barrier period) followed by
    the suffix blocks, with and without ragged cache and suffix tails."""
    B = 20
    w = W.scaled(W.C2, B=B, S=S, P=640, C=640, Hq=16, Hkv=4, D=128, seed=500 + S + tail)
    pl = torch.tensor([32 * k + (tail if k % 3 else 0) for k in range(B)], dtype=torch.int32)
    sl = torch.tensor([S - (tail if k % 2 else 0) for k in range(B)], dtype=torch.int32)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    got = _run(lsp, kv, pl, sl)
    rows = torch.tensor([[b, i, h] for b in range(B) for i in (0, 1, 31, 32, 77, int(sl[b]) - 1) for h in (0, 9, 15)],
                        dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
    err = (sel - ref).abs().reshape(B, -1).max(dim=1).values
    assert err.max().item() <= TOL["bf16"], err
    for b in range(B):
        assert torch.all(got[b, int(sl[b]):] == 123.0)
        assert not torch.isnan(got[b, : int(sl[b])]).any()


def test_long_suffix_last_tile_with_one_to_eight_active_waves(lsp, oracle):
    """The last 256-query tile of a suffix that is not a multiple of 256 rows has waves with
    no active query; they run the loader-only loop next to waves that run the full one.
    Suffix lengths put 1..8 active waves into the last tile (a wave's 32 rows full, and cut
    short by 5), over key streams whose cache part ends on both barrier parities; every active
    row of every head is compared with the oracle, and rows beyond the suffix stay untouched."""
    lens = [256 + 32 * k - d for k in range(1, 9) for d in (0, 5)] + [65, 96, 97, 255]
    B = len(lens)
    w = W.scaled(W.C2, B=B, S=512, P=200, C=224, Hq=2, Hkv=1, D=128, seed=909)
    pl = torch.tensor([(200, 160, 131, 96)[b % 4] for b in range(B)], dtype=torch.int32)
    sl = torch.tensor(lens, dtype=torch.int32)
    _check_full(lsp, oracle, w, pl, sl)


def test_very_long_prefix(lsp, oracle):
    """131 000 cached keys per sequence (4 094 key blocks: hundreds of turns of the ring, block counters and
    stream pointers far beyond the workload sizes), ragged at both ends, one KV head shared by 64 query
    heads; sampled rows against the oracle."""
    w = W.scaled(W.C2, B=2, S=256, P=131072, C=131072, Hq=64, Hkv=1, D=128, seed=4242)
    pl = torch.tensor([131000, 65537], dtype=torch.int32)
    sl = torch.tensor([256, 201], dtype=torch.int32)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    got = _run(lsp, kv, pl, sl)
    rows = torch.tensor([[b, i, h] for b in range(2) for i in (0, 31, 100, int(sl[b]) - 1) for h in (0, 33, 63)], dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
    assert (sel - ref).abs().max().item() <= TOL["bf16"]
    assert torch.all(got[1, 201:] == 123.0) and not torch.isnan(got[0]).any() and not torch.isnan(got[1, :201]).any()


def test_strided_views_many_rows_sampled(lsp, oracle):
    """Q/K/V sliced out of one fused [B,S,Hq+2Hkv,D] buffer and a cache with padded
    rows, at a size that takes the long-suffix launch shape."""
    w = W.scaled(W.C2, B=2, S=520, P=300, C=384, Hq=32, Hkv=8, D=128, seed=17)
    pl = torch.tensor([300, 123], dtype=torch.int32)
    sl = torch.tensor([520, 407], dtype=torch.int32)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    fused = torch.cat([kv["q"], kv["k_suf"], kv["v_suf"]], dim=2).cuda()
    q, k, v = fused[:, :, :32], fused[:, :, 32:40], fused[:, :, 40:48]
    pad_k = torch.zeros((2, 384, 12, 128), dtype=torch.bfloat16, device="cuda")
    pad_v = torch.zeros_like(pad_k)
    pad_k[:, :, 2:10] = kv["k_cache"].cuda()
    pad_v[:, :, 2:10] = kv["v_cache"].cuda()
    out = torch.full((2, 520, 32, 128), 123.0, dtype=torch.bfloat16, device="cuda")
    lsp.attn_step(q, k, v, pad_k[:, :, 2:10], pad_v[:, :, 2:10], pl.cuda(), sl.cuda(), out=out)
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(6)
    rows = []
    for b in range(2):
        n = int(sl[b])
        rows += [[b, int(i), int(h)] for i, h in zip(torch.randint(0, n, (30,), generator=g), torch.randint(0, 32, (30,), generator=g))]
        rows += [[b, 0, 0], [b, n - 1, 31]]
    rows = torch.tensor(rows, dtype=torch.int32)
    ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
    got = out[rows[:, 0].long().cuda(), rows[:, 1].long().cuda(), rows[:, 2].long().cuda()].float().cpu()
    assert (got - ref).abs().max().item() <= 2e-2
    assert torch.all(out[1, 407:].float() == 123.0)


@pytest.mark.parametrize("cfg", ["f32_small", "bf16_short", "bf16_long_ragged", "bf16_d64"])
def test_all_layers_in_one_launch(lsp, oracle, cfg):
    """lsp_attn_step_layers over 3-5 layers with their own operands: every layer's output
    against the oracle, and bit-identical to lsp_attn_step called layer by layer wherever
    both take the same launch shape (one launch for all layers may pick a wider tile)."""
    w, pl, sl, nl = {
        "f32_small": (W.scaled(W.C1, B=2, S=40, P=30, C=64), torch.tensor([30, 7]), torch.tensor([40, 13]), 3),
        "bf16_short": (W.scaled(W.C2, B=2, S=96, P=100, C=128, Hq=4, Hkv=2), torch.tensor([100, 0]), torch.tensor([96, 33]), 4),
        "bf16_long_ragged": (W.scaled(W.C2, B=5, S=600, P=300, C=384, Hq=16, Hkv=4),
                             torch.tensor([300, 0, 77, 131, 384]), torch.tensor([600, 529, 0, 1, 257]), 3),
        "bf16_d64": (W.scaled(W.C2, B=3, S=520, P=64, C=128, Hq=16, Hkv=16, D=64), torch.tensor([64, 1, 128]), torch.tensor([520, 64, 300]), 5),
    }[cfg]
    pl, sl = pl.to(torch.int32), sl.to(torch.int32)
    host = [W.make_layer_kv(w, l, prefix_len=pl) for l in range(nl)]
    dev = [{k: v.cuda() for k, v in L.items()} for L in host]
    outs = [torch.full(L["q"].shape, 123.0, dtype=L["q"].dtype, device="cuda") for L in dev]
    table = lsp.AttnLayerTable(*[[L[k] for L in dev] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")], outs)
    lsp.attn_step_layers(table, pl.cuda(), sl.cuda())
    torch.cuda.synchronize()
    g = torch.Generator().manual_seed(3)
    for l, (L, o) in enumerate(zip(host, outs)):
        got = o.float().cpu()
        if w.B * w.S * w.Hq <= 40000:
            ref = oracle.attention(**L, prefix_len=pl, suffix_len=sl)
            act = ~torch.isnan(ref)
            assert (got[act] - ref[act]).abs().max().item() <= TOL[w.dtype], l
            assert torch.all(got[~act] == 123.0)
        else:
            rows = torch.tensor([[b, i, int(torch.randint(0, w.Hq, (1,), generator=g))] for b in range(w.B)
                                 for i in ([0, int(sl[b]) - 1] + torch.randint(0, max(int(sl[b]), 1), (14,), generator=g).tolist())
                                 if int(sl[b]) > 0], dtype=torch.int32)
            ref = oracle.attention(**L, prefix_len=pl, suffix_len=sl, rows=rows)
            assert (got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()] - ref).abs().max().item() <= TOL[w.dtype], l
            for b in range(w.B):
                assert torch.all(got[b, int(sl[b]):] == 123.0)
        single = _run(lsp, L, pl, sl)
        assert (single - got).abs().max().item() <= 2 * TOL[w.dtype]      # both are within TOL of the oracle


@pytest.mark.parametrize("S,Hq", [(40, 4), (160, 32)])
def test_more_layers_than_one_launch_holds(lsp, oracle, S, Hq):
    """35 layers: lsp_attn_step_layers issues them as a launch of 32 and a launch of 3 (the short-suffix
    kernel and the long-suffix kernel); every layer has its own operands, the first, the 32nd, the 33rd
    and the last are compared with the oracle, and every layer with the single-layer call."""
    nl = 35
    w = W.scaled(W.C2, B=8, S=S, P=96, C=128, Hq=Hq, Hkv=Hq // 2, D=128, seed=900 + S)
    pl = torch.tensor([96, 0, 31, 64, 128, 5, 96, 33], dtype=torch.int32)
    sl = torch.tensor([S, S - 7, 1, S, 0, S // 2, S, 9], dtype=torch.int32)
    host = [W.make_layer_kv(w, l, prefix_len=pl) for l in range(nl)]
    dev = [{k: v.cuda() for k, v in L.items()} for L in host]
    outs = [torch.full(L["q"].shape, 123.0, dtype=L["q"].dtype, device="cuda") for L in dev]
    table = lsp.AttnLayerTable(*[[L[k] for L in dev] for k in ("q", "k_suf", "v_suf", "k_cache", "v_cache")], outs)
    lsp.attn_step_layers(table, pl.cuda(), sl.cuda())
    torch.cuda.synchronize()
    rows = torch.tensor([[b, i, h] for b in range(w.B) for i in {0, int(sl[b]) // 2, int(sl[b]) - 1} if int(sl[b]) > 0
                         for h in (0, Hq - 1)], dtype=torch.int32)
    for l in range(nl):
        got = outs[l].float().cpu()
        single = _run(lsp, host[l], pl, sl)
        assert (single - got).abs().max().item() <= 2 * TOL["bf16"], l   # (one launch for all layers may pick another key split)
        if l in (0, 31, 32, nl - 1):
            ref = oracle.attention(**host[l], prefix_len=pl, suffix_len=sl, rows=rows)
            assert (got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()] - ref).abs().max().item() <= TOL["bf16"], l

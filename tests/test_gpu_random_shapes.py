"""GPU parity on seeded random shapes: every entry point against the CPU oracle
on a few hundred small problems whose sizes, lengths, strides and parameters are
drawn at random (Algorithm 1 lines 4-10; Eq. 1; Eq. 2; Section 4.3.3).  The fixed cases of the
other files aim at known edges; this file covers combinations nobody thought of.
All sizes stay inside the documented limits of the entry points.

Tolerances.  Attention: 2e-2 (bf16) / 1e-5 (fp32) on workload-scale inputs
(unit-variance q, k, v and the default scale).  Trials that multiply q or use a
larger scale have scores of magnitude 10-30; an fp32 score of magnitude s carries
an absolute error of about s * 1e-6, which is the RELATIVE error of its
exponential, and a bf16 probability that takes most of the weight multiplies
values of magnitude up to 4 with a relative rounding error of 2^-9: those trials
are held to 1e-4 / 4e-2.  Confidence and commit are exact except top1_prob."""
import random

import pytest
import torch

import workloads as W
import test_gpu_commit as tc
import test_gpu_lm_head as tl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


def _attention_trial(lsp, oracle, rng):
    dtype = rng.choice(["bf16", "bf16", "f32"])
    D = rng.choice([64, 128])
    Hkv = rng.choice([1, 2, 4, 8])
    Hq = Hkv * rng.choice([1, 2, 4, 7])
    if rng.random() < 0.35:  # enough (sequence, head, row) triples for the shared-tile kernels
        B, S = rng.choice([2, 4, 8]), rng.choice([129, 200, 256, 300, 513])
        Hq, Hkv = (32 if D == 128 else 16), rng.choice([4, 8])
    else:
        B, S = rng.randint(1, 5), rng.randint(1, 330)
    C = rng.choice([S, 64, 200, 512, 700])
    P = rng.randint(0, C)
    w = W.scaled(W.C2, dtype=dtype, B=B, S=S, P=P, C=C, Hq=Hq, Hkv=Hkv, D=D, seed=rng.randint(0, 10**6))
    pl = torch.tensor([rng.choice([0, P, rng.randint(0, C), C]) for _ in range(B)], dtype=torch.int32)
    sl = torch.tensor([rng.choice([0, 1, S, rng.randint(0, S), rng.randint(0, min(S, 70))]) for _ in range(B)],
                      dtype=torch.int32)
    scale = rng.choice([0.0, 0.0, 0.05, 0.3])
    qmul = rng.choice([1.0, 1.0, 1.0, 2.0, 4.0])
    case = f"attn {dtype} D={D} Hq={Hq} Hkv={Hkv} B={B} S={S} C={C} pl={pl.tolist()} sl={sl.tolist()} scale={scale} qmul={qmul}"
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    if qmul != 1.0:
        kv["q"] = (kv["q"].float() * qmul).to(kv["q"].dtype)
    g = {k: v.cuda() for k, v in kv.items()}
    out = torch.full(g["q"].shape, 123.0, dtype=g["q"].dtype, device="cuda")
    lsp.attn_step(g["q"], g["k_suf"], g["v_suf"], g["k_cache"], g["v_cache"], pl.cuda(), sl.cuda(), scale=scale, out=out)
    torch.cuda.synchronize()
    got = out.float().cpu()
    keys = int((pl + sl).max())
    work = sum(int(sl[b]) * (int(pl[b]) + int(sl[b])) for b in range(B)) * Hq * D
    if work > 2e8:  # the oracle evaluates a sample of (sequence, row, head) triples
        rows = [[b, i, h] for b in range(B) for i in range(int(sl[b])) for h in range(Hq)]
        rows = rng.sample(rows, min(len(rows), max(50, int(2e8 / (D * max(1, keys))))))
        for b in range(B):
            if int(sl[b]) > 0:
                rows += [[b, 0, 0], [b, int(sl[b]) - 1, Hq - 1]]
        rt = torch.tensor(rows, dtype=torch.int32)
        ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, scale=scale or None, rows=rt)
        err = (got[rt[:, 0].long(), rt[:, 1].long(), rt[:, 2].long()] - ref).abs().max().item()
    else:
        ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, scale=scale or None)
        act = ~torch.isnan(ref)
        err = (got[act] - ref[act]).abs().max().item() if act.any() else 0.0
        assert torch.all(got[~act] == 123.0), case  # rows >= suffix_len untouched
    plain = qmul == 1.0 and scale == 0.0
    tol = (2e-2 if dtype == "bf16" else 1e-5) if plain else (4e-2 if dtype == "bf16" else 1e-4)
    assert err <= tol, (case, err)


def _confidence_trial(lsp, oracle, rng):
    dtype = rng.choice([torch.bfloat16, torch.float32])
    B, S = rng.randint(1, 4), rng.choice([1, 3, 17, 64, 130, 300])
    V = rng.choice([2, 3, 7, 31, 33, 255, 1000, 4097, 32000, 50257, 126464, rng.randint(2, 70000)])
    if B * S * V > 2e7:
        S = max(1, int(2e7 / (B * V)))
    pad, off = rng.choice([0, 0, 1, 3, 8, 13]), rng.choice([0, 0, 1, 5])  # row stride > V, unaligned first element
    kind = rng.choice(["normal", "wide", "ties", "neginf"])
    case = f"conf {dtype} B={B} S={S} V={V} pad={pad} off={off} {kind}"
    g = torch.Generator().manual_seed(rng.randint(0, 10**6))
    z = torch.randn((B, S, V + pad + off), generator=g)
    if kind == "wide":
        z = z * rng.choice([10.0, 40.0])
    if kind == "ties":
        z = torch.round(z * 2) / 2
    if kind == "neginf":
        z[torch.rand((B, S, V + pad + off), generator=g) < 0.3] = -float("inf")
        z[..., off + rng.randrange(V)] = 1.0  # the row maximum stays finite
    z = z.to(dtype)
    sl = None
    if rng.random() < 0.5:
        sl = torch.tensor([rng.choice([0, S, rng.randint(0, S)]) for _ in range(B)], dtype=torch.int32)
    ref = oracle.confidence(z[..., off:off + V].contiguous(), suffix_len=sl)
    out = (torch.full((B, S), -7, dtype=torch.int32, device="cuda"), torch.full((B, S), -7.0, device="cuda"),
           torch.full((B, S), -7.0, device="cuda"))
    ids, p, m = lsp.confidence(z.cuda()[..., off:off + V], None if sl is None else sl.cuda(), out=out)
    torch.cuda.synchronize()
    ids, p, m = ids.cpu(), p.cpu(), m.cpu()
    act = ref[0] >= 0
    assert torch.equal(ids[act], ref[0][act]) and torch.equal(m[act], ref[2][act]), case
    if act.any():
        assert (p[act] - ref[1][act]).abs().max().item() <= (2e-2 if dtype == torch.bfloat16 else 1e-5), case
    assert torch.all(ids[~act] == -7) and torch.all(m[~act] == -7.0) and torch.all(p[~act] == -7.0), case


def _commit_trial(lsp, oracle, rng):
    B, S = rng.randint(1, 9), rng.choice([1, 5, 64, 65, 200, 256, 257, 700, 1024, 1500])
    Vv = rng.choice([64, 1000, 4096, 126464])
    g = torch.Generator().manual_seed(rng.randint(0, 10**6))
    p_unstable = rng.choice([0.0, 0.002, 0.02, 0.3])
    margin = torch.where(torch.rand((B, S), generator=g) < p_unstable, torch.rand((B, S), generator=g) * 0.9,
                         1.0 + torch.rand((B, S), generator=g) * 5)
    ids = torch.randint(0, Vv, (B, S), generator=g, dtype=torch.int32)
    nd = rng.choice([0, 1, Vv // 12, Vv // 3])
    bm = tc._bitmap(torch.randperm(Vv, generator=g)[:nd].tolist(), Vv)
    tau = rng.choice([0.9, 0.0, 2.5, float("inf"), -float("inf")])
    Wn, Lmin, snap = rng.choice([-1, 0, 1, 16, 100, 5000]), rng.choice([0, 1, 2, 50]), rng.choice([0, 1, 1])
    C = rng.choice([S, 2 * S + 10, 64])  # 64: most sequences overflow the cache (clamp + flag)
    pl = torch.tensor([rng.randint(0, C) for _ in range(B)], dtype=torch.int32)
    sl = torch.tensor([rng.choice([0, S, rng.randint(0, S)]) for _ in range(B)], dtype=torch.int32)
    tokens = torch.full((B, C), -1, dtype=torch.int32)
    sizing = {}
    if rng.random() < 0.4:
        a_ = rng.choice([0.01, 0.1, 0.25])
        sizing = dict(adaptive=1, alpha=a_, beta=max(a_, rng.choice([0.25, 0.5, 1.0])), max_commit=rng.choice([0, 0, 3, 100]))
    layers = None
    if rng.random() < 0.6:
        nl, Hkv, D = rng.choice([1, 2, 5]), rng.choice([1, 2, 8]), rng.choice([64, 128])
        dt = rng.choice([torch.bfloat16, torch.float32])
        layers = [dict(k_suf=torch.randn((B, S, Hkv, D), generator=g).to(dt), v_suf=torch.randn((B, S, Hkv, D), generator=g).to(dt),
                       k_cache=torch.randn((B, C, Hkv, D), generator=g).to(dt), v_cache=torch.randn((B, C, Hkv, D), generator=g).to(dt))
                  for _ in range(nl)]
    try:
        tc._both(lsp, oracle, margin, ids, bm, Vv, tau, Wn, Lmin, snap, pl, sl, tokens=tokens, layers=layers, C=C, **sizing)
    except AssertionError as e:
        raise AssertionError(f"commit B={B} S={S} V={Vv} nd={nd} tau={tau} W={Wn} Lmin={Lmin} snap={snap} C={C} "
                             f"pl={pl.tolist()} sl={sl.tolist()} sizing={sizing}: {e}") from e


def _lm_head_trial(lsp, oracle, rng):
    B, S = rng.randint(1, 3), rng.choice([1, 5, 64, 130, 257, 300])
    K, V = 8 * rng.randint(1, 40), rng.choice([2, 100, 256, 257, 513, 1031, 3000])
    w = W.scaled(W.C2, B=B, S=S, V=V, n_delim=min(64, max(1, V // 4)), seed=rng.randint(0, 10**6))
    hidden, weight, _ = W.make_lm_head(w, K)
    sl = None
    if rng.random() < 0.5:
        sl = torch.tensor([rng.choice([0, S, rng.randint(0, S)]) for _ in range(B)], dtype=torch.int32)
    ref = oracle.lm_head_confidence(hidden, weight, suffix_len=sl, return_logits=True)
    got = tl._run(lsp, hidden.cuda(), weight.cuda(), sl)
    if not (ref[0] >= 0).any():
        assert all(torch.all(t == -7) for t in got)
        return
    tl._compare(got, ref[:3], ref[3])


def _scattered_trial(lsp, oracle, rng):
    """Section 4.3.3's comparison pieces: top-k selection by margin, then the gathered append."""
    B, S = rng.randint(1, 9), rng.choice([1, 5, 64, 65, 257, 700, 1024, 2000])
    g = torch.Generator().manual_seed(rng.randint(0, 10**6))
    margin = torch.rand((B, S), generator=g)
    if rng.random() < 0.4:
        margin = (margin * rng.choice([2, 4, 16])).floor() / 16   # ties: the lower position wins
    sl = torch.tensor([rng.choice([0, 1, S, rng.randint(0, S)]) for _ in range(B)], dtype=torch.int32)
    ct = torch.tensor([rng.choice([0, 1, S, rng.randint(0, S)]) for _ in range(B)], dtype=torch.int32)
    case = f"scattered B={B} S={S} sl={sl.tolist()} ct={ct.tolist()}"
    ri, rm = oracle.select_scattered(margin, sl, ct)
    gi, gm = lsp.select_scattered(margin.cuda(), sl.cuda(), ct.cuda())
    torch.cuda.synchronize()
    assert torch.equal(gi.cpu(), ri) and torch.equal(gm.cpu(), rm), case
    if S > 300:
        return
    nl, Hkv, D = rng.choice([1, 3]), rng.choice([1, 2]), rng.choice([64, 128])
    dt = rng.choice([torch.bfloat16, torch.float32])
    C = rng.choice([S, S + 37, 64])
    pl = torch.tensor([rng.randint(0, C) for _ in range(B)], dtype=torch.int32)
    layers = [dict(k_suf=torch.randn((B, S, Hkv, D), generator=g).to(dt), v_suf=torch.randn((B, S, Hkv, D), generator=g).to(dt),
                   k_cache=torch.randn((B, C, Hkv, D), generator=g).to(dt), v_cache=torch.randn((B, C, Hkv, D), generator=g).to(dt))
              for _ in range(nl)]
    cnt = torch.minimum(ct, sl)
    ref = [{k: v.clone() for k, v in L.items()} for L in layers]
    pl_r = pl.clone()
    oracle.gather_append(ri, cnt, pl_r, [L["k_suf"] for L in ref], [L["v_suf"] for L in ref],
                         [L["k_cache"] for L in ref], [L["v_cache"] for L in ref])
    dev = [{k: v.cuda() for k, v in L.items()} for L in layers]
    table = lsp.LayerTable([L["k_suf"] for L in dev], [L["v_suf"] for L in dev], [L["k_cache"] for L in dev],
                           [L["v_cache"] for L in dev])
    pl_g = pl.cuda()
    app = lsp.kv_gather_append(gi, cnt.cuda(), pl_g, table)
    torch.cuda.synchronize()
    assert torch.equal(pl_g.cpu(), pl_r) and app.cpu().tolist() == (pl_r - pl).tolist(), case
    view = torch.int16 if dt == torch.bfloat16 else torch.int32
    for Lg, Lr in zip(dev, ref):
        for name in ("k_cache", "v_cache"):
            assert torch.equal(Lg[name].cpu().view(view), Lr[name].view(view)), (case, name)


def _long_suffix_trial(lsp, oracle, rng):
    """Shapes that take the long-suffix head_dim-128 kernels (the hand-scheduled loop for a contiguous
    cache, the compiler-scheduled ring for an indexed one): enough (sequence, head, row) triples, suffix
    buffers of more than 128 rows, per-sequence lengths that are full, ragged, a multiple of 32, below
    the key-split switch, or zero."""
    Hkv = rng.choice([1, 2, 4, 8])
    Hq = Hkv * rng.choice([1, 2, 4, 7])
    S = rng.choice([129, 160, 200, 256, 257, 300, 384, 511, 640])
    B = max(1, -(-32768 // (Hq * S))) + rng.randint(0, 2)
    C = rng.choice([64, 200, 512, 700, 1300])
    w = W.scaled(W.C2, dtype="bf16", B=B, S=S, P=C, C=C, Hq=Hq, Hkv=Hkv, D=128, seed=rng.randint(0, 10**6))
    pl = torch.tensor([rng.choice([0, C, rng.randint(0, C), 32 * rng.randint(0, C // 32), 31, 33]) for _ in range(B)],
                      dtype=torch.int32).clamp(max=C)
    sl = torch.tensor([rng.choice([S, S, rng.randint(0, S), 32 * rng.randint(0, S // 32), rng.randint(0, 70), 0, 1, 64, 65])
                       for _ in range(B)], dtype=torch.int32).clamp(max=S)
    kv = W.make_layer_kv(w, 0, prefix_len=pl)
    g = {k: v.cuda() for k, v in kv.items()}
    index = None
    if rng.random() < 0.25:
        gen = torch.Generator().manual_seed(rng.randint(0, 10**6))
        index = torch.stack([torch.randperm(C, generator=gen) for _ in range(B)]).to(torch.int32)
        for name in ("k_cache", "v_cache"):
            sh = torch.full_like(kv[name], float("nan"))
            for b in range(B):
                sh[b][index[b, : int(pl[b])].long()] = kv[name][b, : int(pl[b])]
            g[name] = sh.cuda()
    out = torch.full(g["q"].shape, 123.0, dtype=g["q"].dtype, device="cuda")
    lsp.attn_step(g["q"], g["k_suf"], g["v_suf"], g["k_cache"], g["v_cache"], pl.cuda(), sl.cuda(), out=out,
                  cache_row_index=None if index is None else index.cuda())
    torch.cuda.synchronize()
    got = out.float().cpu()
    case = dict(B=B, S=S, C=C, Hq=Hq, Hkv=Hkv, pl=pl.tolist(), sl=sl.tolist(), indexed=index is not None)
    rows = []
    for b in range(B):
        n = int(sl[b])
        if n:
            rows += [[b, i, rng.randint(0, Hq - 1)] for i in {0, n - 1, n // 2} | {rng.randint(0, n - 1) for _ in range(5)}]
    if rows:
        rows = torch.tensor(rows, dtype=torch.int32)
        ref = oracle.attention(**kv, prefix_len=pl, suffix_len=sl, rows=rows)
        sel = got[rows[:, 0].long(), rows[:, 1].long(), rows[:, 2].long()]
        assert (sel - ref).abs().max().item() <= 2e-2, case
    for b in range(B):
        assert torch.all(got[b, int(sl[b]):] == 123.0), case
        assert not torch.isnan(got[b, : int(sl[b])]).any(), case


TRIALS = {"attention": (_attention_trial, 150), "long_suffix": (_long_suffix_trial, 60), "confidence": (_confidence_trial, 150),
          "commit": (_commit_trial, 150), "lm_head": (_lm_head_trial, 60), "scattered": (_scattered_trial, 100)}


@pytest.mark.parametrize("name", list(TRIALS))
def test_random_shapes(lsp, oracle, name):
    trial, count = TRIALS[name]
    rng = random.Random(f"lsp-{name}")
    for _ in range(count):
        trial(lsp, oracle, rng)

"""Pins for the attention oracle (Algorithm 1 line 4; Section 3.2): library
routine on the fresh-cache identity, closed forms, GQA reduction, brute force."""
import math

import pytest
import torch

import workloads as W


def _mk(B=2, S=5, Hq=4, Hkv=2, D=8, P=7, C=12, dtype=torch.float32, seed=0):
    g = torch.Generator().manual_seed(seed)
    r = lambda *s: torch.randn(*s, generator=g).to(dtype)
    return dict(q=r(B, S, Hq, D), k_suf=r(B, S, Hkv, D), v_suf=r(B, S, Hkv, D),
                k_cache=r(B, C, Hkv, D), v_cache=r(B, C, Hkv, D))


def _full_recompute(t, pl, sl, scale=None):
    """Fresh-cache identity: run ordinary bidirectional self-attention with every
    one of the P+N rows as key/value (library SDPA, fp64), queries = suffix rows."""
    B, S, Hq, D = t["q"].shape
    Hkv = t["k_suf"].shape[2]
    out = torch.full((B, S, Hq, D), float("nan"), dtype=torch.float64)
    for b in range(B):
        P, N = int(pl[b]), int(sl[b])
        if N == 0:
            continue
        k = torch.cat([t["k_cache"][b, :P], t["k_suf"][b, :N]]).double()   # [T,Hkv,D]
        v = torch.cat([t["v_cache"][b, :P], t["v_suf"][b, :N]]).double()
        k = k.repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)        # [Hq,T,D]
        v = v.repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
        q = t["q"][b, :N].double().permute(1, 0, 2)                         # [Hq,N,D]
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, scale=scale)
        out[b, :N] = o.permute(1, 0, 2)
    return out


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (6, 1)])
def test_matches_library_full_recompute(oracle, dtype, Hq, Hkv):
    t = _mk(Hq=Hq, Hkv=Hkv, dtype=dtype, seed=3)
    pl = torch.tensor([7, 0], dtype=torch.int32)
    sl = torch.tensor([5, 3], dtype=torch.int32)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    ref = _full_recompute(t, pl, sl)
    act = ~torch.isnan(ref)
    assert torch.equal(torch.isnan(got), ~act)          # inactive rows untouched
    assert torch.allclose(got[act].double(), ref[act], atol=1e-6, rtol=1e-6)


def test_scale_argument(oracle):
    t = _mk(seed=5)
    pl = torch.tensor([4, 6], dtype=torch.int32)
    sl = torch.tensor([5, 5], dtype=torch.int32)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl, scale=0.37)
    ref = _full_recompute(t, pl, sl, scale=0.37)
    assert torch.allclose(got.double(), ref, atol=1e-6)


def test_zero_query_gives_mean_of_values(oracle):
    t = _mk(seed=1)
    t["q"].zero_()
    pl = torch.tensor([7, 3], dtype=torch.int32)
    sl = torch.tensor([5, 2], dtype=torch.int32)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    for b in range(2):
        P, N = int(pl[b]), int(sl[b])
        vv = torch.cat([t["v_cache"][b, :P], t["v_suf"][b, :N]]).double().mean(0)  # [Hkv,D]
        for h in range(4):
            for i in range(N):
                assert torch.allclose(got[b, i, h].double(), vv[h // 2], atol=1e-6)


def test_identical_values_pass_through(oracle):
    t = _mk(seed=2)
    row = torch.arange(8, dtype=torch.float32)
    t["v_suf"][:] = row
    t["v_cache"][:] = row
    pl = torch.tensor([7, 7], dtype=torch.int32)
    sl = torch.tensor([5, 5], dtype=torch.int32)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    assert torch.allclose(got, row.expand_as(got), atol=1e-6)


def test_dominant_key_selects_its_value(oracle):
    """One key aligned with the query with a huge norm: soft-max collapses onto it.
    The key sits in the cache for b=0 and in the suffix for b=1, which also
    checks the order [cache rows, then suffix rows]."""
    t = _mk(B=2, Hq=2, Hkv=2, seed=4)
    t["q"][:] = 0
    t["q"][..., 0] = 1.0
    t["k_cache"][:] = 0
    t["k_suf"][:] = 0
    t["k_cache"][0, 3, :, 0] = 500.0
    t["k_suf"][1, 2, :, 0] = 500.0
    pl = torch.tensor([7, 7], dtype=torch.int32)
    sl = torch.tensor([5, 5], dtype=torch.int32)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    for h in range(2):
        for i in range(5):
            assert torch.allclose(got[0, i, h], t["v_cache"][0, 3, h], atol=1e-6)
            assert torch.allclose(got[1, i, h], t["v_suf"][1, 2, h], atol=1e-6)


def test_gqa_equals_mha_on_repeated_heads(oracle):
    t = _mk(Hq=6, Hkv=2, seed=6)
    pl = torch.tensor([7, 5], dtype=torch.int32)
    sl = torch.tensor([5, 4], dtype=torch.int32)
    a = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    t2 = dict(t)
    for k in ("k_suf", "v_suf", "k_cache", "v_cache"):
        t2[k] = t[k].repeat_interleave(3, dim=2).contiguous()
    b = oracle.attention(**t2, prefix_len=pl, suffix_len=sl)
    assert torch.equal(torch.nan_to_num(a, nan=7.0), torch.nan_to_num(b, nan=7.0))


def test_rows_beyond_prefix_len_in_cache_are_ignored(oracle):
    t = _mk(seed=8)
    pl = torch.tensor([4, 6], dtype=torch.int32)
    sl = torch.tensor([5, 5], dtype=torch.int32)
    a = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    t["k_cache"][0, 4:] = 99.0
    t["v_cache"][1, 6:] = -99.0
    b = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    assert torch.equal(a, b)


def test_brute_force_python_loops(oracle):
    """Element-by-element definition in pure Python on a tiny case."""
    t = _mk(B=1, S=3, Hq=2, Hkv=1, D=4, P=2, C=4, seed=9)
    pl = torch.tensor([2], dtype=torch.int32)
    sl = torch.tensor([3], dtype=torch.int32)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    sc = 1 / math.sqrt(4)
    for i in range(3):
        for h in range(2):
            keys = [t["k_cache"][0, r, 0] for r in range(2)] + [t["k_suf"][0, r, 0] for r in range(3)]
            vals = [t["v_cache"][0, r, 0] for r in range(2)] + [t["v_suf"][0, r, 0] for r in range(3)]
            s = [sc * sum(float(t["q"][0, i, h, d]) * float(k[d]) for d in range(4)) for k in keys]
            m = max(s)
            w = [math.exp(x - m) for x in s]
            for d in range(4):
                o = sum(wi * float(v[d]) for wi, v in zip(w, vals)) / sum(w)
                assert abs(float(got[0, i, h, d]) - o) < 1e-6


def test_sampled_rows_equal_full(oracle):
    t = _mk(seed=10, dtype=torch.bfloat16)
    pl = torch.tensor([7, 2], dtype=torch.int32)
    sl = torch.tensor([5, 4], dtype=torch.int32)
    full = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    rows = torch.tensor([[0, 0, 0], [0, 4, 3], [1, 3, 1], [1, 0, 2]], dtype=torch.int32)
    part = oracle.attention(**t, prefix_len=pl, suffix_len=sl, rows=rows)
    for r, (b, i, h) in enumerate(rows.tolist()):
        assert torch.equal(part[r], full[b, i, h])


def test_workload_c1_against_library(oracle):
    w = W.C1
    t = W.make_layer_kv(w, 0)
    pl, sl = W.make_lengths(w)
    got = oracle.attention(**t, prefix_len=pl, suffix_len=sl)
    ref = _full_recompute(t, pl, sl)
    assert torch.allclose(got.double(), ref, atol=2e-6)

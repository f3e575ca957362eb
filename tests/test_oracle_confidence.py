"""Pins for the confidence oracle (Eq. 1, Algorithm 1 line 5): closed forms,
library routines (sort, topk, logsumexp in fp64), inequalities, planted rows."""
import math

import pytest
import torch

import workloads as W


def test_constant_row(oracle):
    V = 37
    z = torch.full((1, 1, V), 1.25)
    ids, p, m = oracle.confidence(z)
    assert ids.item() == 0 and m.item() == 0.0
    assert abs(p.item() - 1.0 / V) < 1e-7


@pytest.mark.parametrize("a,k", [(3.0, 0), (5.5, 11), (0.25, 36)])
def test_single_spike(oracle, a, k):
    V = 37
    z = torch.zeros((1, 1, V))
    z[0, 0, k] = a
    ids, p, m = oracle.confidence(z)
    assert ids.item() == k
    assert m.item() == a
    assert abs(p.item() - math.exp(a) / (math.exp(a) + V - 1)) < 1e-7


def test_duplicate_maximum_lowest_index_zero_margin(oracle):
    z = torch.randn((1, 1, 50), generator=torch.Generator().manual_seed(0))
    z[0, 0, 31] = 9.0
    z[0, 0, 7] = 9.0
    ids, p, m = oracle.confidence(z)
    assert ids.item() == 7 and m.item() == 0.0


def test_negative_rows_and_minus_inf(oracle):
    z = torch.full((1, 2, 9), -float("inf"))
    z[0, 0, 4] = -3.0
    z[0, 0, 6] = -5.0
    z[0, 1, 8] = -1.0          # a single finite entry: z2 = -inf, margin = +inf, p1 = 1
    ids, p, m = oracle.confidence(z)
    assert ids.tolist() == [[4, 8]]
    assert m[0, 0].item() == 2.0 and math.isinf(m[0, 1].item())
    assert abs(p[0, 0].item() - 1 / (1 + math.exp(-2.0))) < 1e-7 and p[0, 1].item() == 1.0


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_against_library_sort_and_logsumexp(oracle, dtype):
    g = torch.Generator().manual_seed(11)
    z = (2.0 * torch.randn((3, 17, 1031), generator=g)).to(dtype)
    ids, p, m = oracle.confidence(z)
    zd = z.double()
    srt = zd.sort(dim=-1, descending=True, stable=True)
    # second order statistic counts duplicates: sorted[1]
    ref_m = (srt.values[..., 0].float() - srt.values[..., 1].float())
    assert torch.equal(m, ref_m)
    # lowest index among maxima
    is_max = zd == srt.values[..., :1]
    first = torch.where(is_max, torch.arange(1031).expand_as(zd), 10**9).amin(-1)
    assert torch.equal(ids.long(), first)
    ref_p = torch.exp(srt.values[..., 0] - torch.logsumexp(zd, -1))
    assert torch.allclose(p.double(), ref_p, atol=1e-7, rtol=1e-6)
    # topk agrees wherever the maximum is unique
    tk = torch.topk(zd, 2, dim=-1)
    uniq = tk.values[..., 0] > tk.values[..., 1]
    assert torch.equal(ids.long()[uniq], tk.indices[..., 0][uniq])


def test_bf16_ties_are_common_and_resolved_low(oracle):
    """bf16 N(0,1) rows of realistic width do tie at the maximum now and then;
    the id must be the first occurrence and the margin exactly 0 there."""
    g = torch.Generator().manual_seed(5)
    z = torch.randn((1, 64, 20000), generator=g).to(torch.bfloat16)
    ids, p, m = oracle.confidence(z)
    zf = z.float()
    mx = zf.amax(-1, keepdim=True)
    cnt = (zf == mx).sum(-1)
    assert (cnt > 1).any()                      # the case is really exercised
    assert torch.all(m[cnt > 1] == 0)
    first = torch.where(zf == mx, torch.arange(20000).expand_as(zf), 10**9).amin(-1)
    assert torch.equal(ids.long(), first)


def test_probability_bounds(oracle):
    g = torch.Generator().manual_seed(2)
    V = 513
    z = (3 * torch.randn((2, 9, V), generator=g))
    ids, p, m = oracle.confidence(z)
    assert torch.all(p <= 1.0) and torch.all(p >= 1.0 / V)
    lower = 1.0 / (1.0 + (V - 1) * torch.exp(-m.double()))
    assert torch.all(p.double() >= lower - 1e-9)


def test_suffix_len_skips_rows(oracle):
    z = torch.randn((2, 6, 40), generator=torch.Generator().manual_seed(3))
    sl = torch.tensor([4, 0], dtype=torch.int32)
    ids, p, m = oracle.confidence(z, sl)
    assert torch.all(ids[0, :4] >= 0) and torch.all(ids[0, 4:] == -1) and torch.all(ids[1] == -1)
    assert torch.isnan(m[1]).all() and not torch.isnan(m[0, :4]).any()


def test_planted_rows_process_workload(oracle):
    """The process workload fixes the background maximum at 4 and plants
    4 + |c| (rounded to bf16): id and margin are known by construction."""
    w = W.scaled(W.C5, B=2, S=24, V=4096, P=8, gen_len=24, layers=1)
    pl = torch.tensor([8, 8], dtype=torch.int32)
    z, info = W.make_logits(w, step=1, prefix_len=pl)
    ids, p, m = oracle.confidence(z)
    top = (4.0 + info["conf"].abs()).to(torch.bfloat16).float()
    want_m = top - 4.0
    assert torch.equal(m, want_m)
    nz = want_m > 0
    assert torch.equal(ids.long()[nz], info["planted_id"][nz])


def test_planted_decay_workload_c1(oracle):
    w = W.C1
    z, info = W.make_logits(w)
    ids, p, m = oracle.confidence(z)
    # early positions carry a boost of ~8 over a background maximum of ~3.3
    assert torch.equal(ids[0, :8].long(), info["planted_id"][0, :8])
    assert torch.all(m[0, :6] > 0.9)

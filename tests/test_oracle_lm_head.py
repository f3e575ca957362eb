"""Pins for the output-head oracle (Algorithm 1 lines 4-5: the denoiser's last
projection followed by Eq. 1): a hand-worked example, closed forms, exact
integer cases checked through the logits-based confidence oracle, and the
library's fp64 matmul / sort / logsumexp on random rectangular operands."""
import math

import numpy as np
import pytest
import torch

import workloads as W


def test_hand_worked(oracle):
    h = torch.tensor([[[1.0, 2.0]]])
    w = torch.tensor([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0], [-1.0, 0.5]])   # z = 1, 2, 3, 0
    ids, p, m, z = oracle.lm_head_confidence(h, w, return_logits=True)
    assert z.flatten().tolist() == [1.0, 2.0, 3.0, 0.0]
    assert ids.item() == 2 and m.item() == 1.0
    e = math.e
    assert abs(p.item() - e ** 3 / (e + e ** 2 + e ** 3 + 1.0)) < 1e-7


def test_two_entry_vocabulary_is_a_sigmoid_of_the_margin(oracle):
    g = torch.Generator().manual_seed(2)
    h = torch.randn((1, 33, 19), generator=g)
    w = torch.randn((2, 19), generator=g)
    ids, p, m = oracle.lm_head_confidence(h, w)
    z = h[0].double() @ w.double().T
    d = (z[:, 0] - z[:, 1])
    assert torch.equal(ids[0], (d < 0).to(torch.int32))
    assert torch.allclose(m[0].double(), d.abs(), rtol=1e-6, atol=1e-7)
    assert torch.allclose(p[0].double(), torch.sigmoid(d.abs()), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_selection_matrix_reads_hidden_entries(oracle, dtype):
    """weight rows that are scaled unit vectors make the logits a scaled,
    permuted copy of the hidden state: everything is exact."""
    g = torch.Generator().manual_seed(3)
    K = V = 48
    h = (torch.randint(-256, 257, (2, 5, K), generator=g).float() / 64.0).to(dtype)
    perm = torch.randperm(K, generator=g)
    c = torch.tensor([0.5, 1.0, 2.0])[torch.randint(0, 3, (V,), generator=g)]
    w = torch.zeros((V, K))
    w[torch.arange(V), perm] = c
    w = w.to(dtype)
    ids, p, m, z = oracle.lm_head_confidence(h, w, return_logits=True)
    z_ref = h.double()[..., perm] * c.double()
    assert torch.equal(z, z_ref)
    ids2, p2, m2 = oracle.confidence(z_ref.float())      # exact in fp32
    assert torch.equal(ids, ids2) and torch.equal(m, m2)
    assert torch.allclose(p, p2, rtol=1e-6, atol=0)


def test_small_integers_ties_and_lowest_index(oracle):
    """Integer operands: exact integer logits with many duplicated maxima."""
    g = torch.Generator().manual_seed(4)
    h = torch.randint(-2, 3, (3, 9, 7), generator=g).float()
    w = torch.randint(-2, 3, (61, 7), generator=g).float()
    ids, p, m, z = oracle.lm_head_confidence(h, w, return_logits=True)
    zi = torch.einsum("bsk,vk->bsv", h.long(), w.long())
    assert torch.equal(z, zi.double())
    ids2, p2, m2 = oracle.confidence(zi.float())
    assert torch.equal(ids, ids2) and torch.equal(m, m2)
    assert (m == 0).any() and (m > 0).any()              # both cases occur
    assert torch.allclose(p, p2, rtol=1e-6, atol=0)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_against_library_matmul_sort_logsumexp(oracle, dtype):
    """Rectangular operands (rows != K != V) so that a transposed or mis-strided
    operand cannot pass."""
    g = torch.Generator().manual_seed(5)
    B, S, K, V = 2, 13, 96, 517
    h = torch.randn((B, S, K), generator=g).to(dtype)
    w = (torch.randn((V, K), generator=g) / math.sqrt(K)).to(dtype)
    ids, p, m, z = oracle.lm_head_confidence(h, w, return_logits=True)
    z_ref = torch.from_numpy(np.matmul(h.double().numpy().reshape(B * S, K), w.double().numpy().T)).view(B, S, V)
    assert torch.allclose(z, z_ref, rtol=0, atol=1e-12)
    srt = z_ref.sort(dim=-1, descending=True)
    assert torch.equal(ids.long(), srt.indices[..., 0])
    assert torch.allclose(m.double(), srt.values[..., 0] - srt.values[..., 1], rtol=1e-6, atol=1e-7)
    p_ref = torch.exp(srt.values[..., 0] - torch.logsumexp(z_ref, dim=-1))
    assert torch.allclose(p.double(), p_ref, rtol=1e-6, atol=1e-9)


def test_inactive_rows_untouched(oracle):
    g = torch.Generator().manual_seed(6)
    h = torch.randn((2, 6, 8), generator=g)
    w = torch.randn((11, 8), generator=g)
    sl = torch.tensor([4, 0], dtype=torch.int32)
    ids, p, m = oracle.lm_head_confidence(h, w, suffix_len=sl)
    full = oracle.lm_head_confidence(h, w)
    assert torch.equal(ids[0, :4], full[0][0, :4]) and torch.equal(m[0, :4], full[2][0, :4])
    assert (ids[0, 4:] == -1).all() and (ids[1] == -1).all()
    assert torch.isnan(p[0, 4:]).all() and torch.isnan(m[1]).all()


def test_planted_rows_of_the_workload_generator(oracle):
    """The generator lifts the planted id's logit by the requested amount: early
    rows (large boost) must report the planted id with a margin near boost - 4."""
    w = W.scaled(W.C2, S=24, V=2048, boost=16.0, decay=128.0)
    hidden, weight, info = W.make_lm_head(w, K=128)
    ids, p, m = oracle.lm_head_confidence(hidden, weight)
    assert torch.equal(ids[0, :8].long(), info["planted_id"][0, :8])
    assert (m[0, :8] > 6.0).all() and (p[0, :8] > 0.9).all()

"""GPU checks of the two measurement helpers the benchmark calls (they are not part of the
scheduler step, but their figures are quoted next to it, so what they compute is pinned):
lsp_bench_read must fold every word of the buffer exactly once, lsp_bench_mfma must issue
exactly the stated number of matrix instructions."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lsp():
    import paper_2603_05454_amd as m
    assert torch.cuda.is_available()
    return m


@pytest.mark.parametrize("words,workgroups", [(4 * 512 * 7, 7), (4 * 3 * 2048 + 4 * 2048, 4), (4 * 5, 5), (1 << 20, 256)])
def test_bench_read_folds_every_word_once(lsp, words, workgroups):
    g = torch.Generator().manual_seed(words)
    host = torch.randint(-2**31, 2**31 - 1, (words,), generator=g, dtype=torch.int64).to(torch.int32)
    out = torch.zeros(workgroups, dtype=torch.int32, device="cuda")
    lsp.bench_read(host.cuda(), workgroups, out)
    seg = host.numpy().view(np.uint32).reshape(workgroups, -1)
    want = np.bitwise_xor.reduce(seg, axis=1)
    assert np.array_equal(out.cpu().numpy().view(np.uint32), want)
    # `out` is accumulated: a second call over the same buffer cancels it
    lsp.bench_read(host.cuda(), workgroups, out)
    assert int(out.abs().sum()) == 0


def test_bench_read_rejects_uneven_split(lsp):
    buf = torch.zeros(4 * 5 + 4, dtype=torch.int32, device="cuda")
    out = torch.zeros(5, dtype=torch.int32, device="cuda")
    with pytest.raises(lsp.LspError):
        lsp.bench_read(buf, 5, out)


@pytest.mark.parametrize("iters,workgroups", [(1, 1), (5, 3)])
def test_bench_mfma_issues_the_stated_number_of_products(lsp, iters, workgroups):
    """All operands 0.5: every 32x32x16 product adds 16 * 0.25 = 4 to each accumulator entry;
    8 products per iteration over 4 accumulators of 16 entries per lane -> the per-lane sum of
    all accumulator entries is iters * 8 * 16 * 4 (exact in fp32)."""
    ops = torch.full((lsp.MFMA_BENCH_OPERAND_BYTES // 2,), 0.5, dtype=torch.bfloat16, device="cuda")
    out = torch.full((workgroups * 512,), -1.0, dtype=torch.float32, device="cuda")
    lsp.bench_mfma(ops, iters, workgroups, out)
    assert torch.equal(out.cpu(), torch.full((workgroups * 512,), float(iters * 8 * 16 * 4)))
    assert lsp.MFMA_BENCH_FLOP_PER_WG_ITER == 8 * 8 * 2 * 32 * 32 * 16


def test_bench_mfma_rejects_short_operand_buffer(lsp):
    ops = torch.zeros(128, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(512, dtype=torch.float32, device="cuda")
    with pytest.raises(ValueError):
        lsp.bench_mfma(ops, 1, 1, out)

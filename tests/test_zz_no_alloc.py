"""GPU test of lsp_confidence_static, the allocation-free form of lsp_confidence
(the per-segment results of split rows go to a buffer inside the library's
device image instead of a caller's workspace).  Called through the C-ABI, two
calls in a row on the same GPU, the second with a smaller input, each checked
against lsp_confidence with a workspace (same kernels: ids and margins must be
bit-identical, probabilities within the parity tolerance) and against the CPU
oracle."""
import ctypes

import pytest
import torch

pytestmark = pytest.mark.gpu


def _call_static(L, z, sl, out):
    B, S, V = z.shape
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return L.lsp_confidence_static(1 if z.dtype == torch.bfloat16 else 0, ctypes.c_void_p(z.data_ptr()), B, S, V,
                                   ctypes.c_int64(z.stride(1)), ctypes.c_int64(z.stride(0)),
                                   ctypes.c_void_p(0 if sl is None else sl.data_ptr()),
                                   ctypes.c_void_p(out[0].data_ptr()), ctypes.c_void_p(out[1].data_ptr()),
                                   ctypes.c_void_p(out[2].data_ptr()), st)


def _call_workspace(L, z, sl, out, ws):
    B, S, V = z.shape
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return L.lsp_confidence(1 if z.dtype == torch.bfloat16 else 0, ctypes.c_void_p(z.data_ptr()), B, S, V,
                            ctypes.c_int64(z.stride(1)), ctypes.c_int64(z.stride(0)),
                            ctypes.c_void_p(0 if sl is None else sl.data_ptr()),
                            ctypes.c_void_p(out[0].data_ptr()), ctypes.c_void_p(out[1].data_ptr()),
                            ctypes.c_void_p(out[2].data_ptr()), ctypes.c_void_p(ws.data_ptr()),
                            ctypes.c_size_t(ws.numel()), st)


def _outs(B, S):
    return (torch.full((B, S), -7, dtype=torch.int32, device="cuda"),
            torch.full((B, S), -7.0, device="cuda"), torch.full((B, S), -7.0, device="cuda"))


def test_two_calls_in_a_row_second_smaller(oracle):
    import paper_2603_05454_amd as lsp
    assert torch.cuda.is_available()
    L = lsp.lib()
    assert L.lsp_confidence_static_scratch_bytes() == 65536
    g = torch.Generator().manual_seed(77)
    # first: 2 x 40 rows of 70 001 bf16 logits (rows split into segments: the scratch buffer is in use),
    # one sequence ragged; second: 1 x 5 rows of 33 333 fp32 logits (fewer rows, other split count)
    cases = [((2, 40, 70001), torch.bfloat16, torch.tensor([40, 23], dtype=torch.int32)),
             ((1, 5, 33333), torch.float32, None),
             ((3, 300, 4099), torch.bfloat16, torch.tensor([300, 0, 17], dtype=torch.int32))]   # unsplit rows
    used_scratch = 0
    # The first launch of a kernel makes the HIP runtime load its code (device memory of the
    # runtime's own); from the second pass over the cases on, free device memory must not move.
    for rep, (shape, dt, sl) in [(r, c) for r in range(2) for c in cases]:
        z = (2 * torch.randn(shape, generator=g)).to(dt)
        z[0, 1, 5] = z[0, 1, shape[2] - 3] = 11.0        # a tied maximum far apart: lowest index, margin 0
        zg = z.cuda()
        slg = None if sl is None else sl.cuda()
        need = L.lsp_confidence_workspace_bytes(*shape)
        used_scratch += need > 0
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
        a, b = _outs(shape[0], shape[1]), _outs(shape[0], shape[1])
        free0 = torch.cuda.mem_get_info()[0]
        assert _call_static(L, zg, slg, a) == 0, L.lsp_last_error()
        torch.cuda.synchronize()
        assert rep == 0 or torch.cuda.mem_get_info()[0] == free0      # nothing was allocated on the device
        assert _call_workspace(L, zg, slg, b, ws) == 0, L.lsp_last_error()
        torch.cuda.synchronize()
        for x, y in zip(a, b):
            assert torch.equal(x, y)                      # same kernels: bit-identical, untouched rows included
        ids_r, p_r, m_r = oracle.confidence(z, sl)
        act = ids_r >= 0
        assert torch.equal(a[0].cpu()[act], ids_r[act]) and torch.equal(a[2].cpu()[act], m_r[act])
        assert (a[1].cpu()[act] - p_r[act]).abs().max().item() <= (2e-2 if dt == torch.bfloat16 else 1e-5)
        assert torch.all(a[0].cpu()[~act] == -7)
    assert used_scratch >= 4


def test_bad_arguments_launch_nothing():
    import paper_2603_05454_amd as lsp
    L = lsp.lib()
    rc = L.lsp_confidence_static(7, None, 1, 1, 8, ctypes.c_int64(0), ctypes.c_int64(0), None, None, None, None, None)
    assert rc == -1 and b"dtype" in L.lsp_last_error()

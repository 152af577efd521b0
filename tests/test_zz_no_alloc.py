"""sale_select_static (the Selection-Pass on the library's static scratch, for callers that cannot allocate)
against sale_select, through the C ABI: two calls in a row, the second with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2505_24179_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


def _case(sale, w, block_k=64, flags=0):
    q, k, _ = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=block_k, flags=flags)
    qd, kd = q.unsqueeze(0).cuda(), k.unsqueeze(0).cuda()
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    return p, qd, kd, q4, k4, qs, ks, tau


def _both(sale, case):
    """-> (mask, counts, m, l) of sale_select with a caller workspace and of sale_select_static, raw C-ABI calls."""
    p, qd, kd, q4, k4, qs, ks, tau = case
    lib = sale.raw()
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    outs = []
    for static in (False, True):
        mask = torch.full((1, p.n_q_heads, p.n_q, p.words), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
        counts = torch.full((1, p.n_q_heads, p.n_q), -7, dtype=torch.int32, device="cuda")
        m = torch.full((1, p.n_q_heads, p.seq_len), float("nan"), dtype=torch.float32, device="cuda")
        l = torch.full_like(m, float("nan"))
        ptrs = [ctypes.c_void_p(t.data_ptr()) for t in (qd, kd, q4, k4, qs, ks, tau)]
        if static:
            rc = lib.sale_select_static(ctypes.byref(p.c()), *ptrs, 1, ctypes.c_void_p(mask.data_ptr()),
                                        ctypes.c_void_p(counts.data_ptr()), ctypes.c_void_p(m.data_ptr()),
                                        ctypes.c_void_p(l.data_ptr()), st)
        else:
            ws = torch.empty(sale.workspace_bytes(p, sale.WS_SELECT), dtype=torch.uint8, device="cuda")
            rc = lib.sale_select(ctypes.byref(p.c()), *ptrs, 1, ctypes.c_void_p(mask.data_ptr()),
                                 ctypes.c_void_p(counts.data_ptr()), ctypes.c_void_p(m.data_ptr()),
                                 ctypes.c_void_p(l.data_ptr()), ctypes.c_void_p(ws.data_ptr()), ws.numel(), st)
        assert rc == 0, (static, sale.status_string(rc))
        torch.cuda.synchronize()
        outs.append((mask, counts, m, l))
    return outs


def test_static_scratch_select_equals_workspace_select_twice_in_a_row(sale):
    """Integer and bit work: masks and counts bit-exact, statistics bit-exact too (same kernels, same order).
    The second call is smaller, so it runs on scratch that still holds the first call's thresholds and operands."""
    big = inputs.scaled(inputs.LLAMA_32K, 8192, 8, 2, "noalloc-8k")          # 19.7 MB of scratch
    small = inputs.scaled(inputs.LLAMA_32K, 1088, 4, 1, "noalloc-1k")        # 17 blocks: ragged last mask word
    for w, bk in ((big, 64), (small, 64), (small, 32)):
        case = _case(sale, w, block_k=bk)
        assert sale.workspace_bytes(case[0], sale.WS_SELECT) <= sale.SELECT_STATIC_MAX_BYTES
        (m0, c0, s0, l0), (m1, c1, s1, l1) = _both(sale, case)
        assert torch.equal(m0, m1) and torch.equal(c0, c1), w.name
        assert torch.equal(s0, s1) and torch.equal(l0, l1), w.name
        assert int(c0.min()) >= 1 and torch.isfinite(s0).all()
    # the binding's wrapper takes the same route
    p, qd, kd, q4, k4, qs, ks, tau = _case(sale, small)
    mask = torch.empty(1, p.n_q_heads, p.n_q, p.words, dtype=torch.int64, device="cuda")
    counts = torch.empty(1, p.n_q_heads, p.n_q, dtype=torch.int32, device="cuda")
    sale.select_static(p, qd, kd, q4, k4, qs, ks, tau, out=(mask, counts))
    ref_mask, ref_counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    torch.cuda.synchronize()
    assert torch.equal(mask, ref_mask) and torch.equal(counts, ref_counts)


def test_static_scratch_select_rejects_what_does_not_fit(sale):
    """A geometry whose scratch exceeds the static array is refused before anything is launched."""
    lib = sale.raw()
    p = sale.Params(1, 32, 8, 131072)
    assert sale.workspace_bytes(p, sale.WS_SELECT) > sale.SELECT_STATIC_MAX_BYTES
    f = ctypes.c_void_p(0x1000)        # never dereferenced
    assert lib.sale_select_static(ctypes.byref(p.c()), f, f, f, f, f, f, f, 1, f, f, None, None, None) == -4
    assert lib.sale_select_static(ctypes.byref(p.c()), f, f, f, f, f, f, None, 1, f, f, None, None, None) == -1

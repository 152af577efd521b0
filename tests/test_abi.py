"""The C-ABI library loads without a GPU, exports every function the header
declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sale.h")


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sale_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported(sale):
    names = _declared_functions()
    assert {"sale_quantize_qk", "sale_select", "sale_sparse_attn", "sale_dense_attn", "sale_calibrate_tau",
            "sale_qk_int4_products", "sale_attn_int8_operands", "sale_attn_fp8_operands", "sale_select_static",
            "sale_workspace_bytes", "sale_status_string"} <= set(names)
    lib = sale.raw()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in sale.h but not exported"
    assert set(sale.EXPORTED) == set(names)


def test_status_strings(sale):
    assert sale.status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -5):
        assert sale.status_string(s) not in ("ok", "unknown status")
    assert sale.status_string(-99) == "unknown status"


def test_workspace_sizes(sale):
    p = sale.Params(1, 32, 8, 131072)
    assert sale.workspace_bytes(p, sale.WS_SELECT) == 32 * 131072 * 4 + 8 * 131072 * 96
    kv = 2 * 8 * 131072 * 128 * 2                     # K', V' in operand order
    units = 32 * 2048
    fixed = kv + units * 4 * (1 + 1 + 32) + (128 << 10) + 64      # order, slot per row block, 32 window tables, head loads, counter
    assert sale.workspace_bytes(p, sale.WS_SPARSE_ATTN_MIN) == fixed
    assert sale.workspace_bytes(p, sale.WS_SPARSE_ATTN) == fixed + units * sale.PARKED_ROW_BYTES
    assert sale.PARKED_ROW_BYTES == 32768 + 1024
    assert sale.workspace_bytes(p, sale.WS_DENSE_ATTN) == kv      # the dense kernel parks nothing and needs no tables
    p8 = sale.Params(1, 32, 8, 131072, flags=sale.FLAG_ATTN_INT8_QK)
    assert sale.workspace_bytes(p8, sale.WS_DENSE_ATTN) > kv + (32 + 8) * 131072 * 128
    assert sale.workspace_bytes(sale.Params(1, 32, 8, 100), sale.WS_SELECT) == 0   # invalid geometry


def _call_quant(sale, p, fake=0x1000):
    f = ctypes.c_void_p(fake)
    return sale.raw().sale_quantize_qk(ctypes.byref(p.c()), f, f, f, f, f, f, None)


def test_argument_validation_launches_nothing(sale):
    lib = sale.raw()
    good = sale.Params(1, 4, 2, 256)
    f = ctypes.c_void_p(0x1000)   # never dereferenced: every call below fails validation first
    assert lib.sale_quantize_qk(ctypes.byref(good.c()), None, f, f, f, f, f, None) == -1
    assert lib.sale_quantize_qk(None, f, f, f, f, f, f, None) == -1
    assert _call_quant(sale, sale.Params(1, 4, 2, 250)) == -2          # N not a multiple of the block
    assert _call_quant(sale, sale.Params(0, 4, 2, 256)) == -2
    assert _call_quant(sale, sale.Params(1, 4, 3, 256)) == -2          # heads not divisible
    assert _call_quant(sale, sale.Params(1, 4, 2, 256, head_dim=64)) == -3
    assert _call_quant(sale, sale.Params(1, 4, 2, 256, block_q=16, block_k=16)) == -3
    assert _call_quant(sale, sale.Params(1, 4, 2, 256, flags=32)) == -3
    assert _call_quant(sale, sale.Params(1, 4, 2, 256, flags=16)) == -3           # FP8 second product without the 8-bit first
    assert _call_quant(sale, sale.Params(1, 4, 2, 256, block_k=32, flags=24)) == -3   # ... or on 32-key blocks
    # select: query blocks must be 64 rows, at most 4096 key blocks; workspace too small; bad tau_len
    sel = lib.sale_select
    p3232 = sale.Params(1, 4, 2, 256, block_q=32, block_k=32)
    assert sel(ctypes.byref(p3232.c()), f, f, f, f, f, f, f, 1, f, f, None, None, f, 1 << 30, None) == -3
    plong = sale.Params(1, 1, 1, 32 * 4096 + 64, block_k=32)
    assert sel(ctypes.byref(plong.c()), f, f, f, f, f, f, f, 1, f, f, None, None, f, 1 << 40, None) == -3
    assert sel(ctypes.byref(good.c()), f, f, f, f, f, f, f, 1, f, f, None, None, f, 16, None) == -4
    assert sel(ctypes.byref(good.c()), f, f, f, f, f, f, f, 1, f, f, None, None, None, 0, None) == -4
    assert sel(ctypes.byref(good.c()), f, f, f, f, f, f, f, 3, f, f, None, None, f, 1 << 30, None) == -2
    assert sel(ctypes.byref(good.c()), f, f, f, f, f, f, None, 1, f, f, None, None, f, 1 << 30, None) == -1
    # attention
    assert lib.sale_dense_attn(ctypes.byref(good.c()), f, f, None, f, None, f, 1 << 30, None) == -1
    assert lib.sale_dense_attn(ctypes.byref(good.c()), f, f, f, f, None, f, 16, None) == -4
    assert lib.sale_sparse_attn(ctypes.byref(good.c()), f, f, f, None, None, f, None, f, 1 << 30, None) == -1
    assert lib.sale_sparse_attn(ctypes.byref(good.c()), f, f, f, f, None, f, None, None, 0, None) == -4
    assert lib.sale_dense_attn(ctypes.byref(p3232.c()), f, f, f, f, None, f, 1 << 30, None) == -3
    assert lib.sale_sparse_attn(ctypes.byref(p3232.c()), f, f, f, f, None, f, None, f, 1 << 30, None) == -3
    too_long = sale.Params(1, 1, 1, 64 * 64 * 64 + 64)
    assert lib.sale_dense_attn(ctypes.byref(too_long.c()), f, f, f, f, None, f, 1 << 40, None) == -3
    # calibration
    cal = lib.sale_calibrate_tau
    cal.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_float, ctypes.c_float, ctypes.c_int32] + [ctypes.c_void_p] * 4 + \
        [ctypes.c_size_t, ctypes.c_void_p]
    gp = ctypes.byref(good.c())
    aligned = ctypes.c_void_p(0x10000)
    assert cal(gp, f, f, f, 0.008, 0.4, 6, None, None, None, aligned, 1 << 40, None) == -1
    assert cal(gp, f, f, f, 0.0, 0.4, 6, f, None, None, aligned, 1 << 40, None) == -2       # tau0 outside (0, 1)
    assert cal(gp, f, f, f, 0.008, -1.0, 6, f, None, None, aligned, 1 << 40, None) == -2
    assert cal(gp, f, f, f, 0.008, 0.4, 65, f, None, None, aligned, 1 << 40, None) == -2
    assert cal(gp, f, f, f, 0.008, 0.4, 6, f, None, None, aligned, 1024, None) == -4
    assert cal(gp, f, f, f, 0.008, 0.4, 6, f, None, None, ctypes.c_void_p(0x10010), 1 << 40, None) == -4   # not 256-aligned
    assert sale.workspace_bytes(good, sale.WS_CALIBRATE) > sale.workspace_bytes(good, sale.WS_SPARSE_ATTN)
    # parity hook range checks
    prod = lib.sale_qk_int4_products
    assert prod(ctypes.byref(good.c()), f, f, 4, 0, 0, 1, f, None) == -2
    assert prod(ctypes.byref(good.c()), f, f, 0, 4, 0, 1, f, None) == -2
    assert prod(ctypes.byref(good.c()), f, f, 0, 0, 2, 1, f, None) == -2
    assert prod(ctypes.byref(good.c()), f, f, 0, 0, 0, 5, f, None) == -2
    assert prod(ctypes.byref(good.c()), f, f, 0, 0, 1, 1, f, None) == 0    # empty range: nothing to do


def test_binding_rejects_wrong_tensors_on_the_host():
    """The binding checks device, dtype, contiguity and element count of every tensor before marshalling: the C
    ABI takes raw pointers of contiguous buffers, so a CPU tensor, a transposed view or a short buffer must not
    reach a kernel.  (Runs without a GPU: the checks come before any library call.)"""
    import torch
    sale = pytest.importorskip("paper_2505_24179_amd.sale")
    p = sale.Params(1, 2, 1, 128)
    q = torch.zeros(1, 2, 128, 128, dtype=torch.bfloat16)
    k = torch.zeros(1, 1, 128, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError, match="device tensor"):
        sale._expect("q", q, torch.bfloat16, q.numel())
    meta_q = torch.zeros(1, 128, 2, 128, dtype=torch.bfloat16, device="meta").transpose(1, 2)     # [B][N][H][d] viewed as [B][H][N][d]
    assert not meta_q.is_contiguous()

    class FakeCuda:          # what _expect looks at, with is_cuda forced on
        def __init__(self, t): self.t = t
        is_cuda = True
        dtype = property(lambda self: self.t.dtype)
        shape = property(lambda self: self.t.shape)
        def is_contiguous(self): return self.t.is_contiguous()
        def stride(self): return self.t.stride()
        def numel(self): return self.t.numel()
    with pytest.raises(ValueError, match="contiguous"):
        sale._expect("q", FakeCuda(meta_q), torch.bfloat16, q.numel())
    with pytest.raises(ValueError, match="dtype"):
        sale._expect("q", FakeCuda(q.float()), torch.bfloat16, q.numel())
    with pytest.raises(ValueError, match="elements"):
        sale._expect("k", FakeCuda(k), torch.bfloat16, q.numel())
    with pytest.raises(ValueError, match="None"):
        sale._expect("q", None, torch.bfloat16, 1)
    sale._expect("row_counts", None, torch.int32, 1, optional=True)
    sale._expect("q", FakeCuda(q), torch.bfloat16, q.numel())


def test_static_scratch_select_checks_before_touching_the_gpu(sale):
    import ctypes
    lib = sale.raw()
    f = ctypes.c_void_p(0x1000)        # never dereferenced
    too_big = sale.Params(1, 32, 8, 131072)
    assert sale.workspace_bytes(too_big, sale.WS_SELECT) > sale.SELECT_STATIC_MAX_BYTES
    assert lib.sale_select_static(ctypes.byref(too_big.c()), f, f, f, f, f, f, f, 1, f, f, None, None, None) == -4
    fits = sale.Params(1, 32, 8, 16384)
    assert sale.workspace_bytes(fits, sale.WS_SELECT) <= sale.SELECT_STATIC_MAX_BYTES
    assert lib.sale_select_static(ctypes.byref(fits.c()), f, f, f, f, f, f, None, 1, f, f, None, None, None) == -1
    assert lib.sale_select_static(ctypes.byref(fits.c()), f, f, f, f, f, f, f, 5, f, f, None, None, None) == -2
    bad = sale.Params(1, 32, 8, 16384, block_q=32)
    assert lib.sale_select_static(ctypes.byref(bad.c()), f, f, f, f, f, f, f, 1, f, f, None, None, None) == -3


def test_strides_are_validated(sale):
    """Strides are element counts of (batch, head, token): all zero = contiguous; otherwise non-negative multiples
    of 8 with rows at least head_dim apart and a head / batch stride wherever there is more than one."""
    import ctypes
    lib = sale.raw()
    f = ctypes.c_void_p(0x1000)        # never dereferenced
    good = sale.Params(2, 4, 2, 256)

    def call(**strides):
        cp = good.c()
        for name, val in strides.items():
            getattr(cp, name)[:] = val
        return lib.sale_dense_attn(ctypes.byref(cp), f, f, f, f, None, f, 16, None)

    assert call() == -4                                                  # valid geometry: fails on the tiny workspace only
    assert call(q_stride=[4 * 256 * 128, 128, 4 * 128]) == -4            # [B][N][H][d]
    assert call(o_stride=[4 * 256 * 160, 256 * 160, 160]) == -4          # padded rows
    assert call(q_stride=[4 * 256 * 128, 128, 4 * 128 + 4]) == -2        # not a multiple of 8 elements
    assert call(k_stride=[2 * 256 * 128, 256 * 128, 64]) == -2           # rows closer than head_dim
    assert call(v_stride=[2 * 256 * 128, 0, 128]) == -2                  # two KV heads on top of each other
    assert call(q_stride=[0, 256 * 128, 128]) == -2                      # two batch entries on top of each other
    assert call(q_stride=[-8, 256 * 128, 128]) == -2
    # the struct grew at the end: a caller that fills only the leading fields gets contiguous tensors
    assert ctypes.sizeof(good.c()) == 40 + 4 * 3 * 8 + 16      # (+ n_seqs and the offsets pointer)

"""Thin ctypes binding over libsale.so (the C ABI declared in include/sale.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch supplies device memory and the current stream.  Importing this
module fails loudly when the built library is missing; there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libsale.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python -m paper_2505_24179_amd.build` "
        "(there is no CPU or PyTorch fallback for the SALE kernels)")
_lib = ctypes.CDLL(_LIB_PATH)

OK = 0
FLAG_STATS_CAUSAL = 1
FLAG_SELECT_16BIT = 2
FLAG_SEGMENT_LOCAL = 4
FLAG_ATTN_INT8_QK = 8
FLAG_ATTN_FP8_PV = 16
WS_SELECT = 1
WS_SPARSE_ATTN = 2
WS_DENSE_ATTN = 3
WS_CALIBRATE = 4
WS_INT8_OPERANDS = 5
WS_FP8_OPERANDS = 6
WS_SPARSE_ATTN_MIN = 7
PARKED_ROW_BYTES = 33792      # one parking slot of sparse_attn's workspace (see include/sale.h)


class _Params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "batch", "n_q_heads", "n_kv_heads", "seq_len", "head_dim",
        "block_q", "block_k", "sink_blocks", "local_blocks")] + [("flags", ctypes.c_uint32)] + \
        [(n, ctypes.c_int64 * 3) for n in ("q_stride", "k_stride", "v_stride", "o_stride")] + \
        [("n_seqs", ctypes.c_int32), ("cu_seqlens", ctypes.POINTER(ctypes.c_int32))]


@dataclass(frozen=True)
class Params:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    seq_len: int
    head_dim: int = 128
    block_q: int = 64
    block_k: int = 64
    sink_blocks: int = 1
    local_blocks: int = 4
    flags: int = 0
    cu_seqlens: tuple = ()      # variable-length batch: token offsets (0, ..., seq_len) of the packed sequences

    def c(self, q=None, k=None, v=None, o=None) -> _Params:
        """The C struct.  Strides of Q, K, V, O are taken from the tensors given: zero (= contiguous) for a
        contiguous tensor, otherwise its (batch, head, token) element strides, e.g. for a [B, N, H, d]
        projection output viewed as [B, H, N, d] with .transpose(1, 2)."""
        cp = _Params(self.batch, self.n_q_heads, self.n_kv_heads, self.seq_len, self.head_dim,
                     self.block_q, self.block_k, self.sink_blocks, self.local_blocks, self.flags)
        for name, t in (("q_stride", q), ("k_stride", k), ("v_stride", v), ("o_stride", o)):
            if t is not None and not t.is_contiguous():
                getattr(cp, name)[:] = [int(x) for x in t.stride()[:3]]
        if self.cu_seqlens:
            offsets = (ctypes.c_int32 * len(self.cu_seqlens))(*self.cu_seqlens)
            cp.n_seqs = len(self.cu_seqlens) - 1
            cp.cu_seqlens = ctypes.cast(offsets, ctypes.POINTER(ctypes.c_int32))
            cp._offsets = offsets      # (the host array lives as long as the struct)
        return cp

    @property
    def n_q(self) -> int:
        return self.seq_len // self.block_q

    @property
    def n_k(self) -> int:
        return self.seq_len // self.block_k

    @property
    def words(self) -> int:
        """Mask words per row: those of the longest sequence."""
        longest = self.seq_len
        if self.cu_seqlens:
            longest = max(b - a for a, b in zip(self.cu_seqlens[:-1], self.cu_seqlens[1:]))
        return (longest // self.block_k + 63) // 64


_vp, _sz, _i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
_pp = ctypes.POINTER(_Params)
_SIGS = {
    "sale_workspace_bytes": (_sz, [_pp, ctypes.c_int]),
    "sale_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "sale_quantize_qk": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "sale_select": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sale_select_static": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _vp]),
    "sale_sparse_attn": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sale_dense_attn": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sale_qk_int4_products": (ctypes.c_int, [_pp, _vp, _vp, _i32, _i32, _i32, _i32, _vp, _vp]),
    "sale_attn_int8_operands": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sale_attn_fp8_operands": (ctypes.c_int, [_pp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sale_calibrate_tau": (ctypes.c_int, [_pp, _vp, _vp, _vp, ctypes.c_float, ctypes.c_float, _i32, _vp, _vp, _vp,
                                          _vp, _sz, _vp]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(_lib, _name)
    _fn.restype = _res
    _fn.argtypes = _args

EXPORTED = tuple(_SIGS)


class SaleError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libsale status {status}: {_lib.sale_status_string(status).decode()}")


def _check(status: int) -> None:
    if status != OK:
        raise SaleError(status)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _expect(name: str, t, dtype, numel: int, optional: bool = False):
    """Host-side check of one tensor argument before anything is launched: the C ABI takes raw device pointers
    of contiguous buffers, so a wrong dtype, a strided view or a short buffer would be read or written out of
    bounds on the GPU."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name}: required tensor is None")
    if not t.is_cuda:
        raise ValueError(f"{name}: expected a device tensor, got {t.device}")
    dtypes = dtype if isinstance(dtype, tuple) else (dtype,)
    if t.dtype not in dtypes:
        raise ValueError(f"{name}: expected dtype {dtypes}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: expected a contiguous tensor (the library takes no strides), got strides {t.stride()}")
    if t.numel() != numel:
        raise ValueError(f"{name}: expected {numel} elements for these parameters, got {t.numel()} (shape {tuple(t.shape)})")


def _expect_bhnd(name: str, t, p: "Params", heads: int):
    """Q, K, V or O: a bf16 device tensor, either contiguous with batch * heads * seq_len * head_dim elements or
    a strided view of shape [batch, heads, seq_len, head_dim] whose last dimension is contiguous (its other
    three strides then go into the C struct: non-negative multiples of 8 elements)."""
    if t is not None and t.is_cuda and not t.is_contiguous():
        want = (p.batch, heads, p.seq_len, p.head_dim)
        if t.dtype != torch.bfloat16:
            raise ValueError(f"{name}: expected dtype torch.bfloat16, got {t.dtype}")
        if tuple(t.shape) != want:
            raise ValueError(f"{name}: a strided tensor must have shape {want}, got {tuple(t.shape)}")
        st = t.stride()
        if st[3] != 1 or any(x < 0 or x % 8 for x in st[:3]) or st[2] < p.head_dim:
            raise ValueError(f"{name}: strides {st} are not supported (last dimension contiguous, the others "
                             "non-negative multiples of 8 elements, rows at least head_dim apart)")
        return
    _expect(name, t, torch.bfloat16, p.batch * heads * p.seq_len * p.head_dim)


def _expect_ws(ws, need: int):
    """-> the workspace's size in BYTES (whatever its dtype).  Size and alignment are the library's to judge
    (SALE_ERR_WORKSPACE)."""
    if ws is None or not ws.is_cuda or not ws.is_contiguous():
        raise ValueError("workspace: expected a contiguous device tensor")
    return ws.numel() * ws.element_size()


def _qkv_numel(p: "Params"):
    return (p.batch * p.n_q_heads * p.seq_len * p.head_dim, p.batch * p.n_kv_heads * p.seq_len * p.head_dim)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def raw():
    """The ctypes library handle (tests of error paths call entry points directly)."""
    return _lib


def workspace_bytes(p: Params, which: int) -> int:
    return int(_lib.sale_workspace_bytes(ctypes.byref(p.c()), which))


def status_string(status: int) -> str:
    return _lib.sale_status_string(status).decode()


def quantize_qk(p: Params, q: torch.Tensor, k: torch.Tensor, out=None):
    """-> (q4 u8 [B,Hq,N,64], k4 u8 [B,Hkv,N,64], q_scale f32 [B,Hq,N/bq], k_scale f32 [B,Hkv,N/bk])"""
    dev = q.device
    if out is None:
        q4 = torch.empty(p.batch, p.n_q_heads, p.seq_len, p.head_dim // 2, dtype=torch.uint8, device=dev)
        k4 = torch.empty(p.batch, p.n_kv_heads, p.seq_len, p.head_dim // 2, dtype=torch.uint8, device=dev)
        qs = torch.empty(p.batch, p.n_q_heads, p.seq_len // p.block_q, dtype=torch.float32, device=dev)
        ks = torch.empty(p.batch, p.n_kv_heads, p.seq_len // p.block_k, dtype=torch.float32, device=dev)
    else:
        q4, k4, qs, ks = out
    nq, nk = _qkv_numel(p)
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads)
    _expect("q4", q4, torch.uint8, nq // 2); _expect("k4", k4, torch.uint8, nk // 2)
    _expect("q_scale", qs, torch.float32, p.batch * p.n_q_heads * (p.seq_len // p.block_q))
    _expect("k_scale", ks, torch.float32, p.batch * p.n_kv_heads * (p.seq_len // p.block_k))
    _check(_lib.sale_quantize_qk(ctypes.byref(p.c(q, k)), _ptr(q), _ptr(k), _ptr(q4), _ptr(k4), _ptr(qs), _ptr(ks), _stream()))
    return q4, k4, qs, ks


def select(p: Params, q, k, q4, k4, q_scale, k_scale, tau: torch.Tensor, want_stats: bool = False, out=None, ws=None):
    """-> (block_mask int64-viewed-u64 [B,Hq,Nq,W], row_counts i32 [B,Hq,Nq], m~, l~ or None)"""
    dev = q.device
    if out is None:
        mask = torch.empty(p.batch, p.n_q_heads, p.n_q, p.words, dtype=torch.int64, device=dev)
        counts = torch.empty(p.batch, p.n_q_heads, p.n_q, dtype=torch.int32, device=dev)
    else:
        mask, counts = out
    m = l = None
    if want_stats:
        m = torch.empty(p.batch, p.n_q_heads, p.seq_len, dtype=torch.float32, device=dev)
        l = torch.empty_like(m)
    need = workspace_bytes(p, WS_SELECT)
    if ws is None:
        ws = torch.empty(max(need, 1), dtype=torch.uint8, device=dev)
    nq, nk = _qkv_numel(p)
    est16 = bool(p.flags & FLAG_SELECT_16BIT)          # the 16-bit estimate does not read the codes
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads)
    _expect("q4", q4, torch.uint8, nq // 2, optional=est16); _expect("k4", k4, torch.uint8, nk // 2, optional=est16)
    _expect("q_scale", q_scale, torch.float32, p.batch * p.n_q_heads * p.n_q, optional=est16)
    _expect("k_scale", k_scale, torch.float32, p.batch * p.n_kv_heads * p.n_k, optional=est16)
    if tau.numel() not in (1, p.n_q_heads):
        raise ValueError(f"tau: expected 1 or {p.n_q_heads} thresholds, got {tau.numel()}")
    _expect("tau", tau, torch.float32, tau.numel())
    _expect("block_mask", mask, (torch.int64, torch.uint64), p.batch * p.n_q_heads * p.n_q * p.words)
    _expect("row_counts", counts, torch.int32, p.batch * p.n_q_heads * p.n_q)
    _check(_lib.sale_select(ctypes.byref(p.c(q, k)), _ptr(q), _ptr(k), _ptr(q4), _ptr(k4), _ptr(q_scale), _ptr(k_scale),
                            _ptr(tau), tau.numel(), _ptr(mask), _ptr(counts), _ptr(m), _ptr(l),
                            _ptr(ws), _expect_ws(ws, need), _stream()))
    return mask, counts, m, l


SELECT_STATIC_MAX_BYTES = 64 << 20


def select_static(p: Params, q, k, q4, k4, q_scale, k_scale, tau: torch.Tensor, out):
    """sale_select on the library's static scratch: allocates nothing, so `out` = (block_mask, row_counts) is
    required.  -> (block_mask, row_counts)"""
    mask, counts = out
    nq, nk = _qkv_numel(p)
    est16 = bool(p.flags & FLAG_SELECT_16BIT)
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads)
    _expect("q4", q4, torch.uint8, nq // 2, optional=est16); _expect("k4", k4, torch.uint8, nk // 2, optional=est16)
    _expect("q_scale", q_scale, torch.float32, p.batch * p.n_q_heads * p.n_q, optional=est16)
    _expect("k_scale", k_scale, torch.float32, p.batch * p.n_kv_heads * p.n_k, optional=est16)
    _expect("tau", tau, torch.float32, tau.numel())
    _expect("block_mask", mask, (torch.int64, torch.uint64), p.batch * p.n_q_heads * p.n_q * p.words)
    _expect("row_counts", counts, torch.int32, p.batch * p.n_q_heads * p.n_q)
    _check(_lib.sale_select_static(ctypes.byref(p.c(q, k)), _ptr(q), _ptr(k), _ptr(q4), _ptr(k4), _ptr(q_scale), _ptr(k_scale),
                                   _ptr(tau), tau.numel(), _ptr(mask), _ptr(counts), None, None, _stream()))
    return mask, counts


def sparse_attn(p: Params, q, k, v, block_mask, row_counts=None, want_lse: bool = False, out=None, ws=None):
    """-> (o bf16 [B,Hq,N,d], lse f32 [B,Hq,N] or None)"""
    o = torch.empty_like(q) if out is None else out
    lse = torch.empty(p.batch, p.n_q_heads, p.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    if ws is None:
        ws = torch.empty(max(1, workspace_bytes(p, WS_SPARSE_ATTN)), dtype=torch.uint8, device=q.device)
    nq, nk = _qkv_numel(p)
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads); _expect_bhnd("v", v, p, p.n_kv_heads)
    _expect_bhnd("o", o, p, p.n_q_heads)
    _expect("block_mask", block_mask, (torch.int64, torch.uint64), p.batch * p.n_q_heads * p.n_q * p.words)
    _expect("row_counts", row_counts, torch.int32, p.batch * p.n_q_heads * p.n_q, optional=True)
    _check(_lib.sale_sparse_attn(ctypes.byref(p.c(q, k, v, o)), _ptr(q), _ptr(k), _ptr(v), _ptr(block_mask), _ptr(row_counts),
                                 _ptr(o), _ptr(lse), _ptr(ws), _expect_ws(ws, workspace_bytes(p, WS_SPARSE_ATTN)), _stream()))
    return o, lse


def dense_attn(p: Params, q, k, v, want_lse: bool = False, out=None, ws=None):
    """-> (o bf16 [B,Hq,N,d], lse f32 [B,Hq,N] or None)"""
    o = torch.empty_like(q) if out is None else out
    lse = torch.empty(p.batch, p.n_q_heads, p.seq_len, dtype=torch.float32, device=q.device) if want_lse else None
    if ws is None:
        ws = torch.empty(max(1, workspace_bytes(p, WS_DENSE_ATTN)), dtype=torch.uint8, device=q.device)
    nq, nk = _qkv_numel(p)
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads); _expect_bhnd("v", v, p, p.n_kv_heads)
    _expect_bhnd("o", o, p, p.n_q_heads)
    _check(_lib.sale_dense_attn(ctypes.byref(p.c(q, k, v, o)), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                _ptr(ws), _expect_ws(ws, workspace_bytes(p, WS_DENSE_ATTN)), _stream()))
    return o, lse


def qk_int4_products(p: Params, q4, k4, q_head: int, q_block: int, k_block_begin: int, k_block_end: int):
    """-> int32 [block_q, (k_block_end - k_block_begin) * block_k]"""
    nq, nk = _qkv_numel(p)
    _expect("q4", q4, torch.uint8, nq // 2); _expect("k4", k4, torch.uint8, nk // 2)
    out = torch.empty(p.block_q, max(0, k_block_end - k_block_begin) * p.block_k, dtype=torch.int32, device=q4.device)
    _check(_lib.sale_qk_int4_products(ctypes.byref(p.c()), _ptr(q4), _ptr(k4), q_head, q_block,
                                      k_block_begin, k_block_end, _ptr(out), _stream()))
    return out


def attn_int8_operands(p: Params, q, k):
    """-> (q8 int8 [B,Hq,N,d], k8 int8 [B,Hkv,N,d], q_scale8 f32 [B,Hq,N/64], k_scale8 f32 [B,Hkv,N/64],
    k_mean f32 [B,Hkv,d]): the 8-bit operands of the quantized Computation-Pass (parity hook)."""
    dev = q.device
    nq, nk = _qkv_numel(p)
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads)
    q8 = torch.empty(p.batch, p.n_q_heads, p.seq_len, p.head_dim, dtype=torch.int8, device=dev)
    k8 = torch.empty(p.batch, p.n_kv_heads, p.seq_len, p.head_dim, dtype=torch.int8, device=dev)
    qs = torch.empty(p.batch, p.n_q_heads, p.seq_len // 64, dtype=torch.float32, device=dev)
    ks = torch.empty(p.batch, p.n_kv_heads, p.seq_len // 64, dtype=torch.float32, device=dev)
    mean = torch.empty(p.batch, p.n_kv_heads, p.head_dim, dtype=torch.float32, device=dev)
    ws = torch.empty(max(1, workspace_bytes(p, WS_INT8_OPERANDS)), dtype=torch.uint8, device=dev)
    _check(_lib.sale_attn_int8_operands(ctypes.byref(p.c(q, k)), _ptr(q), _ptr(k), _ptr(q8), _ptr(k8), _ptr(qs), _ptr(ks),
                                        _ptr(mean), _ptr(ws), ws.numel(), _stream()))
    return q8, k8, qs, ks, mean


def attn_fp8_operands(p: Params, v):
    """-> (v8 uint8 [B,Hkv,N,d] FP8 E4M3 bit patterns, v_scale f32 [B,Hkv,d]): the FP8 operand of the low-precision
    second product (parity hook)."""
    dev = v.device
    _expect_bhnd("v", v, p, p.n_kv_heads)
    v8 = torch.empty(p.batch, p.n_kv_heads, p.seq_len, p.head_dim, dtype=torch.uint8, device=dev)
    vs = torch.empty(p.batch, p.n_kv_heads, p.head_dim, dtype=torch.float32, device=dev)
    ws = torch.empty(max(1, workspace_bytes(p, WS_FP8_OPERANDS)), dtype=torch.uint8, device=dev)
    _check(_lib.sale_attn_fp8_operands(ctypes.byref(p.c(v=v)), _ptr(v), _ptr(v8), _ptr(vs), _ptr(ws), _expect_ws(ws, 0),
                                       _stream()))
    return v8, vs


def calibrate_tau(p: Params, q, k, v, tau0: float = 0.008, theta: float = 0.4, max_halvings: int = 8, ws=None):
    """-> (tau f32 [Hq], err f32 [Hq], halvings i32 [Hq]); synchronises the current stream."""
    dev = q.device
    nq, nk = _qkv_numel(p)
    _expect_bhnd("q", q, p, p.n_q_heads); _expect_bhnd("k", k, p, p.n_kv_heads); _expect_bhnd("v", v, p, p.n_kv_heads)
    tau = torch.empty(p.n_q_heads, dtype=torch.float32, device=dev)
    err = torch.empty(p.n_q_heads, dtype=torch.float32, device=dev)
    halv = torch.empty(p.n_q_heads, dtype=torch.int32, device=dev)
    if ws is None:
        ws = torch.empty(max(1, workspace_bytes(p, WS_CALIBRATE)), dtype=torch.uint8, device=dev)
    _check(_lib.sale_calibrate_tau(ctypes.byref(p.c(q, k, v)), _ptr(q), _ptr(k), _ptr(v), tau0, theta, max_halvings,
                                   _ptr(tau), _ptr(err), _ptr(halv), _ptr(ws), _expect_ws(ws, workspace_bytes(p, WS_CALIBRATE)),
                                   _stream()))
    return tau, err, halv

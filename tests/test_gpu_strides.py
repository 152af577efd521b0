"""Q, K, V and O addressed through the element strides of sale_params_t: the [batch][token][head][d] layout of a
projection output, and a padded layout, must give the results of the contiguous [batch][head][token][d] call,
bit for bit (same kernels, same arithmetic, other addresses), and those match the oracle."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from parity_utils import check_output, compare_mask_row, f32, words_to_bool

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


def _bnhd_view(x):
    """[B, H, N, d] values stored as [B][N][H][d]; returned as the [B, H, N, d] view of that storage."""
    return x.permute(0, 2, 1, 3).contiguous().transpose(1, 2)


def _padded_view(x, row_pad=32, head_pad=3, fill=float("nan")):
    """[B, H, N, d] values inside a larger [B, H + head_pad, N, d + row_pad] allocation (NaN elsewhere)."""
    B, H, N, d = x.shape
    big = torch.full((B, H + head_pad, N, d + row_pad), fill, dtype=x.dtype, device=x.device)
    big[:, :H, :, :d] = x
    return big[:, :H, :, :d]


def _run(sale, p, q, k, v, o, tau, want_int8=False):
    q4, k4, qs, ks = sale.quantize_qk(p, q, k)
    mask, counts, m, l = sale.select(p, q, k, q4, k4, qs, ks, tau, want_stats=True)
    _, lse = sale.sparse_attn(p, q, k, v, mask, counts, want_lse=True, out=o)
    o_sparse = o.clone()
    sale.dense_attn(p, q, k, v, out=o)
    o_dense = o.clone()
    torch.cuda.synchronize()
    return dict(q4=q4, k4=k4, qs=qs, ks=ks, mask=mask, counts=counts, m=m, l=l, lse=lse, o_sparse=o_sparse, o_dense=o_dense)


@pytest.mark.parametrize("layout", ["bnhd", "padded"])
@pytest.mark.parametrize("flags_name", ["bf16", "int8qk", "fp8pv"])
def test_strided_inputs_and_output_equal_the_contiguous_call(sale, layout, flags_name):
    w = inputs.scaled(inputs.LLAMA_32K, 2112, 4, 2, "strided-2k")       # 33 blocks: a ragged second mask word... of one word
    q, k, v = inputs.make_inputs(w)
    B = 2
    g = torch.Generator().manual_seed(3)
    scale = (0.8 + 0.4 * torch.rand(B, 1, 1, 1, generator=g))
    qb = (q[None].float() * scale).bfloat16().cuda()
    kb = k[None].expand(B, -1, -1, -1).contiguous().cuda()
    vb = (v[None].float() * scale).bfloat16().cuda()
    flags = {"bf16": 0, "int8qk": sale.FLAG_ATTN_INT8_QK, "fp8pv": sale.FLAG_ATTN_INT8_QK | sale.FLAG_ATTN_FP8_PV}[flags_name]
    p = sale.Params(B, w.n_q_heads, w.n_kv_heads, w.seq_len, flags=flags)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    ref = _run(sale, p, qb, kb, vb, torch.empty_like(qb), tau)
    view = _bnhd_view if layout == "bnhd" else _padded_view
    qs_, ks_, vs_ = view(qb), view(kb), view(vb)
    os_ = view(torch.zeros_like(qb))
    assert not qs_.is_contiguous() and not os_.is_contiguous()
    got = _run(sale, p, qs_, ks_, vs_, os_, tau)
    for name in ref:
        assert torch.equal(ref[name], got[name]), name
    if layout == "padded":      # nothing was written outside the rows of O
        base = os_._base if os_._base is not None else os_
        assert torch.isnan(base[:, w.n_q_heads:].float()).all() and torch.isnan(base[:, :, :, w.head_dim:].float()).all()
    if flags_name == "bf16":
        # and the contiguous result is the oracle's (batch entry 1)
        geo = so.Geometry(w.seq_len, w.head_dim)
        qf, kf, vf = f32(qb[1]), f32(kb[1]), f32(vb[1])
        qc, oqs = so.quantize_blocks(qf, 64)
        kc, oks = so.quantize_blocks(kf, 64)
        bits = words_to_bool(got["mask"][1].cpu().numpy(), p.n_k)
        hard = 0
        for h in range(w.n_q_heads):
            gk = h // w.group
            omask, margin, mthr, *_ = so.select_head(geo, qf[h], kf[gk], qc[h], kc[gk], oqs[h], oks[gk], w.tau)
            for i in range(geo.n_q):
                a, _ = compare_mask_row(bits[h, i], omask[i], margin[i], mthr[i])
                hard += a
            ref_o, _ = so.attention_head(geo, qf[h], kf[gk], vf[gk], bits[h])
            check_output(f32(got["o_sparse"][1, h]), ref_o, f"strided {layout} h{h}")
        assert hard == 0


def test_strided_calibration_equals_contiguous(sale):
    w = inputs.scaled(inputs.LLAMA_32K, 1024, 2, 1, "strided-cal")
    q, k, v = inputs.make_inputs(w)
    qb, kb, vb = (t[None].cuda() for t in (q, k, v))
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    t0, e0, h0 = sale.calibrate_tau(p, qb, kb, vb, 0.008, 0.05, 6)
    t1, e1, h1 = sale.calibrate_tau(p, _bnhd_view(qb), _bnhd_view(kb), _bnhd_view(vb), 0.008, 0.05, 6)
    torch.cuda.synchronize()
    assert torch.equal(t0, t1) and torch.equal(h0, h1) and torch.equal(e0, e1)

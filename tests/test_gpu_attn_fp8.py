"""GPU parity of the fully quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention": 8-bit first
product, FP8 second product) against the oracle on the same seeded inputs: the FP8 operand of V bit-exact,
attention outputs within the bf16 bars against the oracle that takes the same operands and visits the kept
blocks in the same order; the distance to the unquantized oracle is reported."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from tests.parity_utils import check_lse_fp8, check_output_fp8, f32, fp8_arg_tol, words_to_bool

pytestmark = pytest.mark.gpu

CASES = {
    "toy": inputs.TOY,
    "gqa4-1k": inputs.scaled(inputs.LLAMA_32K, 1024, 8, 2, "gqa4-1k"),
    "gqa3-ragged": inputs.scaled(inputs.LLAMA_32K, 64 * 7, 3, 1, "gqa3-ragged"),
    "one-block": inputs.scaled(inputs.TOY, 64, 1, 1, "one-block"),
    "gqa8-4k": inputs.scaled(inputs.LLAMA_32K, 4096 + 64, 8, 1, "gqa8-4k"),
}


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    w = CASES[request.param]
    q, k, v = inputs.make_inputs(w)
    return w, q, k, v, so.quantize_qk_int8(f32(q), f32(k)), so.quantize_v_fp8(f32(v))


def _dev(*ts):
    return [t.unsqueeze(0).contiguous().cuda() for t in ts]


def _same_fp8_bytes(got: np.ndarray, want: np.ndarray):
    """Bit patterns equal, a zero of either sign being the same value."""
    g = np.where((got & 0x7F) == 0, 0, got)
    w = np.where((want & 0x7F) == 0, 0, want)
    np.testing.assert_array_equal(g, w)


def test_fp8_operand_bit_exact(case, sale):
    w, q, k, v, _, (val, scale) = case
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    (vd,) = _dev(v)
    v8, vs = sale.attn_fp8_operands(p, vd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(vs[0].cpu().numpy().view(np.uint32), scale.view(np.uint32))
    _same_fp8_bytes(v8[0].cpu().numpy(), so.fp8_e4m3_encode(val))


def test_fp8_operand_zero_channel_and_extremes(sale):
    g = torch.Generator().manual_seed(12)
    v = (torch.randn(2, 192, 128, generator=g) * torch.logspace(-3, 3, 128)[None, None, :]).bfloat16()
    v[0, :, 5] = 0.0                                    # an all-zero channel: scale 1, values 0
    v[1, :, 9] = 3.0e38                                 # near the top of bf16
    v[1, 3, 9] = -3.0e38
    v[0, :, 11] = 1.0e-30                               # tiny but regular
    p = sale.Params(1, 2, 2, 192)
    v8, vs = sale.attn_fp8_operands(p, v[None].cuda())
    val, scale = so.quantize_v_fp8(f32(v))
    assert scale[0, 5] == 1.0 and np.all(val[0, :, 5] == 0) and np.all(np.abs(val[1, :, 9]) == 448)
    np.testing.assert_array_equal(vs[0].cpu().numpy().view(np.uint32), scale.view(np.uint32))
    _same_fp8_bytes(v8[0].cpu().numpy(), so.fp8_e4m3_encode(val))


def _oracle_fp8(w, geo, q, ops8, opsv, masks):
    """-> O, lse, and the slack that probabilities at a code midpoint may add to each (the kernel's fp32 argument)."""
    qc, qs, kc, ks, mean = ops8
    val, scale = opsv
    qf = f32(q)
    o = np.zeros((w.n_q_heads, w.seq_len, w.head_dim)); o_slack = np.zeros_like(o)
    lse = np.zeros((w.n_q_heads, w.seq_len)); lse_slack = np.zeros_like(lse)
    for h in range(w.n_q_heads):
        g = h // w.group
        for i in range(geo.n_q):
            rs = slice(i * 64, (i + 1) * 64)
            o[h, rs], lse[h, rs], o_slack[h, rs], lse_slack[h, rs] = so.attention_block_int8qk_fp8pv(
                geo, i, qc[h][rs], qs[h, i], kc[g], ks[g], val[g], scale[g], masks[h][i], q_blk=qf[h][rs], k_mean=mean[g],
                arg_tol=fp8_arg_tol(qs[h, i], ks[g], w.head_dim))
    return o, lse, o_slack, lse_slack


def test_fp8_sparse_and_dense_attention_match_oracle(case, sale):
    w, q, k, v, ops8, opsv = case
    flags = sale.FLAG_ATTN_INT8_QK | sale.FLAG_ATTN_FP8_PV
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, flags=flags)
    qd, kd, vd = _dev(q, k, v)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    o, lse = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True)
    od, lsed = sale.dense_attn(p, qd, kd, vd, want_lse=True)
    ones = torch.full_like(mask, -1)
    o1, _ = sale.sparse_attn(p, qd, kd, vd, ones)
    torch.cuda.synchronize()
    geo = so.Geometry(w.seq_len, w.head_dim)
    got = words_to_bool(mask[0].cpu().numpy(), p.n_k)
    ref, ref_lse, o_sl, lse_sl = _oracle_fp8(w, geo, q, ops8, opsv, got)
    mx, mean = check_output_fp8(f32(o[0]), ref, o_sl, f"fp8 sparse {w.name}")
    check_lse_fp8(lse[0].cpu().numpy(), ref_lse, lse_sl, f"fp8 sparse {w.name}")
    dm = [so.dense_mask(geo)] * w.n_q_heads
    refd, refd_lse, od_sl, lsed_sl = _oracle_fp8(w, geo, q, ops8, opsv, dm)
    mxd, meand = check_output_fp8(f32(od[0]), refd, od_sl, f"fp8 dense {w.name}")
    check_lse_fp8(lsed[0].cpu().numpy(), refd_lse, lsed_sl, f"fp8 dense {w.name}")
    quiet = lse_sl == 0
    print(f"[{w.name}] rows with no probability near a code midpoint: {quiet.mean():.1%}; largest lse slack {lse_sl.max():.3g}, "
          f"largest O slack {o_sl.max():.3g}")
    assert torch.equal(o1, od)                         # every block kept == the dense kernel, bit for bit
    qf, kf, vf = f32(q), f32(k), f32(v)
    plain = np.stack([so.attention_head(geo, qf[h], kf[h // w.group], vf[h // w.group], got[h])[0] for h in range(w.n_q_heads)])
    dq = np.abs(ref - plain)
    print(f"[{w.name}] fp8 sparse max abs {mx:.3g} mean abs {mean:.3g}; dense {mxd:.3g} / {meand:.3g}; "
          f"quantized oracle vs unquantized oracle: max {dq.max():.3g} mean {dq.mean():.3g}")
    assert 0 < dq.mean() < 2e-2 and dq.max() < 0.5      # reported, not a parity bar: the method's own quantization error


def test_fp8_windowed_path_equals_one_sweep(sale):
    """Long rows swept window by window (parked accumulators, the row sum parked with them) against one sweep."""
    w = inputs.Workload("fp8-17k", 17408, 2, 1, seed=0x5A1E0031, tau=0.002)
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, 2, 1, w.seq_len, flags=sale.FLAG_ATTN_INT8_QK | sale.FLAG_ATTN_FP8_PV)
    qd, kd, vd = _dev(q, k, v)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    assert int((counts > 192).sum()) > 8
    o_win = torch.full_like(qd, float("nan")); o_one = torch.full_like(qd, float("nan"))
    _, l_win = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True, out=o_win)
    _, l_one = sale.sparse_attn(p, qd, kd, vd, mask, None, want_lse=True, out=o_one)
    torch.cuda.synchronize()
    assert torch.equal(o_win, o_one) and torch.equal(l_win, l_one)      # parking is exact, the block order the same


def test_fp8_flag_needs_the_8bit_first_product_and_64_key_blocks(sale):
    x = torch.zeros(1, 1, 256, 128, dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(1 << 24, dtype=torch.uint8, device="cuda")
    for p in (sale.Params(1, 1, 1, 256, flags=sale.FLAG_ATTN_FP8_PV),
              sale.Params(1, 1, 1, 256, block_k=32, flags=sale.FLAG_ATTN_FP8_PV | sale.FLAG_ATTN_INT8_QK)):
        with pytest.raises(sale.SaleError) as e:
            sale.dense_attn(p, x, x, x, ws=ws)
        assert e.value.status == -3

"""GPU parity of the quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention": 8-bit Q and
smoothed K for the first product) against the oracle on the same seeded inputs: operands bit-exact (codes,
scales, key means), attention outputs within the bf16 bars against the oracle that takes the same 8-bit
operands; the distance to the unquantized oracle is reported."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from tests.parity_utils import LSE_ATOL, check_output, f32, words_to_bool

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
    ops = so.quantize_qk_int8(f32(q), f32(k))
    return w, q, k, v, ops


def _dev(*ts):
    return [t.unsqueeze(0).contiguous().cuda() for t in ts]


def test_int8_operands_bit_exact(case, sale):
    w, q, k, v, (qc, qs, kc, ks, mean) = case
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    qd, kd = _dev(q, k)
    q8, k8, gqs, gks, gmean = sale.attn_int8_operands(p, qd, kd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(gmean[0].cpu().numpy().view(np.uint32), mean.view(np.uint32))
    np.testing.assert_array_equal(gqs[0].cpu().numpy().view(np.uint32), qs.view(np.uint32))
    np.testing.assert_array_equal(gks[0].cpu().numpy().view(np.uint32), ks.view(np.uint32))
    np.testing.assert_array_equal(q8[0].cpu().numpy(), qc)
    np.testing.assert_array_equal(k8[0].cpu().numpy(), kc)


def test_int8_operands_zero_block_and_shifted_keys(sale):
    g = torch.Generator().manual_seed(11)
    q = (torch.randn(2, 256, 128, generator=g) * 3).bfloat16()
    k = (torch.randn(1, 256, 128, generator=g) + 5.0).bfloat16()      # far from zero mean: smoothing matters
    q[0, 64:128] = 0
    k[0, :, 7] = 2.5                                                   # a constant channel: smoothed to exactly 0
    p = sale.Params(1, 2, 1, 256)
    q8, k8, gqs, gks, gmean = sale.attn_int8_operands(p, q[None].cuda(), k[None].cuda())
    qc, qs, kc, ks, mean = so.quantize_qk_int8(f32(q), f32(k))
    assert mean[0, 7] == 2.5 and np.all(kc[0, :, 7] == 0) and qs[0, 1] == 1.0 and np.all(qc[0, 64:128] == 0)
    np.testing.assert_array_equal(gmean[0].cpu().numpy().view(np.uint32), mean.view(np.uint32))
    np.testing.assert_array_equal(q8[0].cpu().numpy(), qc)
    np.testing.assert_array_equal(k8[0].cpu().numpy(), kc)
    np.testing.assert_array_equal(gqs[0].cpu().numpy().view(np.uint32), qs.view(np.uint32))
    np.testing.assert_array_equal(gks[0].cpu().numpy().view(np.uint32), ks.view(np.uint32))


def _oracle_int8(w, geo, q, k, v, ops, masks):
    qc, qs, kc, ks, mean = ops
    vf, qf = f32(v), f32(q)
    o = np.zeros((w.n_q_heads, w.seq_len, w.head_dim))
    lse = np.zeros((w.n_q_heads, w.seq_len))
    for h in range(w.n_q_heads):
        g = h // w.group
        for i in range(geo.n_q):
            rs = slice(i * 64, (i + 1) * 64)
            o[h, rs], lse[h, rs] = so.attention_block_int8qk(geo, i, qc[h][rs], qs[h, i], kc[g], ks[g], vf[g], masks[h][i],
                                                               q_blk=qf[h][rs], k_mean=mean[g])
    return o, lse


def _oracle_plain(w, geo, q, k, v, masks):
    qf, kf, vf = f32(q), f32(k), f32(v)
    return np.stack([so.attention_head(geo, qf[h], kf[h // w.group], vf[h // w.group], masks[h])[0]
                     for h in range(w.n_q_heads)])


@pytest.mark.parametrize("bk", [64, 32])
def test_int8_sparse_and_dense_attention_match_oracle(case, sale, bk):
    w, q, k, v, ops = case
    flags = sale.FLAG_ATTN_INT8_QK | (sale.FLAG_SEGMENT_LOCAL if bk == 32 else 0)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=bk, flags=flags)
    qd, kd, vd = _dev(q, k, v)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    o, lse = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True)
    od, lsed = sale.dense_attn(p, qd, kd, vd, want_lse=True)
    ones = torch.full_like(mask, -1)
    o1, _ = sale.sparse_attn(p, qd, kd, vd, ones)
    torch.cuda.synchronize()
    geo = so.Geometry(w.seq_len, w.head_dim, 64, bk)
    got = words_to_bool(mask[0].cpu().numpy(), p.n_k)
    ref, ref_lse = _oracle_int8(w, geo, q, k, v, ops, got)
    mx, mean = check_output(f32(o[0]), ref, f"int8 sparse {w.name}")
    np.testing.assert_allclose(lse[0].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)
    dm = [so.dense_mask(geo)] * w.n_q_heads
    refd, refd_lse = _oracle_int8(w, geo, q, k, v, ops, dm)
    mxd, meand = check_output(f32(od[0]), refd, f"int8 dense {w.name}")
    np.testing.assert_allclose(lsed[0].cpu().numpy(), refd_lse, rtol=0, atol=LSE_ATOL)
    assert torch.equal(o1, od)                         # every block kept == the dense kernel, bit for bit
    plain = _oracle_plain(w, geo, q, k, v, got)
    dq = np.abs(ref - plain)
    print(f"[{w.name} 64x{bk}] int8 sparse max abs {mx:.3g} mean abs {mean:.3g}; dense {mxd:.3g} / {meand:.3g}; "
          f"8-bit oracle vs unquantized oracle: max {dq.max():.3g} mean {dq.mean():.3g}")
    assert 0 < dq.mean() < 1e-2 and dq.max() < 0.25     # reported, not a parity bar: the method's own quantization error


def test_int8_flag_changes_the_result_and_workspace(sale):
    w = CASES["gqa4-1k"]
    q, k, v = inputs.make_inputs(w)
    qd, kd, vd = _dev(q, k, v)
    p0 = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    p8 = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, flags=sale.FLAG_ATTN_INT8_QK)
    assert sale.workspace_bytes(p8, sale.WS_DENSE_ATTN) > sale.workspace_bytes(p0, sale.WS_DENSE_ATTN)
    o0, _ = sale.dense_attn(p0, qd, kd, vd)
    o8, _ = sale.dense_attn(p8, qd, kd, vd)
    assert not torch.equal(o0, o8)
    assert (o0.float() - o8.float()).abs().max() < 0.25      # the quantization error itself (reported by the test above)
    small = torch.empty(sale.workspace_bytes(p0, sale.WS_DENSE_ATTN), dtype=torch.uint8, device="cuda")
    with pytest.raises(sale.SaleError) as e:
        sale.dense_attn(p8, qd, kd, vd, ws=small)      # the bf16 call's workspace is too small for the 8-bit one
    assert e.value.status == -4

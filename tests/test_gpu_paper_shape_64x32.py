"""GPU parity of the whole path at the paper's block shape (Sec. 4.1: b_q = 64, b_k = 32; Appendix C: local
area of at least 128 tokens, segments of 4 key blocks whose remainder joins the local area), against the
CPU oracle on the same seeded inputs.  Products bit-exact; masks bit-exact outside the 1e-5 band;
attention output within the bf16 bars of the 64 x 64 tests."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from tests.parity_utils import LSE_ATOL, check_output, compare_mask_row, f32, oracle_quantize, words_to_bool

pytestmark = pytest.mark.gpu

FLAG_STATS_CAUSAL, FLAG_SELECT_16BIT, FLAG_SEGMENT_LOCAL = 1, 2, 4

CASES = {
    "toy": inputs.TOY,                                                          # N = 2048: 64 key blocks, one word
    "gqa4-1k": inputs.scaled(inputs.LLAMA_32K, 1024, 8, 2, "gqa4-1k"),
    "gqa3-ragged": inputs.scaled(inputs.LLAMA_32K, 64 * 7, 3, 1, "gqa3-ragged"),   # odd group: one head per wave
    "one-block": inputs.scaled(inputs.TOY, 64, 1, 1, "one-block"),
    "gqa8-4k": inputs.scaled(inputs.LLAMA_32K, 4096 + 64, 8, 1, "gqa8-4k"),     # three mask words, ragged last
}


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


@pytest.fixture(scope="module", params=list(CASES))
def case(request):
    w = CASES[request.param]
    q, k, v = inputs.make_inputs(w)
    return w, q, k


def _dev(*ts):
    return [t.unsqueeze(0).contiguous().cuda() for t in ts]


def test_products_bit_exact_64x32(case, sale):
    w, q, k = case
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=32)
    qd, kd = _dev(q, k)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    qc, oqs, kc, oks = oracle_quantize(q, k, 64, 32)
    np.testing.assert_array_equal(k4[0].cpu().numpy(), so.pack_int4(kc))
    np.testing.assert_array_equal(ks[0].cpu().numpy().view(np.uint32), oks.view(np.uint32))
    for h in sorted({0, w.n_q_heads - 1}):
        for i in sorted({0, p.n_q // 2, p.n_q - 1}):
            got = sale.qk_int4_products(p, q4, k4, h, i, 0, p.n_k).cpu().numpy()
            np.testing.assert_array_equal(got, so.int_products(qc[h][i * 64:(i + 1) * 64], kc[h // w.group]))
    if p.n_k > 3:       # a sub-range that starts at an odd key block
        got = sale.qk_int4_products(p, q4, k4, 0, p.n_q - 1, 1, 4).cpu().numpy()
        np.testing.assert_array_equal(got, so.int_products(qc[0][-64:], kc[0][32:128]))


@pytest.mark.parametrize("flags", [0, FLAG_SEGMENT_LOCAL, FLAG_SEGMENT_LOCAL | FLAG_STATS_CAUSAL,
                                   FLAG_SELECT_16BIT, FLAG_SELECT_16BIT | FLAG_SEGMENT_LOCAL])
def test_select_mask_matches_oracle_64x32(case, sale, flags):
    w, q, k = case
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=32, sink_blocks=1, local_blocks=4, flags=flags)
    est = "16bit" if flags & FLAG_SELECT_16BIT else "int4"
    qd, kd = _dev(q, k)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    if est == "16bit":
        mask, counts, m, l = sale.select(p, qd, kd, None, None, None, None, tau, want_stats=True)
    else:
        mask, counts, m, l = sale.select(p, qd, kd, q4, k4, qs, ks, tau, want_stats=True)
    torch.cuda.synchronize()
    geo = so.Geometry(w.seq_len, w.head_dim, 64, 32, 1, 4, stats_causal=bool(flags & FLAG_STATS_CAUSAL),
                      segment=4 if flags & FLAG_SEGMENT_LOCAL else 0)
    qc, oqs, kc, oks = oracle_quantize(q, k, 64, 32)
    qf, kf = f32(q), f32(k)
    got = words_to_bool(mask[0].cpu().numpy(), p.n_k)
    hard = soft = kept = 0
    for h in range(w.n_q_heads):
        g = h // w.group
        omask, margin, mthr, thr, om, ol = so.select_head(geo, qf[h], kf[g], qc[h], kc[g], oqs[h], oks[g], w.tau,
                                                          estimate=est)
        np.testing.assert_allclose(m[0, h].cpu().numpy(), om, rtol=2e-6, atol=2e-6)
        np.testing.assert_allclose(l[0, h].cpu().numpy(), ol, rtol=2e-5)
        for i in range(geo.n_q):
            a, b = compare_mask_row(got[h, i], omask[i], margin[i], mthr[i])
            hard += a; soft += b
        np.testing.assert_array_equal(counts[0, h].cpu().numpy(), got[h].sum(axis=1))
        kept += int(omask.sum())
    print(f"[{w.name} 64x32 flags={flags}] density {kept / (w.n_q_heads * so.dense_mask(geo).sum()):.3f}, "
          f"borderline mask differences: {soft}")
    assert hard == 0


def _oracle_attention(w, q, k, v, masks):
    geo = so.Geometry(w.seq_len, w.head_dim, 64, 32)
    qf, kf, vf = f32(q), f32(k), f32(v)
    o = np.zeros((w.n_q_heads, w.seq_len, w.head_dim))
    lse = np.zeros((w.n_q_heads, w.seq_len))
    for h in range(w.n_q_heads):
        g = h // w.group
        o[h], lse[h] = so.attention_head(geo, qf[h], kf[g], vf[g], masks[h])
    return o, lse


@pytest.mark.parametrize("flags", [0, FLAG_SEGMENT_LOCAL])
def test_sparse_attention_on_selected_64x32_mask(case, sale, flags):
    w, q, k = case
    _, _, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=32, flags=flags)
    qd, kd, vd = _dev(q, k, v)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    o, lse = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True)
    o_nc, _ = sale.sparse_attn(p, qd, kd, vd, mask)              # no counts: rows in natural order
    torch.cuda.synchronize()
    got = words_to_bool(mask[0].cpu().numpy(), p.n_k)            # the oracle attends over the GPU's mask
    ref, ref_lse = _oracle_attention(w, q, k, v, got)
    mx, mean = check_output(f32(o[0]), ref, f"sparse 64x32 {w.name}")
    np.testing.assert_allclose(lse[0].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)
    assert torch.equal(o, o_nc)
    odd = int((got.sum(axis=2) % 2 == 1).sum())
    print(f"[{w.name} 64x32 flags={flags}] sparse max abs {mx:.3g} mean abs {mean:.3g}; rows with an odd count: {odd}")


def test_sparse_attention_64x32_random_masks_odd_counts_and_all_ones(sale):
    """Masks the Selection-Pass would not produce: random half-tile patterns (rows with odd and even
    counts, a diagonal block with only its first or only its second half kept), garbage above the diagonal,
    and all ones, which must equal the dense kernel bit for bit."""
    w = CASES["gqa4-1k"]
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=32)
    qd, kd, vd = _dev(q, k, v)
    geo = so.Geometry(w.seq_len, w.head_dim, 64, 32)
    rng = np.random.default_rng(5)
    dm = so.dense_mask(geo)
    masks = []
    for h in range(w.n_q_heads):
        mk = dm & (rng.random(dm.shape) < 0.3)
        i = np.arange(geo.n_q)
        mk[i, 2 * i] = True                                       # every query row keeps its own key ...
        mk[i, 2 * i + 1] = rng.random(geo.n_q) < 0.5              # ... the second diagonal half only sometimes
        if h == 1:
            mk[3, :] = False; mk[3, 6] = True                     # a single half-tile: the diagonal's first
            mk[4, :] = False; mk[4, [8, 9]] = True                # only the diagonal block
            mk[5, :] = False; mk[5, [0, 10]] = True               # sink + first diagonal half
        masks.append(mk)
    counts = np.stack([mk.sum(axis=1) for mk in masks])
    assert (counts % 2 == 1).any() and (counts % 2 == 0).any()
    words = np.stack([np.stack([so.pack_mask_words(mk[i]) for i in range(geo.n_q)]) for mk in masks])
    words_garbage = words.copy()
    for i in range(geo.n_q):
        words_garbage[:, i, 0] |= np.uint64(0xFFFFFFFFFFFFFFFF) << np.uint64(2 * i + 2) if 2 * i + 2 < 64 else np.uint64(0)
    wd = torch.from_numpy(words_garbage.view(np.int64)).unsqueeze(0).cuda()
    cd = torch.from_numpy(counts.astype(np.int32)).unsqueeze(0).cuda()
    o, lse = sale.sparse_attn(p, qd, kd, vd, wd, cd, want_lse=True)
    ref, ref_lse = _oracle_attention(w, q, k, v, masks)
    check_output(f32(o[0]), ref, "random 64x32 masks")
    np.testing.assert_allclose(lse[0].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)
    ones = torch.full((1, w.n_q_heads, geo.n_q, p.words), -1, dtype=torch.int64, device="cuda")
    o1, _ = sale.sparse_attn(p, qd, kd, vd, ones)
    o2, _ = sale.dense_attn(p, qd, kd, vd)
    p64 = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    o3, _ = sale.dense_attn(p64, qd, kd, vd)
    assert torch.equal(o1, o2) and torch.equal(o2, o3)


def test_sparse_attention_64x32_rows_without_keys(sale):
    """Only the second half of the diagonal block kept: the first 32 query rows of the block see no key
    at all (O = 0, lse = -inf by the library's convention), the others match the oracle."""
    w = CASES["gqa3-ragged"]
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=32)
    qd, kd, vd = _dev(q, k, v)
    geo = so.Geometry(w.seq_len, w.head_dim, 64, 32)
    mk = np.zeros((geo.n_q, geo.n_k), dtype=bool)
    i = np.arange(geo.n_q)
    mk[i, 2 * i + 1] = True
    mk[2, 1] = True                                               # block 2: one more half-tile, all rows have keys
    words = np.stack([so.pack_mask_words(mk[r]) for r in range(geo.n_q)])
    wd = torch.from_numpy(np.broadcast_to(words, (1, w.n_q_heads) + words.shape).copy().view(np.int64)).cuda()
    o, lse = sale.sparse_attn(p, qd, kd, vd, wd, want_lse=True)
    torch.cuda.synchronize()
    with np.errstate(invalid="ignore", divide="ignore"):
        ref, ref_lse = _oracle_attention(w, q, k, v, [mk] * w.n_q_heads)
    og, lg = f32(o[0]), lse[0].cpu().numpy()
    empty = np.isnan(ref_lse) | np.isneginf(ref_lse)
    rows = np.arange(w.seq_len)
    assert np.array_equal(empty[0], (rows % 64 < 32) & (rows // 64 != 2))
    assert np.all(og[empty] == 0) and np.all(np.isneginf(lg[empty]))
    check_output(og[~empty], ref[~empty], "rows with keys")
    np.testing.assert_allclose(lg[~empty], ref_lse[~empty], rtol=0, atol=LSE_ATOL)


def test_select_64x32_rejects_what_it_cannot_do(sale):
    """A sequence with more than 4096 key blocks is refused; 32-row query blocks only quantize."""
    p = sale.Params(1, 1, 1, 256, block_k=32)
    assert sale.workspace_bytes(p, sale.WS_SELECT) > 0
    assert sale.workspace_bytes(p, sale.WS_SPARSE_ATTN) == sale.workspace_bytes(sale.Params(1, 1, 1, 256), sale.WS_SPARSE_ATTN)
    big = sale.Params(1, 1, 1, 262144, block_k=32)
    assert sale.workspace_bytes(big, sale.WS_SELECT) == 0
    p32 = sale.Params(1, 1, 1, 256, block_q=32, block_k=32)
    x = torch.zeros(1, 1, 256, 128, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(sale.SaleError):
        sale.dense_attn(p32, x, x, x, ws=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))

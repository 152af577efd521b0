"""GPU parity at the benchmark's full sizes (32K, 64K, 128K tokens, 32/8 heads),
in the launch configuration bench.py times, on sampled (head, query block)
units the oracle can compute one by one.  Query blocks are independent given
all of K and V, so parity on a sampled block is exact parity for its rows."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from tests.parity_utils import (LSE_ATOL, check_lse_fp8, check_output, check_output_fp8, compare_mask_row, fp8_arg_tol,
                                words_to_bool)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


def _sample_units(w, n_q, k, seed):
    rng = np.random.default_rng(seed)
    units = [(0, 0), (w.n_q_heads - 1, n_q - 1), (w.n_q_heads // 2, n_q - 1), (1, 4), (2, 5), (3, 63), (4, 64),
             (5, n_q - 2), (6, 193), (7, 255)]
    while len(units) < k:
        units.append((int(rng.integers(0, w.n_q_heads)), int(rng.integers(0, n_q))))
    return [(h % w.n_q_heads, min(i, n_q - 1)) for h, i in units]


# A mid-size case just above the length from which long rows are swept window by window with parked
# accumulators (9 mask words, ragged last window), with a low threshold so that many rows are long.
LONG_ROWS_16K = inputs.Workload("gqa2-36k-long-rows", 36864, 4, 2, seed=0x5A1E0010, tau=0.0005)
# The same with a single KV head (one lane: nothing to balance over the XCDs) and with three (an odd number of lanes).
LONG_ROWS_1KV = inputs.Workload("gqa4-1kv-33k-long-rows", 33792, 4, 1, seed=0x5A1E0011, tau=0.0005)
LONG_ROWS_3KV = inputs.Workload("gqa2-3kv-33k-long-rows", 33792, 6, 3, seed=0x5A1E0012, tau=0.001)
# The longest sequence the path accepts with 64-key blocks: 4096 key blocks, all 64 mask words, 32 window launches.
MAX_LENGTH_256K = inputs.Workload("gqa2-1kv-256k-max-length", 262144, 2, 1, seed=0x5A1E0013, tau=0.004)
EXTRA = {w.name: w for w in (LONG_ROWS_16K, LONG_ROWS_1KV, LONG_ROWS_3KV, MAX_LENGTH_256K)}


@pytest.mark.parametrize("name,n_units", [("gqa2-36k-long-rows", 24), ("gqa4-1kv-33k-long-rows", 10),
                                          ("gqa2-3kv-33k-long-rows", 12), ("llama31-8b-layer-32k", 14),
                                          ("llama31-8b-layer-64k", 12), ("llama31-8b-layer-128k", 12),
                                          ("gqa2-1kv-256k-max-length", 6)])
def test_full_size_sampled_parity(sale, name, n_units):
    w = EXTRA[name] if name in EXTRA else inputs.WORKLOADS[name]
    print(f"\n[{name}] generating inputs", flush=True)
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    dev = torch.device("cuda:0")
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    tau = torch.tensor([w.tau], dtype=torch.float32, device=dev)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    mask, counts, m, l = sale.select(p, qd, kd, q4, k4, qs, ks, tau, want_stats=True)
    ws = torch.empty(sale.workspace_bytes(p, sale.WS_SPARSE_ATTN), dtype=torch.uint8, device=dev)
    o_sparse, _ = sale.sparse_attn(p, qd, kd, vd, mask, counts, ws=ws)
    o_dense, lse_dense = sale.dense_attn(p, qd, kd, vd, want_lse=True, ws=ws)
    p16 = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, flags=sale.FLAG_SELECT_16BIT)
    mask16, counts16, _, _ = sale.select(p16, qd, kd, None, None, None, None, tau)     # Appendix E ablation
    torch.cuda.synchronize()
    print(f"[{name}] density with the 16-bit estimate "
          f"{int(counts16.sum()) / (w.n_q_heads * p.n_q * (p.n_q + 1) // 2):.4f}", flush=True)
    print(f"[{name}] GPU path done, density "
          f"{int(counts.sum()) / (w.n_q_heads * p.n_q * (p.n_q + 1) // 2):.4f}", flush=True)

    geo = so.Geometry(w.seq_len, w.head_dim)
    kq = {}
    hard = soft = 0
    worst_sparse = worst_dense = 0.0
    for h, i in _sample_units(w, p.n_q, n_units, seed=w.seed & 0xFFFF):
        g = h // w.group
        if g not in kq:
            kf = k[g].float().numpy()
            kc, oks = so.quantize_blocks(kf[None], 64)
            kq = {g: (kf, kc[0], oks[0], v[g].float().numpy())}
            np.testing.assert_array_equal(k4[0, g].cpu().numpy(), so.pack_int4(kc[0]))
            np.testing.assert_array_equal(ks[0, g].cpu().numpy().view(np.uint32), oks[0].view(np.uint32))
        kf, kc, oks, vf = kq[g]
        rs = slice(i * 64, (i + 1) * 64)
        qf = q[h, rs].float().numpy()
        qc, oqs = so.quantize_blocks(qf[None], 64)
        # a1: codes and scale of the sampled query block
        np.testing.assert_array_equal(q4[0, h, rs].cpu().numpy(), so.pack_int4(qc[0]))
        assert qs[0, h, i].cpu().numpy().view(np.uint32) == oqs[0, 0].view(np.uint32)
        # a3: integer products against 3 key-block ranges of this row
        for jb in sorted({0, i // 2, max(0, i - 7)}):
            je = min(jb + 8, i + 1)
            got = sale.qk_int4_products(p, q4, k4, h, i, jb, je).cpu().numpy()
            np.testing.assert_array_equal(got, so.int_products(qc[0], kc[jb * 64:je * 64]))
        # a2, a4, a5: statistics and the mask row
        row, margin, mthr, thr, om, ol = so.select_row(geo, i, qf, kf, qc[0], kc, float(oqs[0, 0]), oks, w.tau)
        np.testing.assert_allclose(m[0, h, rs].cpu().numpy(), om, rtol=2e-6, atol=2e-6)
        np.testing.assert_allclose(l[0, h, rs].cpu().numpy(), ol, rtol=2e-5)
        got_row = words_to_bool(mask[0, h, i].cpu().numpy(), p.n_k)
        a, b = compare_mask_row(got_row, row, margin, mthr)
        hard += a; soft += b
        assert int(counts[0, h, i]) == int(got_row.sum())
        row16, margin16, mthr16, *_ = so.select_row(geo, i, qf, kf, None, None, 0.0, None, w.tau, "16bit")
        a, b = compare_mask_row(words_to_bool(mask16[0, h, i].cpu().numpy(), p.n_k), row16, margin16, mthr16)
        hard += a; soft += b
        # a6, a7: outputs of the sampled rows (the oracle attends over the GPU's mask row)
        ref_s, _ = so.attention_block(geo, i, qf, kf, vf, got_row)
        ref_d, ref_lse = so.attention_block(geo, i, qf, kf, vf, so.dense_mask(geo)[i] if w.seq_len <= 32768
                                            else np.arange(geo.n_k) <= i)
        ms, _ = check_output(o_sparse[0, h, rs].float().cpu().numpy(), ref_s, f"sparse {name} h{h} i{i}")
        md, _ = check_output(o_dense[0, h, rs].float().cpu().numpy(), ref_d, f"dense {name} h{h} i{i}")
        np.testing.assert_allclose(lse_dense[0, h, rs].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)
        worst_sparse, worst_dense = max(worst_sparse, ms), max(worst_dense, md)
        print(f"[{name}] unit (h={h}, i={i}) kept {int(got_row.sum())}/{i + 1} ok", flush=True)
    print(f"[{name}] borderline mask differences {soft}, max abs err sparse {worst_sparse:.3g} dense {worst_dense:.3g}")
    assert hard == 0
    assert soft <= 4


@pytest.mark.parametrize("name,n_units", [("gqa2-36k-long-rows", 16), ("llama31-8b-layer-128k", 10)])
def test_full_size_sampled_parity_paper_shape_64x32(sale, name, n_units):
    """The same sampled check at the paper's block shape (Sec. 4.1: b_q = 64, b_k = 32) with the segment
    rule of Appendix C: 18 and 64 mask words, both above the length from which long rows are swept in
    windows (16 words at b_k = 32)."""
    w = LONG_ROWS_16K if name == LONG_ROWS_16K.name else inputs.WORKLOADS[name]
    print(f"\n[{name} 64x32] generating inputs", flush=True)
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=32, flags=sale.FLAG_SEGMENT_LOCAL)
    dev = torch.device("cuda:0")
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    tau = torch.tensor([w.tau], dtype=torch.float32, device=dev)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    mask, counts, m, l = sale.select(p, qd, kd, q4, k4, qs, ks, tau, want_stats=True)
    o_sparse, lse = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True)
    torch.cuda.synchronize()
    dense_pairs = sum(2 * i + 2 for i in range(p.n_q)) * w.n_q_heads
    print(f"[{name} 64x32] GPU path done, density {int(counts.sum()) / dense_pairs:.4f}", flush=True)

    geo = so.Geometry(w.seq_len, w.head_dim, 64, 32, 1, 4, segment=4)
    kq = {}
    hard = soft = 0
    worst = 0.0
    for h, i in _sample_units(w, p.n_q, n_units, seed=(w.seed + 1) & 0xFFFF):
        g = h // w.group
        if g not in kq:
            kf = k[g].float().numpy()
            kc, oks = so.quantize_blocks(kf[None], 32)
            kq = {g: (kf, kc[0], oks[0], v[g].float().numpy())}
            np.testing.assert_array_equal(ks[0, g].cpu().numpy().view(np.uint32), oks[0].view(np.uint32))
        kf, kc, oks, vf = kq[g]
        rs = slice(i * 64, (i + 1) * 64)
        qf = q[h, rs].float().numpy()
        qc, oqs = so.quantize_blocks(qf[None], 64)
        jb = max(0, 2 * i - 5)
        got = sale.qk_int4_products(p, q4, k4, h, i, jb, 2 * i + 2).cpu().numpy()
        np.testing.assert_array_equal(got, so.int_products(qc[0], kc[jb * 32:(2 * i + 2) * 32]))
        row, margin, mthr, thr, om, ol = so.select_row(geo, i, qf, kf, qc[0], kc, float(oqs[0, 0]), oks, w.tau)
        np.testing.assert_allclose(m[0, h, rs].cpu().numpy(), om, rtol=2e-6, atol=2e-6)
        np.testing.assert_allclose(l[0, h, rs].cpu().numpy(), ol, rtol=2e-5)
        got_row = words_to_bool(mask[0, h, i].cpu().numpy(), p.n_k)
        a, b = compare_mask_row(got_row, row, margin, mthr)
        hard += a; soft += b
        assert int(counts[0, h, i]) == int(got_row.sum())
        ref_s, ref_lse = so.attention_block(geo, i, qf, kf, vf, got_row)
        ms, _ = check_output(o_sparse[0, h, rs].float().cpu().numpy(), ref_s, f"sparse 64x32 {name} h{h} i{i}")
        np.testing.assert_allclose(lse[0, h, rs].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)
        worst = max(worst, ms)
        print(f"[{name} 64x32] unit (h={h}, i={i}) kept {int(got_row.sum())}/{2 * i + 2} ok", flush=True)
    print(f"[{name} 64x32] borderline mask differences {soft}, max abs err sparse {worst:.3g}")
    assert hard == 0
    assert soft <= 4


@pytest.mark.parametrize("fp8", [False, True], ids=["pv16", "pv8"])
@pytest.mark.parametrize("name,n_units", [("gqa2-36k-long-rows", 12), ("llama31-8b-layer-128k", 8)])
def test_full_size_sampled_parity_int8_computation_pass(sale, name, n_units, fp8):
    """The quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention") at full size, windowed sweep
    included: sampled units against the oracle that takes the same 8-bit operands; with the second product in
    16 bit and in FP8 (there with the slack of probabilities at a code midpoint, as in the small cases)."""
    w = LONG_ROWS_16K if name == LONG_ROWS_16K.name else inputs.WORKLOADS[name]
    print(f"\n[{name} int8{' fp8' if fp8 else ''}] generating inputs", flush=True)
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len,
                    flags=sale.FLAG_ATTN_INT8_QK | (sale.FLAG_ATTN_FP8_PV if fp8 else 0))
    dev = torch.device("cuda:0")
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    tau = torch.tensor([w.tau], dtype=torch.float32, device=dev)
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    ws = torch.empty(sale.workspace_bytes(p, sale.WS_SPARSE_ATTN), dtype=torch.uint8, device=dev)
    o_sparse, lse = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True, ws=ws)
    o_sparse = o_sparse.clone()
    o_dense, _ = sale.dense_attn(p, qd, kd, vd, ws=ws)
    q8, k8, qs8, ks8, mean = sale.attn_int8_operands(p, qd, kd)
    v_scale = sale.attn_fp8_operands(p, vd)[1] if fp8 else None
    torch.cuda.synchronize()
    print(f"[{name} int8] GPU path done", flush=True)
    geo = so.Geometry(w.seq_len, w.head_dim)
    kq = {}
    worst_s = worst_d = 0.0
    for h, i in _sample_units(w, p.n_q, n_units, seed=(w.seed + 2) & 0xFFFF):
        g = h // w.group
        if g not in kq:
            kf = k[g].float().numpy()
            ksm, omean = so.smooth_k(kf[None])
            kc, oks = so.quantize_blocks(ksm, 64, 127)
            np.testing.assert_array_equal(mean[0, g].cpu().numpy().view(np.uint32), omean[0].view(np.uint32))
            np.testing.assert_array_equal(k8[0, g].cpu().numpy(), kc[0])
            np.testing.assert_array_equal(ks8[0, g].cpu().numpy().view(np.uint32), oks[0].view(np.uint32))
            v8 = None
            if fp8:
                v8 = so.quantize_v_fp8(v[g].float().numpy()[None])
                np.testing.assert_array_equal(v_scale[0, g].cpu().numpy().view(np.uint32), v8[1][0].view(np.uint32))
            kq = {g: (kc[0], oks[0], v[g].float().numpy(), omean[0], v8)}
        kc, oks, vf, kmean, v8 = kq[g]
        rs = slice(i * 64, (i + 1) * 64)
        qc, oqs = so.quantize_blocks(q[h, rs].float().numpy()[None], 64, 127)
        np.testing.assert_array_equal(q8[0, h, rs].cpu().numpy(), qc[0])
        assert qs8[0, h, i].cpu().numpy().view(np.uint32) == oqs[0, 0].view(np.uint32)
        got_row = words_to_bool(mask[0, h, i].cpu().numpy(), p.n_k)
        if fp8:
            tol = fp8_arg_tol(oqs[0, 0], oks, w.head_dim)
            ref_s, ref_lse, o_sl, lse_sl = so.attention_block_int8qk_fp8pv(
                geo, i, qc[0], oqs[0, 0], kc, oks, v8[0][0], v8[1][0], got_row, q_blk=q[h, rs].float().numpy(), k_mean=kmean,
                arg_tol=tol)
            ref_d, _, od_sl, _ = so.attention_block_int8qk_fp8pv(geo, i, qc[0], oqs[0, 0], kc, oks, v8[0][0], v8[1][0],
                                                                 np.arange(geo.n_k) <= i, arg_tol=tol)
            ms, _ = check_output_fp8(o_sparse[0, h, rs].float().cpu().numpy(), ref_s, o_sl, f"fp8 sparse {name} h{h} i{i}")
            md, _ = check_output_fp8(o_dense[0, h, rs].float().cpu().numpy(), ref_d, od_sl, f"fp8 dense {name} h{h} i{i}")
            check_lse_fp8(lse[0, h, rs].cpu().numpy(), ref_lse, lse_sl, f"fp8 sparse {name} h{h} i{i}")
        else:
            ref_s, ref_lse = so.attention_block_int8qk(geo, i, qc[0], oqs[0, 0], kc, oks, vf, got_row,
                                                       q_blk=q[h, rs].float().numpy(), k_mean=kmean)
            ref_d, _ = so.attention_block_int8qk(geo, i, qc[0], oqs[0, 0], kc, oks, vf, np.arange(geo.n_k) <= i)
            ms, _ = check_output(o_sparse[0, h, rs].float().cpu().numpy(), ref_s, f"int8 sparse {name} h{h} i{i}")
            md, _ = check_output(o_dense[0, h, rs].float().cpu().numpy(), ref_d, f"int8 dense {name} h{h} i{i}")
            np.testing.assert_allclose(lse[0, h, rs].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)
        worst_s, worst_d = max(worst_s, ms), max(worst_d, md)
        print(f"[{name} int8] unit (h={h}, i={i}) kept {int(got_row.sum())}/{i + 1} ok", flush=True)
    print(f"[{name} int8] max abs err sparse {worst_s:.3g} dense {worst_d:.3g}")


def _popcount64(x: torch.Tensor) -> torch.Tensor:
    """Population count of int64 words (bit patterns), on the GPU."""
    c = torch.zeros_like(x)
    for s in range(0, 64, 8):
        b = (x >> s) & 0xFF
        b = (b & 0x55) + ((b >> 1) & 0x55)
        b = (b & 0x33) + ((b >> 2) & 0x33)
        c += (b & 0x0F) + (b >> 4)
    return c


@pytest.mark.parametrize("bk", [64, 32])
def test_full_size_properties_over_every_row_128k(sale, bk):
    """What must hold for EVERY row at the benchmark's size (the sampled test checks values on a few):
    counts = popcount; nothing above the causal boundary; sink and local blocks kept; masks nested in tau;
    tau -> 0 keeps every causal block and then sparse == dense bit for bit; the kept probability mass
    exp(lse_sparse - lse_dense) lies in (0, 1]."""
    w = inputs.WORKLOADS["llama31-8b-layer-128k"]
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len, block_k=bk)
    dev = torch.device("cuda:0")
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    f = 64 // bk
    i = torch.arange(p.n_q, device=dev)
    j = torch.arange(p.words * 64, device=dev)
    causal = (j[None, :] <= ((i + 1) * f - 1)[:, None]).view(p.n_q, p.words, 64)
    weights = torch.tensor([1 << b for b in range(63)] + [-(1 << 63)], dtype=torch.int64, device=dev)
    causal_words = (causal.long() * weights).sum(-1)                                 # [n_q, W] bit patterns
    local = ((j[None, :] <= ((i + 1) * f - 1)[:, None]) & (j[None, :] > ((i + 1) * f - 1 - 4)[:, None])) | (j[None, :] == 0)
    local_words = (local.view(p.n_q, p.words, 64).long() * weights).sum(-1)
    masks = {}
    for tau in (0.008, 0.004, 0.002, 1e-30):
        t = torch.tensor([tau], dtype=torch.float32, device=dev)
        mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, t)
        assert torch.equal(_popcount64(mask[0]).sum(-1).int(), counts[0]), tau
        assert not torch.any(mask[0] & ~causal_words[None]), tau
        assert torch.equal(mask[0] & local_words[None], local_words[None].expand_as(mask[0])), tau
        masks[tau] = (mask, counts)
    for hi, lo in ((0.008, 0.004), (0.004, 0.002), (0.002, 1e-30)):
        assert not torch.any(masks[hi][0] & ~masks[lo][0])                           # nested in tau
    assert int(masks[0.008][1].sum()) < int(masks[0.004][1].sum()) < int(masks[0.002][1].sum())
    assert torch.equal(masks[1e-30][0][0], causal_words[None].expand_as(masks[1e-30][0][0]))
    ws = torch.empty(sale.workspace_bytes(p, sale.WS_SPARSE_ATTN), dtype=torch.uint8, device=dev)
    o_all, lse_all = sale.sparse_attn(p, qd, kd, vd, *masks[1e-30], want_lse=True, ws=ws)
    o_all = o_all.clone()
    o_dense, lse_dense = sale.dense_attn(p, qd, kd, vd, want_lse=True, ws=ws)
    assert torch.equal(o_all, o_dense) and torch.equal(lse_all, lse_dense)
    # Under the real mask: every row through the windowed, balanced path (row_counts given) against the same
    # row through the plain one-sweep path (no counts: no ordering, no windows, no tables).  Both outputs
    # start as NaN, so a unit that a table or a tail rank dropped, or that was written from stale state, shows.
    o_sp = torch.full_like(qd, float("nan"))
    lse_sp = torch.full((1, w.n_q_heads, w.seq_len), float("nan"), dtype=torch.float32, device=dev)
    lib = sale.raw()
    import ctypes
    def run(counts_t, o_t, lse_t):
        rc = lib.sale_sparse_attn(ctypes.byref(p.c()), qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), masks[0.004][0].data_ptr(),
                                  None if counts_t is None else counts_t.data_ptr(), o_t.data_ptr(), lse_t.data_ptr(),
                                  ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        assert rc == 0
    run(masks[0.004][1], o_sp, lse_sp)
    o_one = torch.full_like(qd, float("nan"))
    lse_one = torch.full_like(lse_sp, float("nan"))
    run(None, o_one, lse_one)
    torch.cuda.synchronize()
    assert torch.isfinite(o_sp.float()).all() and torch.isfinite(lse_sp).all()          # every unit was written
    assert torch.isfinite(o_one.float()).all() and torch.isfinite(lse_one).all()
    d_win = (o_sp.float() - o_one.float()).abs()
    # (the two paths add the same blocks in the same order; they differ only where a long row's accumulators
    # were parked between windows, which is exact, so the outputs agree far inside the parity bar)
    assert float(d_win.max()) <= 2e-2 and float(d_win.mean()) <= 2e-4, (float(d_win.max()), float(d_win.mean()))
    assert float((lse_sp - lse_one).abs().max()) <= 2 * LSE_ATOL
    print(f"[128k 64x{bk}] windowed vs one-sweep over every row: max {float(d_win.max()):.3g} mean {float(d_win.mean()):.3g}")
    mass = torch.exp(lse_sp - lse_dense)
    assert float(mass.max()) <= 1.0 + 2 * LSE_ATOL and float(mass.min()) > 0.0
    print(f"[128k 64x{bk}] kept probability mass: min {float(mass.min()):.3f} mean {float(mass.mean()):.4f}")


def test_many_kv_heads_beyond_the_balancing_table(sale):
    """264 (batch x KV head) lanes: more than the balancing tables hold, so the windowed sweep falls back to
    lane = KV head.  The result must agree with the one-sweep-per-row path (no counts given) up to the rounding
    of a different summation order, and a few units are checked against the oracle."""
    w = inputs.Workload("mha-17k", 17408, 1, 1, seed=0x5A1E0020, tau=0.002)
    q, k, v = inputs.make_inputs(w)
    B = 264
    g = torch.Generator().manual_seed(5)
    scale = 0.75 + 0.5 * torch.rand(B, 1, 1, 1, generator=g)              # the batch entries differ
    qb = (q[None].float() * scale).bfloat16().cuda()
    kb = k[None].expand(B, -1, -1, -1).contiguous().cuda()
    vb = v[None].expand(B, -1, -1, -1).contiguous().cuda()
    p = sale.Params(B, 1, 1, w.seq_len)
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    q4, k4, qs, ks = sale.quantize_qk(p, qb, kb)
    mask, counts, _, _ = sale.select(p, qb, kb, q4, k4, qs, ks, tau)
    assert int((counts > 192).sum()) > 1000                               # many long rows: the windowed path runs
    o_win, _ = sale.sparse_attn(p, qb, kb, vb, mask, counts)
    o_one, _ = sale.sparse_attn(p, qb, kb, vb, mask, None)
    torch.cuda.synchronize()
    d = (o_win.float() - o_one.float()).abs()
    assert float(d.max()) <= 2e-2 and float(d.mean()) <= 2e-4
    geo = so.Geometry(w.seq_len, w.head_dim)
    kf, vf = k[0].float().numpy(), v[0].float().numpy()
    for b, i in ((0, geo.n_q - 1), (131, 200), (263, geo.n_q - 1), (263, 5)):
        rs = slice(i * 64, (i + 1) * 64)
        row = words_to_bool(mask[b, 0, i].cpu().numpy(), p.n_k)
        ref, _ = so.attention_block(geo, i, qb[b, 0, rs].float().cpu().numpy(), kf, vf, row)
        check_output(o_win[b, 0, rs].float().cpu().numpy(), ref, f"264 lanes b{b} i{i}")


def test_fewer_parking_slots_than_long_rows_gives_the_same_bits(sale):
    """The workspace beyond SALE_WS_SPARSE_ATTN_MIN holds the parking slots of the windowed sweep; a long row that
    finds none is swept in one go.  With no slot, with slots for about half of the long rows and with one slot per
    row block the outputs and lse are the same bit for bit (the block order of a row never changes)."""
    w = LONG_ROWS_16K
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    qd, kd, vd = (t.unsqueeze(0).cuda() for t in (q, k, v))
    tau = torch.tensor([w.tau], dtype=torch.float32, device="cuda")
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau)
    n_long = int((counts > 192).sum())
    assert n_long > 100
    lo, full = sale.workspace_bytes(p, sale.WS_SPARSE_ATTN_MIN), sale.workspace_bytes(p, sale.WS_SPARSE_ATTN)
    assert lo + p.n_q * w.n_q_heads * sale.PARKED_ROW_BYTES == full
    outs = []
    for nbytes in (full, lo + n_long * sale.PARKED_ROW_BYTES, lo + (n_long // 2) * sale.PARKED_ROW_BYTES, lo + 7, lo):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        o = torch.full_like(qd, float("nan"))
        _, lse = sale.sparse_attn(p, qd, kd, vd, mask, counts, want_lse=True, out=o, ws=ws)
        torch.cuda.synchronize()
        outs.append((o.clone(), lse.clone()))
        assert not torch.isnan(o).any()
    for o, lse in outs[1:]:
        assert torch.equal(o, outs[0][0]) and torch.equal(lse, outs[0][1])
    with pytest.raises(sale.SaleError) as e:
        sale.sparse_attn(p, qd, kd, vd, mask, counts, ws=torch.empty(lo - 1, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -4


def _predict_balance_overflow(mask_bool, counts, n_qb, lanes, win_lo, win_hi, min_count):
    """The placement rule of the window tables, restated on the host from its description (a head whose work in
    the window exceeds the mean sheds n_in * (w - mean) / w units to the heads that lack work, in proportion to
    what they lack): does some lane end up with more entries than it has slots (= units per KV head)?"""
    work, n_in = [], []
    for l in range(lanes):
        w_l = n_l = 0
        for i in range(n_qb):
            if counts[l, i] <= min_count or win_lo > i:
                continue
            c = int(mask_bool[l, i, win_lo:min(win_hi, i + 1)].sum())
            if c > 0 or win_hi > i:
                n_l += 1
                w_l += c
        work.append(w_l); n_in.append(n_l)
    target = sum(work) / lanes
    shed = [int(n_in[l] * (work[l] - target) / work[l]) if work[l] > target else 0 for l in range(lanes)]
    lack = [max(0.0, target - work[l]) for l in range(lanes)]
    total = sum(shed)
    recv, run = [], 0.0
    for l in range(lanes):
        lo = int(total * (run / sum(lack)))
        run += lack[l]
        recv.append(lo)
    recv.append(total)
    return any(n_in[l] - shed[l] + recv[l + 1] - recv[l] > n_qb for l in range(lanes)), n_in, shed


def test_balance_table_overflow_falls_back_to_lane_equals_head(sale):
    """One KV head whose long rows keep a single block in the second window next to three heads that keep everything
    there: the light head's lane would receive more shed units than it has slots, so the window's table falls back
    to lane = KV head.  The result must be that of the one-sweep path, every unit written once, and equal to the
    oracle on sampled units."""
    n, hq = 40960, 4                                       # 640 query blocks, 5 windows of 128 key blocks
    g = torch.Generator().manual_seed(77)
    q = torch.randn(hq, n, 128, generator=g).bfloat16()
    k = torch.randn(hq, n, 128, generator=g).bfloat16()
    v = torch.randn(hq, n, 128, generator=g).bfloat16()
    p = sale.Params(1, hq, hq, n)
    n_qb = p.n_q
    keep = np.zeros((hq, n_qb, n_qb), dtype=bool)
    tri = np.tril(np.ones((n_qb, n_qb), dtype=bool))
    keep[1:] = tri
    keep[0] = tri
    keep[0, :, 129:256] = False                            # head 0: of window 1 (blocks 128..255) only block 128
    keep[0][np.arange(n_qb), np.arange(n_qb)] = True       # (the diagonal block stays)
    keep[0] &= tri
    counts_np = keep.sum(-1).astype(np.int32)
    overflow, n_in, shed = _predict_balance_overflow(keep, counts_np, n_qb, hq, 128, 256, 192)
    assert overflow, (n_in, shed)                          # the case does reach the fallback
    words = np.zeros((hq, n_qb, p.words), dtype=np.uint64)
    for j in range(n_qb):
        words[:, :, j // 64] |= keep[:, :, j].astype(np.uint64) << np.uint64(j % 64)
    dev = torch.device("cuda:0")
    mask = torch.from_numpy(words.view(np.int64)).unsqueeze(0).to(dev)
    counts = torch.from_numpy(counts_np).unsqueeze(0).to(dev)
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    ws = torch.empty(sale.workspace_bytes(p, sale.WS_SPARSE_ATTN), dtype=torch.uint8, device=dev)
    o_win = torch.full_like(qd, float("nan"))
    o_one = torch.full_like(qd, float("nan"))
    sale.sparse_attn(p, qd, kd, vd, mask, counts, out=o_win, ws=ws)
    sale.sparse_attn(p, qd, kd, vd, mask, None, out=o_one, ws=ws)
    torch.cuda.synchronize()
    assert torch.isfinite(o_win.float()).all() and torch.isfinite(o_one.float()).all()
    d = (o_win.float() - o_one.float()).abs()
    assert float(d.max()) <= 2e-2 and float(d.mean()) <= 2e-4
    geo = so.Geometry(n, 128)
    for h, i in ((0, n_qb - 1), (0, 330), (2, n_qb - 1), (3, 200)):
        rs = slice(i * 64, (i + 1) * 64)
        ref, _ = so.attention_block(geo, i, q[h, rs].float().numpy(), k[h].float().numpy(), v[h].float().numpy(), keep[h, i])
        check_output(o_win[0, h, rs].float().cpu().numpy(), ref, f"overflow fallback h{h} i{i}")

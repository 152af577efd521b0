"""Variable-length batches (cu_seqlens-style offsets): one call over sequences of different lengths packed
along the token axis must give, for every sequence, the results of running that sequence alone - bit for bit
(same kernels, same arithmetic) - and those match the oracle called per sequence."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from parity_utils import LSE_ATOL, check_output, compare_mask_row, f32, words_to_bool

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sale():
    from paper_2505_24179_amd import sale as mod
    return mod


def _pipeline(sale, p, q, k, v, tau):
    q4, k4, qs, ks = sale.quantize_qk(p, q, k)
    mask, counts, m, l = sale.select(p, q, k, q4, k4, qs, ks, tau, want_stats=True)
    o = torch.full_like(q, float("nan"))
    _, lse = sale.sparse_attn(p, q, k, v, mask, counts, want_lse=True, out=o)
    od = torch.full_like(q, float("nan"))
    _, lsed = sale.dense_attn(p, q, k, v, want_lse=True, out=od)
    torch.cuda.synchronize()
    return dict(q4=q4, k4=k4, qs=qs, ks=ks, mask=mask, counts=counts, m=m, l=l, o=o, lse=lse, od=od, lsed=lsed)


@pytest.mark.parametrize("bk,flags_name", [(64, "default"), (32, "segment"), (64, "stats_causal"), (64, "16bit")])
def test_ragged_batch_equals_each_sequence_alone(sale, bk, flags_name):
    """Three sequences, the longest beyond the 16K-token threshold of the windowed sweep (so the packed call runs
    window launches with balancing tables over units of all three sequences)."""
    lens = (20480, 4160, 1024)
    hq, hkv = 4, 2
    flags = {"default": 0, "segment": sale.FLAG_SEGMENT_LOCAL, "stats_causal": sale.FLAG_STATS_CAUSAL,
             "16bit": sale.FLAG_SELECT_16BIT}[flags_name]
    seqs = []
    for s, n in enumerate(lens):
        w = inputs.scaled(inputs.LLAMA_32K, n, hq, hkv, f"varlen-{s}")
        w = inputs.replace(w, seed=w.seed + 17 * s)      # the three sequences differ
        seqs.append((w, inputs.make_inputs(w)))
    tau_v = seqs[0][0].tau
    tau = torch.tensor([tau_v], dtype=torch.float32, device="cuda")
    cu = (0,) + tuple(int(x) for x in np.cumsum(lens))
    total = cu[-1]
    qp = torch.cat([t[1][0] for t in seqs], dim=1)[None].cuda()      # [1, H, total, d]
    kp = torch.cat([t[1][1] for t in seqs], dim=1)[None].cuda()
    vp = torch.cat([t[1][2] for t in seqs], dim=1)[None].cuda()
    p = sale.Params(1, hq, hkv, total, block_k=bk, flags=flags, cu_seqlens=cu)
    assert p.words == (lens[0] // bk + 63) // 64
    packed = _pipeline(sale, p, qp, kp, vp, tau)
    assert torch.isfinite(packed["o"].float()).all() and torch.isfinite(packed["od"].float()).all()   # every row written
    for s, (w, (q, k, v)) in enumerate(seqs):
        n = lens[s]
        ps = sale.Params(1, hq, hkv, n, block_k=bk, flags=flags)
        alone = _pipeline(sale, ps, q[None].cuda(), k[None].cuda(), v[None].cuda(), tau)
        t0, t1 = cu[s], cu[s + 1]
        b0, b1 = t0 // 64, t1 // 64
        kb0, kb1 = t0 // bk, t1 // bk
        assert torch.equal(packed["q4"][:, :, t0:t1], alone["q4"]) and torch.equal(packed["k4"][:, :, t0:t1], alone["k4"])
        assert torch.equal(packed["qs"][:, :, b0:b1], alone["qs"]) and torch.equal(packed["ks"][:, :, kb0:kb1], alone["ks"])
        assert torch.equal(packed["m"][:, :, t0:t1], alone["m"]) and torch.equal(packed["l"][:, :, t0:t1], alone["l"])
        assert torch.equal(packed["counts"][:, :, b0:b1], alone["counts"]), s
        wa = ps.words
        assert torch.equal(packed["mask"][:, :, b0:b1, :wa], alone["mask"]), s
        assert not packed["mask"][:, :, b0:b1, wa:].any()              # words beyond the sequence's own length stay 0
        for name in ("o", "od", "lse", "lsed"):
            assert torch.equal(packed[name][:, :, t0:t1], alone[name]), (s, name)
        if flags_name == "16bit":
            continue
        # the oracle, called on this sequence alone (a few units)
        geo = so.Geometry(n, 128, 64, bk, 1, 4, stats_causal=(flags_name == "stats_causal"),
                          segment=4 if flags_name == "segment" else 0)
        qf, kf, vf = f32(q), f32(k), f32(v)
        kc, oks = so.quantize_blocks(kf, bk)
        bits = words_to_bool(alone["mask"][0].cpu().numpy(), ps.n_k)
        for h, i in ((0, geo.n_q - 1), (3, geo.n_q // 2), (2, 0)):
            rs = slice(i * 64, (i + 1) * 64)
            qc, oqs = so.quantize_blocks(qf[h, rs][None], 64)
            row, margin, mthr, *_ = so.select_row(geo, i, qf[h, rs], kf[h // 2], qc[0], kc[h // 2], float(oqs[0, 0]), oks[h // 2],
                                                  tau_v)
            hard, _ = compare_mask_row(bits[h, i], row, margin, mthr)
            assert hard == 0, (s, h, i)
            ref, ref_lse = so.attention_block(geo, i, qf[h, rs], kf[h // 2], vf[h // 2], bits[h, i])
            check_output(f32(packed["o"][0, h, t0 + i * 64:t0 + (i + 1) * 64]), ref, f"varlen seq {s} h{h} i{i}")
            np.testing.assert_allclose(packed["lse"][0, h, t0 + i * 64:t0 + (i + 1) * 64].cpu().numpy(), ref_lse, rtol=0, atol=LSE_ATOL)


def test_varlen_arguments_are_validated(sale):
    import ctypes
    lib = sale.raw()
    f = ctypes.c_void_p(0x1000)      # never dereferenced

    def rc(p):
        return lib.sale_dense_attn(ctypes.byref(p.c()), f, f, f, f, None, f, 16, None)

    assert rc(sale.Params(1, 4, 2, 1024, cu_seqlens=(0, 256, 1024))) == -4           # fine: only the workspace is short
    assert rc(sale.Params(1, 4, 2, 1024, cu_seqlens=(0, 250, 1024))) == -2           # not a multiple of 64
    assert rc(sale.Params(1, 4, 2, 1024, cu_seqlens=(0, 512, 512, 1024))) == -2      # empty sequence
    assert rc(sale.Params(1, 4, 2, 1024, cu_seqlens=(0, 256, 960))) == -2            # does not end at seq_len
    assert rc(sale.Params(1, 4, 2, 1024, cu_seqlens=(64, 256, 1024))) == -2          # does not start at 0
    assert rc(sale.Params(2, 4, 2, 1024, cu_seqlens=(0, 256, 1024))) == -2           # packed batches are batch = 1
    assert rc(sale.Params(1, 4, 2, 1024, flags=sale.FLAG_ATTN_INT8_QK, cu_seqlens=(0, 256, 1024))) == -3
    big = sale.Params(1, 1, 1, 2 * 262144, cu_seqlens=(0, 262144, 2 * 262144))       # two maximal sequences: accepted
    assert sale.workspace_bytes(big, sale.WS_SELECT) > 0
    assert sale.workspace_bytes(sale.Params(1, 1, 1, 2 * 262144), sale.WS_SELECT) == 0   # as ONE sequence it is too long

"""Threshold sweep at 64K tokens on the Llama-3.1-8B layer shape: five thresholds
chosen (by bisection on the GPU mask) to give about 5, 10, 20, 40 and 60 % kept
blocks; at every point the mask and the sparse output of sampled (head, query
block) units are checked against the oracle and density, stage times and errors
are printed."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs
from tests.parity_utils import check_output, compare_mask_row, words_to_bool

pytestmark = pytest.mark.gpu

TARGETS = (0.05, 0.10, 0.20, 0.40, 0.60)


def _time(fn, n=2):
    fn()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(n):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n


def test_threshold_sweep_64k():
    from paper_2505_24179_amd import sale
    w = inputs.LLAMA_64K
    q, k, v = inputs.make_inputs(w)
    p = sale.Params(1, w.n_q_heads, w.n_kv_heads, w.seq_len)
    dev = torch.device("cuda:0")
    qd, kd, vd = (t.unsqueeze(0).to(dev) for t in (q, k, v))
    q4, k4, qs, ks = sale.quantize_qk(p, qd, kd)
    ws_sel = torch.empty(sale.workspace_bytes(p, sale.WS_SELECT), dtype=torch.uint8, device=dev)
    ws_att = torch.empty(sale.workspace_bytes(p, sale.WS_SPARSE_ATTN), dtype=torch.uint8, device=dev)
    causal = w.n_q_heads * p.n_q * (p.n_q + 1) // 2
    o = torch.empty_like(qd)

    def density(tau_value):
        tau = torch.tensor([tau_value], dtype=torch.float32, device=dev)
        mask, counts, _, _ = sale.select(p, qd, kd, q4, k4, qs, ks, tau, ws=ws_sel)
        return int(counts.sum()) / causal, mask, counts, tau

    t_dense = _time(lambda: sale.dense_attn(p, qd, kd, vd, out=o, ws=ws_att))
    t_quant = _time(lambda: sale.quantize_qk(p, qd, kd, out=(q4, k4, qs, ks)))
    geo = so.Geometry(w.seq_len, w.head_dim)
    rng = np.random.default_rng(5)
    units = [(int(rng.integers(0, w.n_q_heads)), int(rng.integers(8, p.n_q))) for _ in range(5)] + [(0, p.n_q - 1)]
    kcache = {}
    rows_out = []
    for target in TARGETS:
        lo, hi = 1e-7, 0.9              # density decreases with tau: bisect in log space
        for _ in range(18):
            mid = float(np.sqrt(lo * hi))
            d, *_ = density(mid)
            if d > target:
                lo = mid
            else:
                hi = mid
        tau_value = float(np.float32(np.sqrt(lo * hi)))
        d, mask, counts, tau = density(tau_value)
        t_sel = _time(lambda: sale.select(p, qd, kd, q4, k4, qs, ks, tau, out=(mask, counts), ws=ws_sel))
        t_sp = _time(lambda: sale.sparse_attn(p, qd, kd, vd, mask, counts, out=o, ws=ws_att))
        hard = soft = 0
        worst = mean_sum = 0.0
        for h, i in units:
            g = h // w.group
            if g not in kcache:
                kf = k[g].float().numpy()
                kc, oks = so.quantize_blocks(kf[None], 64)
                kcache[g] = (kf, kc[0], oks[0], v[g].float().numpy())
            kf, kc, oks, vf = kcache[g]
            rs = slice(i * 64, (i + 1) * 64)
            qf = q[h, rs].float().numpy()
            qc, oqs = so.quantize_blocks(qf[None], 64)
            row, margin, mthr, *_ = so.select_row(geo, i, qf, kf, qc[0], kc, float(oqs[0, 0]), oks, tau_value)
            got = words_to_bool(mask[0, h, i].cpu().numpy(), p.n_k)
            a, b = compare_mask_row(got, row, margin, mthr)
            hard += a; soft += b
            ref, _ = so.attention_block(geo, i, qf, kf, vf, got)
            mx, mn = check_output(o[0, h, rs].float().cpu().numpy(), ref, f"tau={tau_value:.3g} h{h} i{i}")
            worst = max(worst, mx); mean_sum += mn
        assert hard == 0 and soft <= 2
        rows_out.append((target, tau_value, d, t_sel, 100 * (t_quant + t_sel) / t_dense, t_sp, t_dense / t_sp,
                         worst, mean_sum / len(units)))
        print(f"[sweep] target {target:.2f} tau {tau_value:.3e} density {d:.4f} select {t_sel:.2f} ms "
              f"overhead {100 * (t_quant + t_sel) / t_dense:.1f}% sparse {t_sp:.2f} ms speedup {t_dense / t_sp:.2f}x "
              f"max|err| {worst:.3g} mean|err| {mean_sum / len(units):.3g}", flush=True)
    print(f"[sweep] dense {t_dense:.2f} ms, quantize {t_quant:.3f} ms")
    dens = [r[2] for r in rows_out]
    assert all(dens[i] < dens[i + 1] for i in range(len(dens) - 1))      # density rises as tau falls
    assert abs(dens[2] - 0.20) < 0.02 and abs(dens[3] - 0.40) < 0.03

"""Pins for the oracle's per-head threshold calibration (Sec. 3.3)."""
import math

import numpy as np
import torch

from oracle import sale_oracle as so
from paper_2505_24179_amd import inputs


def test_calibration_error_closed_form():
    o = np.array([[1.0, -2.0], [0.5, 0.0], [3.0, 1.0]])
    o2 = np.array([[0.0, -2.0], [0.5, 1.0], [3.5, 1.0]])
    assert so.calibration_error(o, o2) == (1.0 + 1.0 + 0.5) / 3      # ||.||_1 over all entries, divided by N = 3 rows
    assert so.calibration_error(o, o) == 0.0


def _case():
    w = inputs.scaled(inputs.TOY, 1024, 1, 1, "calib-1k")
    q, k, v = inputs.make_inputs(w)
    qf, kf, vf = q.float().numpy()[0], k.float().numpy()[0], v.float().numpy()[0]
    qc, qs = so.quantize_blocks(qf[None], 64)
    kc, ks = so.quantize_blocks(kf[None], 64)
    return so.Geometry(w.seq_len, w.head_dim), qf, kf, vf, qc[0], kc[0], qs[0], ks[0]


def _brute_force_err(geo, qf, kf, vf, mask):
    """Err of a given block mask against full attention, with torch softmax only."""
    n = geo.seq_len
    q, k, v = (torch.from_numpy(x).double() for x in (qf, kf, vf))
    s = q @ k.T / math.sqrt(geo.head_dim)
    causal = torch.tril(torch.ones(n, n, dtype=torch.bool))
    keep = torch.from_numpy(np.repeat(np.repeat(mask, 64, axis=0), 64, axis=1)) & causal
    o_full = torch.softmax(s.masked_fill(~causal, float("-inf")), dim=1) @ v
    o_sale = torch.softmax(s.masked_fill(~keep, float("-inf")), dim=1) @ v
    return float((o_full - o_sale).abs().sum() / n)


def test_calibrate_halves_until_below_theta():
    geo, qf, kf, vf, qc, kc, qs, ks = _case()
    tau_all, n_all, errs = so.calibrate_head(geo, qf, kf, vf, qc, kc, qs, ks, 0.008, 0.0, 6)   # theta 0: never satisfied
    assert n_all == 6 and len(errs) == 7 and tau_all == 0.008 / 64
    assert errs[0] > errs[-1] > 0                      # smaller tau keeps more blocks
    # every reported Err equals the brute-force Err of the mask selected at that tau
    for n in (0, 3, 6):
        mask, *_ = so.select_head(geo, qf, kf, qc, kc, qs, ks, 0.008 / 2 ** n)
        assert abs(errs[n] - _brute_force_err(geo, qf, kf, vf, mask)) < 1e-12
    # a theta between two consecutive errors stops exactly there
    for n in range(1, 7):
        if errs[n] < errs[n - 1] * 0.98 and all(e > errs[n] for e in errs[:n]):
            theta = 0.5 * (errs[n] + min(errs[:n]))
            tau, halvings, tried = so.calibrate_head(geo, qf, kf, vf, qc, kc, qs, ks, 0.008, theta, 6)
            assert halvings == n and tau == 0.008 / 2 ** n
            assert tried[-1] < theta and all(e >= theta for e in tried[:-1])
    # a generous theta keeps tau0, and the result is monotone in theta
    tau, halvings, _ = so.calibrate_head(geo, qf, kf, vf, qc, kc, qs, ks, 0.008, 10.0, 6)
    assert (tau, halvings) == (0.008, 0)
    taus = [so.calibrate_head(geo, qf, kf, vf, qc, kc, qs, ks, 0.008, th, 6)[0] for th in (errs[5] * 1.01, errs[2] * 1.01, 1.0)]
    assert taus[0] <= taus[1] <= taus[2]

"""Pins for the oracle's masked attention (Eq. 1, Eq. 2)."""
import math

import numpy as np
import torch

from oracle import sale_oracle as so


def _case(n=256, d=32, seed=0):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(n, d, generator=g, dtype=torch.float64)
    k = torch.randn(n, d, generator=g, dtype=torch.float64)
    v = torch.randn(n, d, generator=g, dtype=torch.float64)
    return q, k, v


def test_all_selected_equals_brute_force_dense_causal():
    q, k, v = _case()
    n, d = q.shape
    geo = so.Geometry(n, d, 64, 32)
    o, lse = so.attention_head(geo, q.numpy(), k.numpy(), v.numpy(), so.dense_mask(geo))
    s = q @ k.T / math.sqrt(d)
    s = s.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), 1), float("-inf"))
    ref = torch.softmax(s, dim=1) @ v
    np.testing.assert_allclose(o, ref.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, dim=1).numpy(), rtol=1e-12)


def test_probability_rows_sum_to_one_and_respect_masks():
    q, k, v = _case(seed=1)
    n, d = q.shape
    geo = so.Geometry(n, d, 64, 64)
    rng = np.random.default_rng(0)
    for i in range(geo.n_q):
        row = np.zeros(geo.n_k, dtype=bool)
        row[: i + 1] = rng.random(i + 1) < 0.5
        row[i] = True
        p = so.attention_probs_block(geo, i, q[i * 64:(i + 1) * 64].numpy(), k.numpy(), row)
        np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=1e-13)
        assert np.all(p >= 0)
        rows = i * 64 + np.arange(64)
        cols = np.arange(n)
        future = cols[None, :] > rows[:, None]
        assert np.all(p[future] == 0)                                   # causal part of M
        assert np.all(p[:, ~np.repeat(row, 64)] == 0)                   # sparse part of M


def test_dropped_blocks_renormalisation_identity():
    """Dropping blocks only renormalises: O~_r = (O_r - sum_dropped P_rc V_c) / (1 - delta_r)."""
    q, k, v = _case(seed=2)
    n, d = q.shape
    geo = so.Geometry(n, d, 64, 64)
    rng = np.random.default_rng(1)
    mask = so.dense_mask(geo) & (rng.random((geo.n_q, geo.n_k)) < 0.6)
    mask[np.arange(geo.n_q), np.arange(geo.n_q)] = True
    o_sparse, _ = so.attention_head(geo, q.numpy(), k.numpy(), v.numpy(), mask)
    s = q @ k.T / math.sqrt(d)
    s = s.masked_fill(torch.triu(torch.ones(n, n, dtype=torch.bool), 1), float("-inf"))
    p = torch.softmax(s, dim=1)
    keep = torch.from_numpy(np.repeat(np.repeat(mask, 64, axis=0), 64, axis=1))
    p_drop = p * (~keep)
    delta = p_drop.sum(dim=1, keepdim=True)
    expect = (p @ v - p_drop @ v) / (1 - delta)
    np.testing.assert_allclose(o_sparse, expect.numpy(), rtol=1e-10, atol=1e-12)
    bound = 2 * delta / (1 - delta) * v.abs().max()
    assert np.all(np.abs(o_sparse - (p @ v).numpy()).max(axis=1) <= bound[:, 0].numpy() + 1e-12)

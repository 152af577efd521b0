"""Pins of the oracle's low-precision second product (Sec. 3.4 "Integration with SageAttention": the quantized
attention the method builds on; P and V in FP8 E4M3, fp32 accumulation)."""
import math

import numpy as np
import pytest
import torch

from oracle import sale_oracle as so


def test_fp8_grid_literals():
    f = so.fp8_e4m3_round
    lit = {0.0: 0.0, 1.0: 1.0, 448.0: 448.0, 500.0: 448.0, -1000.0: -448.0, 464.0: 448.0,
           1.0625: 1.0,             # halfway between 1 and 1.125: even mantissa 0
           1.1875: 1.25,            # halfway between 1.125 and 1.25: even mantissa 2
           1.07: 1.125, 0.3: 0.3125, 17.0: 16.0, 19.0: 20.0, 18.0: 18.0, 416.0: 416.0, 432.0: 448.0,
           2.0 ** -6: 2.0 ** -6,    # smallest normal
           2.0 ** -9: 2.0 ** -9,    # smallest subnormal
           2.0 ** -10: 0.0,         # halfway between 0 and the smallest subnormal: even = 0
           3 * 2.0 ** -10: 2.0 ** -8,   # halfway between 1 and 2 subnormal steps: even = 2 steps
           0.0146: 0.0146484375,    # 7.5 subnormal steps -> 8 steps = the smallest normal... (0.0146 / 2^-9 = 7.475 -> 7 steps)
           -0.02: -0.01953125}
    lit[0.0146] = 7 * 2.0 ** -9
    for x, want in lit.items():
        assert float(f(x)) == want, (x, float(f(x)), want)
    enc = so.fp8_e4m3_encode(np.array([0.0, 1.0, -448.0, 2.0 ** -9, 2.0 ** -6, 1.125, -0.5, 448.0]))
    assert enc.tolist() == [0x00, 0x38, 0xFE, 0x01, 0x08, 0x39, 0xB0, 0x7E]


def test_fp8_round_matches_the_library_conversion():
    """Library special case: torch's float8_e4m3fn cast (round to nearest even) on values inside the range."""
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(size=4000) * 3, rng.uniform(-448, 448, 4000), rng.uniform(-0.05, 0.05, 4000),
                        np.array([0.0, 448.0, -448.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10])]).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn)
    np.testing.assert_array_equal(so.fp8_e4m3_round(x), lib.float().numpy().astype(np.float64))
    np.testing.assert_array_equal(so.fp8_e4m3_encode(so.fp8_e4m3_round(x)) & 0x7F, lib.view(torch.uint8).numpy() & 0x7F)


def test_quantize_v_fp8_invariants():
    rng = np.random.default_rng(1)
    v = (rng.normal(size=(2, 256, 16)) * rng.uniform(0.1, 5, size=(1, 1, 16))).astype(np.float32)
    v[0, :, 3] = 0.0                                   # an all-zero channel
    v[1, :, 5] = np.float32(0.75)                      # a constant channel: every value becomes 448
    val, scale = so.quantize_v_fp8(v)
    assert np.all(np.abs(val) <= 448) and scale[0, 3] == 1.0 and np.all(val[0, :, 3] == 0)
    assert np.all(val[1, :, 5] == 448) and scale[1, 5] == np.float32(0.75) / np.float32(448)
    nz = np.abs(v).max(axis=1) > 0
    assert np.all(np.abs(val).max(axis=1)[nz] == 448)                       # every channel uses the top of the grid
    # within half a step of the grid at the value's own exponent (2^-4 relative), or half a subnormal step
    err = np.abs(val * scale[:, None, :].astype(np.float64) - v)
    bound = np.maximum(np.abs(v) * 2.0 ** -4, scale[:, None, :] * 2.0 ** -10) * (1 + 1e-6)
    assert np.all(err <= bound)
    np.testing.assert_array_equal(so.fp8_e4m3_round(val), val)              # already on the grid
    # scaling a channel by a power of two changes its scale, not its values
    v2 = v.copy(); v2[:, :, 7] *= 4
    val2, scale2 = so.quantize_v_fp8(v2)
    np.testing.assert_array_equal(val2, val)
    assert scale2[0, 7] == 4 * scale[0, 7]


def _geo(n):
    return so.Geometry(n, 16, 64, 64, 1, 2)


def test_fp8_second_product_closed_forms():
    """Uniform rows: every probability is 1 -> P8 = 448 exactly -> O = the mean of the (quantized) V rows.
    One-hot rows: the other keys fall below half the smallest subnormal -> O = that V row.  A channel of ones:
    numerator and denominator are the same sum -> exactly 1 (the rows of P sum to 1)."""
    n, d = 256, 16
    rng = np.random.default_rng(2)
    v = rng.normal(size=(1, n, d)).astype(np.float32)
    v[0, :, 0] = 1.0
    val, scale = so.quantize_v_fp8(v)
    vq = val[0] * scale[0].astype(np.float64)                     # what the second product sees
    geo = _geo(n)
    i = 2
    row = so.dense_mask(geo)[i].copy(); row[1] = False
    rows = i * 64 + np.arange(64)
    s = np.zeros((64, n))
    o, lse = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], row)
    for r in (0, 17, 63):
        keys = [c for c in range(n) if c <= rows[r] and row[c // 64]]
        np.testing.assert_allclose(o[r], vq[keys].mean(axis=0), rtol=1e-12, atol=1e-12)
        assert abs(lse[r] - math.log(len(keys))) < 1e-12
    # (1 up to the fp32 rounding of the scale 1 / 448: numerator and denominator are the same sum)
    ones = float(np.float32(1.0) / np.float32(448.0)) * 448.0
    np.testing.assert_allclose(o[:, 0], ones, rtol=0, atol=1e-12)
    s = np.full((64, n), -40.0)
    hot = 70
    s[:, hot] = 0.0
    o, lse = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], so.dense_mask(geo)[i])
    np.testing.assert_allclose(o, np.broadcast_to(vq[hot], o.shape), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse, 0.0, atol=1e-12)
    # random scores: the ones channel is still exactly 1, whatever the order in which the maximum was found
    s = rng.normal(size=(64, n)) * 3
    s[:, 200:] += 6                                               # the maximum grows late: exercises the rescale
    o, _ = so.attention_block_fp8pv_from_scores(geo, 3, s, val[0], scale[0], so.dense_mask(geo)[3])
    np.testing.assert_allclose(o[:, 0], ones, rtol=0, atol=1e-12)


def test_fp8_second_product_is_close_to_the_exact_one():
    """Each P8 and each V8 is within 2^-4 relative of its exact value (above the subnormal range), so O moves by
    at most about 2^-3 max|V|; on random data far less, because the errors average out.  A wrong scale, a
    transposed operand, a missing rescale or a denominator taken from unrounded probabilities breaks one of the
    bounds or the ones channel above."""
    n, d = 512, 16
    rng = np.random.default_rng(3)
    v = rng.normal(size=(1, n, d)).astype(np.float32)
    val, scale = so.quantize_v_fp8(v)
    geo = _geo(n)
    s = rng.normal(size=(64, n)) * 2.5
    worst = 0.0
    for i in (0, 3, 7):
        row = so.dense_mask(geo)[i] & (rng.random(geo.n_k) < 0.7)
        row[geo.j_last(i)] = True; row[0] = True
        o8, l8 = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], row)
        o, l = so.attention_block_from_scores(geo, i, s, v[0], row)
        err = np.abs(o8 - o)
        assert err.max() <= 2.0 ** -3 * np.abs(v).max()
        assert err.mean() < 1.5e-2
        worst = max(worst, err.max())
        assert np.abs(l8 - l).max() < 2.0 ** -4 + 1e-9            # the denominator: each term within 2^-4 relative
    assert worst > 1e-3                                            # the quantization is really there


def test_int8qk_fp8pv_composes_the_two():
    n, d = 256, 128
    rng = np.random.default_rng(4)
    q = rng.normal(size=(n, d)).astype(np.float32); k = (rng.normal(size=(n, d)) + 0.5).astype(np.float32)
    v = rng.normal(size=(n, d)).astype(np.float32)
    qc, qs, kc, ks, mean = so.quantize_qk_int8(q[None], k[None])
    val, scale = so.quantize_v_fp8(v[None])
    geo = so.Geometry(n, d, 64, 64, 1, 2)
    i, row = 3, so.dense_mask(so.Geometry(n, d, 64, 64, 1, 2))[3]
    rs = slice(192, 256)
    o, lse = so.attention_block_int8qk_fp8pv(geo, i, qc[0][rs], qs[0, i], kc[0], ks[0], val[0], scale[0], row, q[rs], mean[0])
    a = so.int_products(qc[0][rs], kc[0]).astype(np.float64)
    s = a * float(qs[0, i]) * np.repeat(ks[0].astype(np.float64), 64)[None, :] / math.sqrt(d)
    o2, lse2 = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], row)
    np.testing.assert_array_equal(o, o2)
    np.testing.assert_allclose(lse - lse2, q[rs].astype(np.float64) @ mean[0].astype(np.float64) / math.sqrt(d), atol=1e-12)
    o16, _ = so.attention_block_int8qk(geo, i, qc[0][rs], qs[0, i], kc[0], ks[0], v, row)
    assert 1e-4 < np.abs(o - o16).max() < 0.1


def test_fp8_flip_slack_bounds_the_effect_of_a_perturbed_argument():
    """arg_tol: with tolerance 0 the slack is 0; shifting every (row, key block) group of scores by up to
    arg_tol / 2 (so that s - m moves by up to arg_tol) changes O and lse by no more than the slack plus the
    first-order effect of the shift itself; rows with no probability near a midpoint have zero slack, and some
    rows do flip (the bound is not vacuous)."""
    n, d = 512, 16
    rng = np.random.default_rng(5)
    v = rng.normal(size=(1, n, d)).astype(np.float32)
    val, scale = so.quantize_v_fp8(v)
    geo = _geo(n)
    i, row = 7, so.dense_mask(_geo(n))[7]
    s = rng.normal(size=(64, n)) * 2.5
    o, lse, os0, ls0 = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], row, arg_tol=0.0)
    assert not os0.any() and not ls0.any()
    o_b, lse_b = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], row)
    np.testing.assert_array_equal(o, o_b); np.testing.assert_array_equal(lse, lse_b)
    tol = np.full(geo.n_k, 2e-3); tol[0] = 8e-3                     # one tolerance per key block
    _, _, o_slack, lse_slack = so.attention_block_fp8pv_from_scores(geo, i, s, val[0], scale[0], row, arg_tol=tol)
    assert (lse_slack > 0).sum() > 8 and (o_slack >= 0).all()
    seen = 0.0
    for trial in range(8):
        u = rng.uniform(-0.5, 0.5, size=(64, geo.n_k)) * tol[None, :]
        o2, lse2 = so.attention_block_fp8pv_from_scores(geo, i, s + np.repeat(u, 64, axis=1), val[0], scale[0], row)
        first_order = tol.max()                                     # d lse / d s and d O / d s (|V| <= amax) of the exact map
        assert (np.abs(lse2 - lse) <= lse_slack + first_order).all()
        assert (np.abs(o2 - o) <= o_slack + 2 * first_order * np.abs(v).max()).all()
        _, e0 = so.attention_block_from_scores(geo, i, s, v[0], row)
        _, e1 = so.attention_block_from_scores(geo, i, s + np.repeat(u, 64, axis=1), v[0], row)
        seen = max(seen, np.abs((lse2 - lse) - (e1 - e0)).max())
    assert seen > 2e-4                                              # codes did flip: not the smooth change of the exact lse
    quiet = lse_slack == 0
    if quiet.any():                                                 # no flip possible: only the first-order effect
        assert (np.abs(lse2 - lse)[quiet] <= first_order).all()

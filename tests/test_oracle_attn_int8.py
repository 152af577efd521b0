"""Pins of the oracle's quantized Computation-Pass (Sec. 3.4 "Integration with SageAttention"): 8-bit Q, K
with K smoothing for the first product, everything else as Eq. 1."""
import math

import numpy as np
import torch

from oracle import sale_oracle as so


def _rand(n, d, seed, shift=0.0):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(n, d, generator=g)
    k = torch.randn(n, d, generator=g) + shift
    v = torch.randn(n, d, generator=g)
    return [t.bfloat16().float().numpy() for t in (q, k, v)]


def test_k_smoothing_leaves_softmax_unchanged_and_has_zero_mean():
    """softmax_j(q . (k_j - c)) = softmax_j(q . k_j) for any constant vector c: checked with the library
    softmax on the smoothed and on the raw keys (fp64), with a K far from zero mean."""
    q, k, v = _rand(256, 32, 1, shift=3.0)
    ks, mean = so.smooth_k(k[None])
    assert mean.shape == (1, 32) and np.abs(mean - 3.0).max() < 0.3
    assert np.abs(ks.astype(np.float64).sum(axis=1)).max() < 256 * 2e-7 * 4      # fp32 rounding of the mean only
    a = torch.softmax(torch.from_numpy(q).double() @ torch.from_numpy(k).double().T / math.sqrt(32), dim=1)
    b = torch.softmax(torch.from_numpy(q).double() @ torch.from_numpy(ks[0]).double().T / math.sqrt(32), dim=1)
    assert (a - b).abs().max() < 1e-12
    # the mean is the exact one rounded once: against a pure-Python exact rational sum
    from fractions import Fraction
    col = [Fraction(float(x)) for x in k[:, 5]]
    assert mean[0, 5] == np.float32(float(sum(col) / len(col)))


def test_int8_codes_follow_the_4bit_quantizer_with_127():
    q, k, v = _rand(128, 16, 2)
    codes, scale = so.quantize_blocks(q[None], 64, 127)
    for b in range(2):
        blk = q[b * 64:(b + 1) * 64]
        amax = np.abs(blk).max()
        assert scale[0, b] == np.float32(amax) / np.float32(127)
        assert np.abs(codes[0, b * 64:(b + 1) * 64]).max() == 127
        deq = codes[0, b * 64:(b + 1) * 64].astype(np.float64) * float(scale[0, b])
        assert np.abs(deq - blk).max() <= 0.5 * float(scale[0, b]) * (1 + 1e-5)   # fp32 rounding of x * (127 / amax)
    c7, s7 = so.quantize_blocks(q[None], 64)
    assert np.abs(c7).max() == 7 and np.allclose(s7 * 7, scale * 127, rtol=1e-6)


def test_int8_attention_is_exact_on_the_8bit_grid():
    """Integer inputs in [-127, 127] with a +-127 in every 64-row block and keys whose mean is exactly zero
    quantize without loss (scale 1), so the quantized pass must equal plain masked attention."""
    n, d = 256, 16
    rng = np.random.default_rng(3)
    q = rng.integers(-3, 4, size=(n, d)).astype(np.float32)
    k = rng.integers(-2, 3, size=(n // 2, d)).astype(np.float32)
    k = np.concatenate([k, -k])                       # zero mean per channel, exactly
    perm = rng.permutation(n)
    k = k[perm]
    v = rng.standard_normal((n, d)).astype(np.float32)
    q[:, d - 1] = 0; k[:, d - 1] = 0
    q[0::64, d - 1] = 127
    k[:, d - 2] = 0
    k[0::64, d - 2] = 127; k[1::64, d - 2] = -127     # keeps the mean zero
    qc, qs, kc, ks, mean = so.quantize_qk_int8(q[None], k[None])
    assert np.all(mean == 0) and np.all(qs == 1) and np.all(ks == 1)
    geo = so.Geometry(n, d, 64, 32, 1, 2)
    rng2 = np.random.default_rng(4)
    for i in range(geo.n_q):
        row = so.dense_mask(geo)[i] & (rng2.random(geo.n_k) < 0.6)
        row[geo.j_last(i) - 1] = True
        o8, l8 = so.attention_block_int8qk(geo, i, qc[0][i * 64:(i + 1) * 64], qs[0, i], kc[0], ks[0], v, row)
        o, l = so.attention_block(geo, i, q[i * 64:(i + 1) * 64], k, v, row)
        np.testing.assert_allclose(o8, o, rtol=0, atol=1e-12)
        np.testing.assert_allclose(l8, l, rtol=0, atol=1e-12)


def test_int8_scores_within_the_quantization_bound_of_the_exact_ones():
    """|S8 - S| <= (s_q/2 |k'|_1 + s_k/2 |q|_1 + d s_q s_k / 4) / sqrt(d) element by element (k' the smoothed
    key, each operand off by at most half a step), up to the row constant q . mean that the softmax cancels;
    and the outputs agree to the accuracy the cited method claims (a wrong scale, a transposed operand or a
    missing smoothing term breaks either)."""
    n, d = 512, 128
    q, k, v = _rand(n, d, 5, shift=1.5)
    qc, qs, kc, ks, mean = so.quantize_qk_int8(q[None], k[None])
    kprime = k.astype(np.float64) - mean[0].astype(np.float64)
    geo = so.Geometry(n, d, 64, 64, 1, 2)
    worst = 0.0
    for i in (0, 3, 7):
        rs = slice(i * 64, (i + 1) * 64)
        a = so.int_products(qc[0][rs], kc[0]).astype(np.float64)
        s8 = a * float(qs[0, i]) * np.repeat(ks[0].astype(np.float64), 64)[None, :] / math.sqrt(d)
        s = q[rs].astype(np.float64) @ kprime.T / math.sqrt(d)
        sq, sk = float(qs[0, i]), np.repeat(ks[0].astype(np.float64), 64)
        bound = (0.5 * sq * np.abs(kprime).sum(1)[None, :] + 0.5 * sk[None, :] * np.abs(q[rs]).sum(1)[:, None]
                 + d * sq * sk[None, :] / 4) / math.sqrt(d)
        assert np.all(np.abs(s8 - s) <= bound * (1 + 1e-9))
        assert np.abs(s8 - s).max() > 1e-4                       # the quantization is really there
        row = so.dense_mask(geo)[i]
        o8, _ = so.attention_block_int8qk(geo, i, qc[0][rs], qs[0, i], kc[0], ks[0], v, row)
        o, _ = so.attention_block(geo, i, q[rs], k, v, row)
        worst = max(worst, np.abs(o8 - o).max())
    assert 1e-5 < worst < 2e-2


def test_int8_lse_with_the_shift_added_back_is_the_lse_of_eq1():
    """The 8-bit logits are those of K minus its mean key: lse(S') = lse(S) - q_r . mean / sqrt(d) exactly when
    nothing is lost to quantization, and within the largest logit error of the row otherwise (a log-sum-exp moves
    by at most the largest change of its arguments).  With q_blk and k_mean given the oracle adds the shift back."""
    n, d = 512, 128
    q, k, v = _rand(n, d, 11, shift=1.5)
    qc, qs, kc, ks, mean = so.quantize_qk_int8(q[None], k[None])
    assert np.abs(mean).max() > 1.0                               # the shift is not negligible here
    kprime = k.astype(np.float64) - mean[0].astype(np.float64)
    geo = so.Geometry(n, d, 64, 64, 1, 2)
    for i in (0, 2, 7):
        rs = slice(i * 64, (i + 1) * 64)
        row = so.dense_mask(geo)[i]
        _, l_raw = so.attention_block_int8qk(geo, i, qc[0][rs], qs[0, i], kc[0], ks[0], v, row)
        _, l_fix = so.attention_block_int8qk(geo, i, qc[0][rs], qs[0, i], kc[0], ks[0], v, row, q_blk=q[rs], k_mean=mean[0])
        _, l_exact = so.attention_block(geo, i, q[rs], k, v, row)
        shift = q[rs].astype(np.float64) @ mean[0].astype(np.float64) / math.sqrt(d)
        np.testing.assert_allclose(l_fix - l_raw, shift, rtol=0, atol=1e-12)
        assert np.abs(shift).max() > 0.5 and np.abs(l_raw - l_exact).max() > 0.5     # without the shift lse is far off
        sq, sk = float(qs[0, i]), np.repeat(ks[0].astype(np.float64), 64)
        bound = (0.5 * sq * np.abs(kprime).sum(1)[None, :] + 0.5 * sk[None, :] * np.abs(q[rs]).sum(1)[:, None]
                 + d * sq * sk[None, :] / 4) / math.sqrt(d)
        assert np.all(np.abs(l_fix - l_exact) <= bound.max(axis=1) * (1 + 1e-9))
        assert np.abs(l_fix - l_exact).max() < 0.05


def test_attention_block_from_scores_is_attention_block():
    q, k, v = _rand(256, 32, 6)
    geo = so.Geometry(256, 32, 64, 32, 1, 2)
    row = so.dense_mask(geo)[2]; row[1] = False
    s = q[128:192].astype(np.float64) @ k.astype(np.float64).T / math.sqrt(32)
    o1, l1 = so.attention_block_from_scores(geo, 2, s, v, row)
    o2, l2 = so.attention_block(geo, 2, q[128:192], k, v, row)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(l1, l2)

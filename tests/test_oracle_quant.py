"""Pins for the oracle's quantizer, nibble packing and integer products
(Sec. 3.2 "4-bit attention weight approximation")."""
import numpy as np
import pytest
import torch

from oracle import sale_oracle as so


def _bf16_normal(shape, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).bfloat16().float().numpy()


@pytest.mark.parametrize("block", [32, 64])
def test_quantizer_invariants(block):
    x = _bf16_normal((3, 256, 128), 1, scale=2.5)
    codes, scale = so.quantize_blocks(x, block)
    assert codes.dtype == np.int8 and scale.dtype == np.float32
    assert np.abs(codes).max() <= 7
    cb = codes.reshape(3, 256 // block, -1)
    # every non-zero block reaches +-7 at its largest element
    assert np.all(np.abs(cb).max(axis=2) == 7)
    xb = x.reshape(3, 256 // block, -1)
    amax = np.abs(xb).max(axis=2)
    np.testing.assert_array_equal(scale, (amax / np.float32(7)).astype(np.float32))
    # reconstruction error at most half a step (plus fp32 rounding of x * inv)
    err = np.abs(xb - cb.astype(np.float64) * scale[:, :, None].astype(np.float64))
    assert np.all(err <= 0.5 * scale[:, :, None] * (1 + 1e-5))
    # idempotent: quantizing the reconstruction returns the same codes
    recon = (cb.astype(np.float32) * scale[:, :, None]).reshape(x.shape)
    codes2, _ = so.quantize_blocks(recon, block)
    np.testing.assert_array_equal(codes2, codes)


def test_quantizer_lossless_grid_and_zero_block():
    rng = np.random.default_rng(5)
    x = rng.integers(-7, 8, size=(2, 128, 16)).astype(np.float32)
    x[:, 0::64, 0] = 7.0            # every 64-row block contains a 7
    x[1, 64:128] = 0.0              # one all-zero block
    codes, scale = so.quantize_blocks(x, 64)
    np.testing.assert_array_equal(codes.astype(np.float32), x)
    np.testing.assert_array_equal(scale, np.ones((2, 2), np.float32))


def test_quantizer_ties_round_to_even_and_sign():
    # amax = 7 -> inv = 1: the values themselves are rounded
    x = np.zeros((1, 2, 8), np.float32)
    x[0, 0] = [7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 6.5]
    codes, scale = so.quantize_blocks(x, 2)
    assert scale[0, 0] == 1.0
    np.testing.assert_array_equal(codes[0, 0], [7, 0, 2, 2, 0, -2, -2, 6])


def test_scale_invariance_of_codes():
    x = _bf16_normal((1, 64, 128), 9)
    c1, s1 = so.quantize_blocks(x, 64)
    c2, s2 = so.quantize_blocks(x * np.float32(4.0), 64)   # power of two: exact
    np.testing.assert_array_equal(c1, c2)
    np.testing.assert_array_equal(s2, s1 * np.float32(4.0))


def test_pack_roundtrip_and_layout():
    rng = np.random.default_rng(2)
    codes = rng.integers(-7, 8, size=(5, 128)).astype(np.int8)
    p = so.pack_int4(codes)
    assert p.shape == (5, 64) and p.dtype == np.uint8
    np.testing.assert_array_equal(so.unpack_int4(p), codes)
    # channel 0 = low nibble, channel 1 = high nibble, two's complement
    one = np.array([[-1, 3] + [0] * 126], np.int8)
    assert so.pack_int4(one)[0, 0] == 0x3F
    one = np.array([[5, -7] + [0] * 126], np.int8)
    assert so.pack_int4(one)[0, 0] == 0x95


def test_int_products_brute_force():
    rng = np.random.default_rng(3)
    qc = rng.integers(-7, 8, size=(5, 12)).astype(np.int8)
    kc = rng.integers(-7, 8, size=(7, 12)).astype(np.int8)
    a = so.int_products(qc, kc)
    assert a.dtype == np.int32 and a.shape == (5, 7)
    for r in range(5):
        for c in range(7):
            assert int(a[r, c]) == sum(int(qc[r, t]) * int(kc[c, t]) for t in range(12))
    # extreme case: all +-7 over d = 128 reaches +-6272
    q7 = np.full((1, 128), 7, np.int8)
    assert so.int_products(q7, -q7)[0, 0] == -6272


def test_dequantize_matches_definition():
    a = np.array([[10, -3]], np.int32)
    s = so.dequantize(a, 0.5, 0.25, 16)
    np.testing.assert_allclose(s, [[10 * 0.5 * 0.25 / 4, -3 * 0.5 * 0.25 / 4]], rtol=0, atol=0)

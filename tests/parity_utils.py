"""Helpers shared by the GPU parity tests: run the oracle on the same seeded
inputs and compare.  Imports the oracle and the input generator only."""
from __future__ import annotations

import numpy as np
import torch

from oracle import sale_oracle as so

MAX_ABS_TOL = 2e-2     # attention output, bf16 inputs, against the fp64 oracle
MEAN_ABS_TOL = 2e-3
# lse = m + ln(l): the kernel sums the bf16-rounded probabilities it feeds to the second product (so that
# numerator and denominator of O agree); bf16 keeps 8 significant bits, so each term is off by <= 2^-8
# relative, all terms are positive, hence l is off by <= 2^-8 relative and ln(l) by <= 3.9e-3; fp32
# exp2 / log and the running max add < 1e-3.
LSE_ATOL = 5e-3
# FP8 second product: both sides sum the SAME kind of rounded probabilities, so the bars above hold unless a
# probability lies so close to the midpoint of two E4M3 codes that the kernel's fp32 argument and the oracle's
# fp64 one round it to different neighbours.  The oracle reports, per row, how far such flips can move O and lse
# (its arg_tol); that slack is added to the bars, so rows none of whose probabilities can flip keep the bars above.
# The kernel's argument error: it reads the integer accumulators as floats offset by 1.5 * 2^23 raw units and
# takes the offset out inside the scaling FMA, exp2(fma(S, c_j, -(m - log2 448 + 1.5 * 2^23 c_j))) with c_j =
# s_q s_k[j] log2(e) / sqrt(d); the subtrahend (magnitude up to 1.5 * 2^23 c_j + 2^7) is rounded to fp32 when it
# is formed and when the offset product is, and the running maximum carries the same two roundings of the block it
# came from: 4 half-ulps, 2^-22 relative to the largest subtrahend of the row, plus 2^-21 for the hardware exp2.
def fp8_arg_tol(s_q: float, s_k: np.ndarray, head_dim: int) -> np.ndarray:
    """Absolute tolerance (natural-log units) of the FP8 kernel's exponent argument, one per key block."""
    cj = float(s_q) * np.asarray(s_k, dtype=np.float64) * np.log2(np.e) / np.sqrt(head_dim)
    worst = 1.5 * 2.0 ** 23 * cj.max() + 2.0 ** 7
    return np.full(cj.shape, np.log(2.0) * 2.0 ** -22 * worst + 2.0 ** -21)


BORDER_REL = 1e-5      # mask decisions this close to the threshold may differ


def f32(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy()


def words_to_bool(words: np.ndarray, n_k: int) -> np.ndarray:
    """uint64 words [..., W] -> bool [..., n_k]."""
    w = np.ascontiguousarray(words).view(np.uint64)
    bits = (w[..., :, None] >> np.arange(64, dtype=np.uint64)[None, :]) & np.uint64(1)
    return bits.reshape(*w.shape[:-1], -1)[..., :n_k].astype(bool)


def oracle_quantize(q: torch.Tensor, k: torch.Tensor, bq=64, bk=64):
    qc, qs = so.quantize_blocks(f32(q), bq)
    kc, ks = so.quantize_blocks(f32(k), bk)
    return qc, qs, kc, ks


def compare_mask_row(gpu_row: np.ndarray, ora_row: np.ndarray, margin: np.ndarray, margin_thr: np.ndarray):
    """-> (n_mismatch_outside_band, n_borderline_mismatch)"""
    diff = gpu_row != ora_row
    if not diff.any():
        return 0, 0
    border = so.is_borderline(np.nan_to_num(margin, nan=1e30), np.nan_to_num(margin_thr, nan=0.0), BORDER_REL)
    return int((diff & ~border).sum()), int((diff & border).sum())


def check_output(o_gpu: np.ndarray, o_ref: np.ndarray, what: str = ""):
    err = np.abs(o_gpu.astype(np.float64) - o_ref)
    assert err.max() <= MAX_ABS_TOL, f"{what}: max abs err {err.max():.4g} > {MAX_ABS_TOL}"
    assert err.mean() <= MEAN_ABS_TOL, f"{what}: mean abs err {err.mean():.4g} > {MEAN_ABS_TOL}"
    return float(err.max()), float(err.mean())


def check_output_fp8(o_gpu: np.ndarray, o_ref: np.ndarray, o_slack: np.ndarray, what: str = ""):
    """Output of the FP8 second product against the oracle's; o_slack: the oracle's flip slack (see fp8_arg_tol)."""
    err = np.abs(o_gpu.astype(np.float64) - o_ref)
    over = err - o_slack
    assert over.max() <= MAX_ABS_TOL, f"{what}: max abs err beyond the flip slack {over.max():.4g} > {MAX_ABS_TOL}"
    assert err.mean() <= MEAN_ABS_TOL, f"{what}: mean abs err {err.mean():.4g} > {MEAN_ABS_TOL}"
    return float(err.max()), float(err.mean())


def check_lse_fp8(lse_gpu: np.ndarray, lse_ref: np.ndarray, lse_slack: np.ndarray, what: str = ""):
    """lse of the FP8 second product against the oracle's; lse_slack as o_slack above."""
    finite = np.isfinite(lse_ref)
    assert np.array_equal(np.isfinite(lse_gpu), finite), f"{what}: empty rows differ"
    err = np.abs(lse_gpu.astype(np.float64) - lse_ref)[finite]
    if err.size == 0:
        return 0.0
    over = err - lse_slack[finite]
    assert over.max() <= LSE_ATOL, f"{what}: lse max abs err beyond the flip slack {over.max():.4g} > {LSE_ATOL}"
    return float(err.max())

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

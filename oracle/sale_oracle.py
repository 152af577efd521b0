"""CPU oracle for SALE's prefill attention path (arXiv 2505.24179).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what
the GPU library must compute.  Only the test-suite, the smoke check and the
`cpu_baseline` leg of the benchmark may import it; no product code path does.
It shares nothing with the HIP sources (no tables, no helpers, no packing
code) and never imports the GPU binding.

Everything is numpy.  Floating point is fp64 except where the method itself
fixes a precision: the 4-bit quantizer works in fp32 (the codes are integer
decisions, and both sides must take them in the same precision).

Notation follows the paper: Q, K, V are N x d per head, b_q / b_k the block
sizes, N_q = N / b_q, N_k = N / b_k, M_bs the block mask, S the attention
weights, m~ / l~ the sink-local statistics, tau the threshold.

Pins (tests/test_oracle_*.py): quantizer invariants and the lossless grid;
integer products against pure-Python brute force; the hand-derived 4x4-block
toy; the lossless-grid case of the mask against a library logsumexp; Eq. 3
against Eq. 4; structural invariants of the mask; attention with every block
selected against brute-force causal softmax; the renormalisation identity for
dropped blocks; the 8-bit Computation-Pass against the unquantized one (exact on
the 8-bit grid, within the quantization-step bound elsewhere) and the softmax
invariance of the K smoothing; the FP8 grid against literal values and a library conversion, the FP8 second
product against closed forms (uniform and one-hot rows, a ones channel) and an error bound; the borderline band (is_borderline) against
literal margins at |thr| <= 1, 10 and 100 and NaN margins.  No function here is
"parity unpinned".
"""

from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

QMAX = 7  # symmetric signed 4-bit codes in [-7, 7]; -8 is never produced


# --------------------------------------------------------------------------
# Sec. 3.2 "4-bit attention weight approximation": quantization of Q and K
# --------------------------------------------------------------------------
def quantize_blocks(x: np.ndarray, block: int, qmax: int = QMAX):
    """Per-block symmetric quantization; 4 bit by default (Sec. 3.2; Alg. 1 inputs Q~, K~),
    8 bit with qmax = 127 (the quantized Computation-Pass of Sec. 3.4; then read 127 for 7 below).

    x      : float32 [H, N, d], values exactly representable in bf16.
    block  : rows per block (b_q for Q, b_k for K); one fp32 scale per
             (head, block) shared by all block*d elements.
    returns: codes int8 [H, N, d] in [-7, 7], scales float32 [H, N/block].

    All arithmetic is IEEE fp32, one operation at a time:
      amax = max|x|;  scale = amax / 7;  inv = 7 / amax;
      code = clamp(round_half_even(x * inv), -7, 7).
    A block of zeros gets scale 1 and codes 0.
    """
    x = np.asarray(x, dtype=np.float32)
    H, N, d = x.shape
    assert N % block == 0
    nb = N // block
    xb = x.reshape(H, nb, block * d)
    amax = np.max(np.abs(xb), axis=2).astype(np.float32)            # [H, nb]
    zero = amax == np.float32(0.0)
    safe = np.where(zero, np.float32(1.0), amax).astype(np.float32)
    seven = np.float32(qmax)
    scale = np.where(zero, np.float32(1.0), safe / seven).astype(np.float32)
    inv = np.where(zero, np.float32(0.0), seven / safe).astype(np.float32)
    y = (xb * inv[:, :, None]).astype(np.float32)                    # one fp32 multiply
    code = np.rint(y)                                                # ties to even
    code = np.clip(code, -qmax, qmax).astype(np.int8)
    return code.reshape(H, N, d), scale


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """Nibble packing of the boundary format: byte c of a row holds channel 2c
    in bits 0..3 and channel 2c+1 in bits 4..7, each 4-bit two's complement."""
    c = np.asarray(codes).astype(np.int16)
    lo = c[..., 0::2] & 0xF
    hi = c[..., 1::2] & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_int4(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8).astype(np.int16)
    lo = p & 0xF
    hi = (p >> 4) & 0xF
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def int_products(q_codes: np.ndarray, k_codes: np.ndarray) -> np.ndarray:
    """A[r, c] = sum_k Q~[r, k] * K~[c, k]  (Alg. 1, the product inside
    Dequantize).  Exact: every partial sum is an integer below 2^53, so the
    fp64 library matmul used as the step is exact; returned as int32."""
    a = np.asarray(q_codes, dtype=np.float64) @ np.asarray(k_codes, dtype=np.float64).T
    return a.astype(np.int32)


def dequantize(a_int: np.ndarray, s_q: float, s_k, d: int) -> np.ndarray:
    """S~ = A * s_q * s_k / sqrt(d)  (Alg. 1, approximate attention weight)."""
    return np.asarray(a_int, dtype=np.float64) * float(s_q) * np.asarray(s_k, dtype=np.float64) / math.sqrt(d)


# --------------------------------------------------------------------------
# Sec. 3.2 "Relative importance estimation" and Alg. 1
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Geometry:
    """Block geometry (Sec. 3.1; Alg. 1 inputs)."""
    seq_len: int
    head_dim: int
    block_q: int = 64
    block_k: int = 64
    sink_blocks: int = 1
    local_blocks: int = 4
    stats_causal: bool = False   # False: the statistics ignore the causal mask (Alg. 1 comment)
    segment: int = 0             # > 0: segment rule of Appendix C with that many key blocks per segment

    @property
    def n_q(self) -> int:
        return self.seq_len // self.block_q

    @property
    def n_k(self) -> int:
        return self.seq_len // self.block_k

    def j_last(self, i: int) -> int:
        """Last key block any row of query block i may attend causally."""
        return ((i + 1) * self.block_q - 1) // self.block_k

    def local_count(self, i: int) -> int:
        """Key blocks in the local area of query block i.  Without segments: local_blocks.
        With segments (Appendix C) the middle blocks, i.e. those between the sink blocks and
        the local_blocks blocks at the diagonal, are taken `segment` at a time from the left
        and the ones left over at the end of the row count as local too."""
        if self.segment <= 0:
            return self.local_blocks
        middle = self.j_last(i) + 1 - self.sink_blocks - self.local_blocks
        return self.local_blocks + (middle % self.segment if middle > 0 else 0)

    def sink_local(self, i: int) -> list:
        """I_SL of Alg. 1 in key-block units: the sink blocks and the
        local_count(i) blocks ending at (and including) the diagonal one."""
        jl = self.j_last(i)
        s = set(range(min(self.sink_blocks, jl + 1)))
        s |= set(range(max(0, jl - self.local_count(i) + 1), jl + 1))
        return sorted(s)


def sink_local_stats(geo: Geometry, i: int, q_blk: np.ndarray, k: np.ndarray):
    """m~_r = max S[r, c], l~_r = sum exp(S[r, c] - m~_r) over the key tokens c
    of the sink-local blocks of query block i (display equation of Sec. 3.2),
    S from the unquantized inputs, in fp64.  q_blk: [b_q, d], k: [N, d]."""
    q = np.asarray(q_blk, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    cols = np.concatenate([np.arange(j * geo.block_k, (j + 1) * geo.block_k) for j in geo.sink_local(i)])
    s = (q @ kk[cols].T) / math.sqrt(geo.head_dim)                   # [b_q, |I_SL| * b_k]
    if geo.stats_causal:
        rows = i * geo.block_q + np.arange(geo.block_q)
        s = np.where(cols[None, :] <= rows[:, None], s, -np.inf)
    m = s.max(axis=1)
    l = np.exp(s - m[:, None]).sum(axis=1)
    return m, l


def select_row(geo: Geometry, i: int, q_blk, k, q_codes_blk, k_codes, s_q_i: float, s_k, tau: float,
               estimate: str = "int4"):
    """One query block of Alg. 1: returns (mask_row bool [N_k], margin float64
    [N_k], margin_thr float64 [N_k], thr float64 [b_q], m~, l~).

    estimate = "int4": S~ from the 4-bit codes (the method).  estimate = "16bit": the
    ablation of Appendix E ("w/o QK Quant"): S~ = S from the unquantized Q, K (the codes
    and scales are then unused and may be None).

    mask_row[j] = 1 for j in I_SL; for a middle block j (0 <= j <= j_last, not
    in I_SL) it is 1 iff some row r has max_c S~[r, c] >= ln(tau * l~_r) + m~_r,
    the log form of "max P~ >= tau" (Eq. 3, Eq. 4 with the parenthesis where
    Eq. 3 puts it); blocks past j_last are 0.  margin[j] = max_r (rowmax S~ -
    thr_r) for middle blocks (nan elsewhere) and margin_thr[j] the thr_r of the
    row attaining it: the caller uses them to find decisions that sit on the
    threshold.
    """
    m, l = sink_local_stats(geo, i, q_blk, k)
    thr = np.log(tau * l) + m
    jl = geo.j_last(i)
    isl = set(geo.sink_local(i))
    mask = np.zeros(geo.n_k, dtype=bool)
    margin = np.full(geo.n_k, np.nan)
    margin_thr = np.full(geo.n_k, np.nan)
    for j in isl:
        mask[j] = True
    middle = [j for j in range(jl + 1) if j not in isl]
    if middle:
        bk = geo.block_k
        if estimate == "int4":
            a = int_products(q_codes_blk, k_codes[: (jl + 1) * bk])      # [b_q, (jl+1) b_k]
        else:
            assert estimate == "16bit"
            s_full = (np.asarray(q_blk, dtype=np.float64) @ np.asarray(k[: (jl + 1) * bk], dtype=np.float64).T) \
                / math.sqrt(geo.head_dim)
        for j in middle:
            if estimate == "int4":
                s_tilde = dequantize(a[:, j * bk:(j + 1) * bk], s_q_i, s_k[j], geo.head_dim)
            else:
                s_tilde = s_full[:, j * bk:(j + 1) * bk]
            row_max = s_tilde.max(axis=1)
            r_star = int(np.argmax(row_max - thr))
            margin[j] = row_max[r_star] - thr[r_star]
            margin_thr[j] = thr[r_star]
            mask[j] = bool(np.any(row_max >= thr))
    return mask, margin, margin_thr, thr, m, l


def select_head(geo: Geometry, q, k, q_codes, k_codes, s_q, s_k, tau: float, estimate: str = "int4"):
    """Alg. 1 for one (query head, its KV head): M_bs bool [N_q, N_k] plus the
    margins and statistics of every query block."""
    bq = geo.block_q
    mask = np.zeros((geo.n_q, geo.n_k), dtype=bool)
    margin = np.full((geo.n_q, geo.n_k), np.nan)
    margin_thr = np.full((geo.n_q, geo.n_k), np.nan)
    thr = np.zeros(geo.seq_len)
    m = np.zeros(geo.seq_len)
    l = np.zeros(geo.seq_len)
    for i in range(geo.n_q):
        rs = slice(i * bq, (i + 1) * bq)
        mask[i], margin[i], margin_thr[i], thr[rs], m[rs], l[rs] = select_row(
            geo, i, q[rs], k, None if q_codes is None else q_codes[rs], k_codes,
            0.0 if s_q is None else float(s_q[i]), s_k, tau, estimate)
    return mask, margin, margin_thr, thr, m, l


def relative_attention_score(s_tilde, m, l):
    """Eq. 3: P~[r, c] = exp(S~[r, c] - m~_r) / l~_r."""
    return np.exp(np.asarray(s_tilde, dtype=np.float64) - np.asarray(m)[:, None]) / np.asarray(l)[:, None]


def pack_mask_words(mask_row: np.ndarray) -> np.ndarray:
    """Boundary layout of one mask row: bit (j mod 64) of word j // 64."""
    n_k = mask_row.shape[-1]
    words = np.zeros((n_k + 63) // 64, dtype=np.uint64)
    for j in np.nonzero(mask_row)[0]:
        words[j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return words


# --------------------------------------------------------------------------
# Sec. 3.1: masked attention (Eq. 1 with the block mask of Eq. 2)
# --------------------------------------------------------------------------
def attention_probs_block(geo: Geometry, i: int, q_blk, k, mask_row):
    """P = Softmax(S + M) for the rows of query block i; M = M_c + M_s with
    M_s from the block mask row (Eq. 1, Eq. 2).  Returns [b_q, N] fp64."""
    q = np.asarray(q_blk, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    n = kk.shape[0]
    s = (q @ kk.T) / math.sqrt(geo.head_dim)
    rows = i * geo.block_q + np.arange(geo.block_q)
    cols = np.arange(n)
    allowed = (cols[None, :] <= rows[:, None]) & np.repeat(np.asarray(mask_row, dtype=bool), geo.block_k)[None, :]
    s = np.where(allowed, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    return e / e.sum(axis=1, keepdims=True)


def attention_block(geo: Geometry, i: int, q_blk, k, v, mask_row):
    """O rows of query block i (Eq. 1): returns (O fp64 [b_q, d], lse fp64 [b_q])."""
    q = np.asarray(q_blk, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    n = kk.shape[0]
    s = (q @ kk.T) / math.sqrt(geo.head_dim)
    rows = i * geo.block_q + np.arange(geo.block_q)
    cols = np.arange(n)
    allowed = (cols[None, :] <= rows[:, None]) & np.repeat(np.asarray(mask_row, dtype=bool), geo.block_k)[None, :]
    s = np.where(allowed, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    den = e.sum(axis=1, keepdims=True)
    o = (e / den) @ np.asarray(v, dtype=np.float64)
    return o, (mx + np.log(den))[:, 0]


def attention_head(geo: Geometry, q, k, v, mask):
    """Eq. 1 for one head with block mask M_bs [N_q, N_k]; O fp64 [N, d]."""
    bq = geo.block_q
    o = np.zeros((geo.seq_len, np.asarray(v).shape[1]))
    lse = np.zeros(geo.seq_len)
    for i in range(geo.n_q):
        rs = slice(i * bq, (i + 1) * bq)
        o[rs], lse[rs] = attention_block(geo, i, q[rs], k, v, mask[i])
    return o, lse


def attention_block_from_scores(geo: Geometry, i: int, s: np.ndarray, v, mask_row):
    """Eq. 1 for the rows of query block i given their attention weights s [b_q, N] (already divided by
    sqrt(d)): masks, softmax, product with V.  Returns (O fp64 [b_q, d], lse fp64 [b_q])."""
    n = s.shape[1]
    rows = i * geo.block_q + np.arange(geo.block_q)
    cols = np.arange(n)
    allowed = (cols[None, :] <= rows[:, None]) & np.repeat(np.asarray(mask_row, dtype=bool), geo.block_k)[None, :]
    s = np.where(allowed, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    den = e.sum(axis=1, keepdims=True)
    o = (e / den) @ np.asarray(v, dtype=np.float64)
    return o, (mx + np.log(den))[:, 0]


# --------------------------------------------------------------------------
# Sec. 3.4 "Integration with SageAttention": the quantized Computation-Pass
# --------------------------------------------------------------------------
QMAX8 = 127      # symmetric signed 8-bit codes in [-127, 127]
BLOCK8 = 64      # rows per quantization block of Q and of K in the Computation-Pass


def smooth_k(k: np.ndarray):
    """The cited 8-bit attention's K smoothing: subtract from every key its head's mean key (per
    channel, over all N tokens).  Every attention weight of a query row moves by the same amount
    q . mean, which the softmax of that row cancels, so the result of Eq. 1 is unchanged while the
    values to quantize get smaller.  k: float32 [H, N, d] -> (k - mean float32 [H, N, d], mean float32
    [H, d]).  The mean is the exact sum (fp64) divided by N, rounded once to fp32; the subtraction is
    one fp32 operation."""
    k = np.asarray(k, dtype=np.float32)
    mean = (k.astype(np.float64).sum(axis=1) / k.shape[1]).astype(np.float32)
    return (k - mean[:, None, :]).astype(np.float32), mean


def quantize_qk_int8(q: np.ndarray, k: np.ndarray):
    """Operands of the quantized Computation-Pass: Q per (head, 64-row block) and the smoothed K per
    (head, 64-row block) in symmetric 8-bit codes with one fp32 scale per block (same arithmetic as
    quantize_blocks with 127 in place of 7).  q: float32 [Hq, N, d], k: float32 [Hkv, N, d] ->
    (q_codes int8, q_scale [Hq, N/64], k_codes int8, k_scale [Hkv, N/64], k_mean [Hkv, d])."""
    ks, mean = smooth_k(k)
    qc, qs = quantize_blocks(q, BLOCK8, QMAX8)
    kc, ksc = quantize_blocks(ks, BLOCK8, QMAX8)
    return qc, qs, kc, ksc, mean


def attention_block_int8qk(geo: Geometry, i: int, q_codes_blk, s_q_i: float, k_codes, s_k, v, mask_row,
                           q_blk=None, k_mean=None):
    """Rows of query block i with the attention weights taken from the 8-bit operands,
    S' = (Q~_i K~^T) s_q s_k[j] / sqrt(d) with K~ the codes of the smoothed K (exact integer products), and the
    rest of Eq. 1 unchanged: causal and block mask, softmax, product with the unquantized V.
    q_codes_blk int8 [64, d]; k_codes int8 [N, d]; s_k fp32 [N/64]; mask_row bool [N_k].
    S' estimates the logits of K minus its mean key, i.e. Eq. 1's S minus q_r . k_mean / sqrt(d) per row; O does
    not see that shift.  With q_blk (the unquantized rows, [64, d]) and k_mean ([d]) given, the returned lse has
    the shift added back, so that it is the log-sum-exp of (the estimate of) Eq. 1's S; without them it is that
    of S'."""
    assert geo.block_q == BLOCK8
    a = int_products(q_codes_blk, k_codes).astype(np.float64)                       # [64, N]
    s = a * float(s_q_i) * np.repeat(np.asarray(s_k, dtype=np.float64), BLOCK8)[None, :] / math.sqrt(geo.head_dim)
    o, lse = attention_block_from_scores(geo, i, s, v, mask_row)
    if q_blk is not None:
        shift = np.asarray(q_blk, dtype=np.float64) @ np.asarray(k_mean, dtype=np.float64) / math.sqrt(geo.head_dim)
        lse = lse + shift
    return o, lse


# --------------------------------------------------------------------------
# Sec. 3.4 "Integration with SageAttention": low-precision second product (FP8 P and V)
# --------------------------------------------------------------------------
FP8_MAX = 448.0        # largest finite value of OCP FP8 E4M3 (4 exponent bits, bias 7, 3 mantissa bits, no infinities)


def fp8_e4m3_round(x):
    """Nearest value of the OCP FP8 E4M3 grid, ties to the even mantissa, saturating at +-448.
    Grid: normal numbers 2^e * (1 + m/8), e = -6..8, m = 0..7 (2^8 * 1.875 = 480 is not a number: the top is 448);
    subnormal numbers m * 2^-9, m = 0..7.  Returns float64 (every grid value is exact in it)."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), FP8_MAX)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6, 8)                        # below 2^-6 the spacing stays that of the subnormals
    quantum = np.exp2(e - 3)
    r = np.rint(a / quantum) * quantum           # np.rint rounds half to even; a / quantum is exact (power of two)
    return np.sign(x) * np.minimum(r, FP8_MAX)


def fp8_e4m3_encode(values) -> np.ndarray:
    """Bit patterns (uint8: sign, 4 exponent bits, 3 mantissa bits) of values already on the E4M3 grid."""
    v = np.asarray(values, dtype=np.float64)
    a = np.abs(v)
    sign = (np.signbit(v)).astype(np.uint8) << 7
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0))).astype(np.int64)
    normal = a >= 2.0 ** -6
    e = np.where(normal, e, -6)
    mant = np.where(normal, np.rint((a / np.exp2(e) - 1.0) * 8), np.rint(a / 2.0 ** -9)).astype(np.int64)
    expo = np.where(normal, e + 7, 0).astype(np.int64)
    return (sign | (expo.astype(np.uint8) << 3) | mant.astype(np.uint8)).astype(np.uint8)


def quantize_v_fp8(v: np.ndarray):
    """V of the low-precision second product: per (head, channel) over all N tokens, in IEEE fp32,
      amax = max |v|;  scale = amax / 448;  value = fp8_e4m3(v * (448 / amax))
    (one fp32 multiply, then round to nearest even on the E4M3 grid; an all-zero channel gets scale 1, values 0).
    v: float32 [H, N, d] -> (values float64 [H, N, d] on the E4M3 grid, scale float32 [H, d])."""
    v = np.asarray(v, dtype=np.float32)
    amax = np.max(np.abs(v), axis=1).astype(np.float32)                 # [H, d]
    zero = amax == np.float32(0.0)
    safe = np.where(zero, np.float32(1.0), amax)
    scale = np.where(zero, np.float32(1.0), (safe / np.float32(FP8_MAX)).astype(np.float32)).astype(np.float32)
    inv = np.where(zero, np.float32(0.0), (np.float32(FP8_MAX) / safe).astype(np.float32)).astype(np.float32)
    scaled = (v * inv[:, None, :]).astype(np.float32)
    return fp8_e4m3_round(scaled), scale


def attention_block_fp8pv_from_scores(geo: Geometry, i: int, s: np.ndarray, v8: np.ndarray, v_scale: np.ndarray, mask_row,
                                      arg_tol=None):
    """Eq. 1 for the rows of query block i from their attention weights s [b_q, N] with the second product in
    FP8: the probabilities are taken block by block, online, as the quantized attention the method builds on does.
    The kept 64-key blocks are visited in ascending order; a row's running maximum m is updated with each block,
    the block's probabilities are P8 = fp8_e4m3(448 * exp(s - m)) (448: the top of the grid, so that small
    probabilities stay above the subnormal range), and numerator and denominator are both sums of those P8,
    rescaled by exp(m_old - m_new) whenever m grows:
        O[r, c] = v_scale[c] * (sum_k P8[r, k] V8[k, c]) / (sum_k P8[r, k]),   lse = m + ln(sum_k P8 / 448).
    Needs b_k = 64.  v8: values of quantize_v_fp8 [N, d]; v_scale [d].  Returns (O fp64 [b_q, d], lse fp64 [b_q]).

    arg_tol (None, or one absolute tolerance per key block [n_k]): P8 is a rounding decision, so an implementation
    whose argument s - m is off by up to arg_tol may round a probability near the midpoint of two codes to the
    other one.  With arg_tol the function also returns how far that can move the results: (O, lse, o_slack
    [b_q, d], lse_slack [b_q]), computed by rounding every probability at both ends of its tolerance interval
    and carrying the differences through the same sums (zero for a row none of whose probabilities can flip)."""
    assert geo.block_k == 64
    bq, n = s.shape
    rows = i * geo.block_q + np.arange(bq)
    v8 = np.asarray(v8, dtype=np.float64)
    m = np.full(bq, -np.inf)
    num = np.zeros((bq, v8.shape[1]))
    den = np.zeros(bq)
    num_slack = np.zeros_like(num)
    den_slack = np.zeros_like(den)
    for j in range(geo.j_last(i) + 1):
        if not mask_row[j]:
            continue
        cols = np.arange(j * 64, (j + 1) * 64)
        st = np.where(cols[None, :] <= rows[:, None], s[:, cols], -np.inf)
        m_new = np.maximum(m, st.max(axis=1))                       # (finite: key j * 64 <= every row of block i >= j)
        alpha = np.where(np.isneginf(m), 0.0, np.exp(np.where(np.isneginf(m), 0.0, m) - m_new))
        p8 = fp8_e4m3_round(FP8_MAX * np.exp(st - m_new[:, None]))
        num = num * alpha[:, None] + p8 @ v8[cols]
        den = den * alpha + p8.sum(axis=1)
        if arg_tol is not None:
            t = float(np.asarray(arg_tol, dtype=np.float64).reshape(-1)[j if np.ndim(arg_tol) else 0])
            hi = fp8_e4m3_round(np.minimum(FP8_MAX * np.exp(st - m_new[:, None] + t), FP8_MAX))
            lo = fp8_e4m3_round(FP8_MAX * np.exp(st - m_new[:, None] - t))
            num_slack = num_slack * alpha[:, None] + (hi - lo) @ np.abs(v8[cols])
            den_slack = den_slack * alpha + (hi - lo).sum(axis=1)
        m = m_new
    vs = np.asarray(v_scale, dtype=np.float64)[None, :]
    with np.errstate(divide="ignore", invalid="ignore"):
        o = vs * num / den[:, None]
        lse = m + np.log(den / FP8_MAX)
        if arg_tol is None:
            return o, lse
        rest = np.maximum(den - den_slack, 1e-300)[:, None]         # |d(num/den)| <= (d num + |num/den| d den) / (den - d den)
        o_slack = vs * (num_slack + np.abs(num / den[:, None]) * den_slack[:, None]) / rest
        lse_slack = -np.log1p(-np.minimum(den_slack / den, 0.5))    # |d ln den| <= -ln(1 - d den / den)
    return o, lse, np.nan_to_num(o_slack), np.nan_to_num(lse_slack)


def attention_block_int8qk_fp8pv(geo: Geometry, i: int, q_codes_blk, s_q_i: float, k_codes, s_k, v8, v_scale, mask_row,
                                 q_blk=None, k_mean=None, arg_tol=None):
    """The fully quantized Computation-Pass: attention weights from the 8-bit operands as in
    attention_block_int8qk, second product in FP8 as in attention_block_fp8pv_from_scores (arg_tol as there)."""
    assert geo.block_q == BLOCK8
    a = int_products(q_codes_blk, k_codes).astype(np.float64)
    s = a * float(s_q_i) * np.repeat(np.asarray(s_k, dtype=np.float64), BLOCK8)[None, :] / math.sqrt(geo.head_dim)
    out = list(attention_block_fp8pv_from_scores(geo, i, s, v8, v_scale, mask_row, arg_tol))
    if q_blk is not None:
        out[1] = out[1] + np.asarray(q_blk, dtype=np.float64) @ np.asarray(k_mean, dtype=np.float64) / math.sqrt(geo.head_dim)
    return tuple(out)


def dense_mask(geo: Geometry) -> np.ndarray:
    """Every causally visible block selected."""
    mask = np.zeros((geo.n_q, geo.n_k), dtype=bool)
    for i in range(geo.n_q):
        mask[i, : geo.j_last(i) + 1] = True
    return mask


def is_borderline(margin, thr_scale, rel: float = 1e-5):
    """Decisions whose margin lies within rel * max(1, |thr|) of zero."""
    return np.abs(margin) <= rel * np.maximum(1.0, np.abs(thr_scale))


# --------------------------------------------------------------------------
# Sec. 3.3: per-head threshold calibration
# --------------------------------------------------------------------------
def calibration_error(o_full: np.ndarray, o_sale: np.ndarray) -> float:
    """Err = ||O - O~||_1 / N for one head (O: N x d)."""
    o_full = np.asarray(o_full, dtype=np.float64)
    return float(np.abs(o_full - np.asarray(o_sale, dtype=np.float64)).sum() / o_full.shape[0])


def calibrate_head(geo: Geometry, q, k, v, q_codes, k_codes, s_q, s_k, tau0: float, theta: float, max_halvings: int):
    """Sec. 3.3 for one head: start at tau0 and halve tau until Err(tau) < theta (at most max_halvings
    times).  Returns (tau, halvings, [Err at every tau tried])."""
    o_full, _ = attention_head(geo, q, k, v, dense_mask(geo))
    tau, errs = float(tau0), []
    for n in range(max_halvings + 1):
        mask, *_ = select_head(geo, q, k, q_codes, k_codes, s_q, s_k, tau)
        o_sale, _ = attention_head(geo, q, k, v, mask)
        errs.append(calibration_error(o_full, o_sale))
        if errs[-1] < theta or n == max_halvings:
            return tau, n, errs
        tau = tau / 2.0
    raise AssertionError("unreachable")

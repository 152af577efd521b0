"""Pins for the oracle's Selection-Pass (Alg. 1, Eq. 3, Eq. 4) that do not
call back into the oracle's own formulas: a hand-derived toy, the lossless
special case against library logsumexp, and the invariants of the rule."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import sale_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "toy4x4.txt")


def _load_toy():
    rows, mask = {}, []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        if key == "M":
            mask.append([int(v) for v in vals])
        else:
            rows[key] = np.array([float(v) for v in vals])
    t = np.arange(8)
    even = (t % 2 == 0).astype(np.float64)
    q = np.stack([rows["x"], rows["y"], 7 * even, 0 * even], axis=1).astype(np.float32)
    k = np.stack([rows["u"], rows["w"], 0 * even, 7 * even], axis=1).astype(np.float32)
    v = ((4 * t[:, None] + np.arange(4)[None, :]) / 10.0)
    return q, k, v, rows, np.array(mask, dtype=bool)


@pytest.mark.parametrize("stats_causal", [False, True])
def test_toy_4x4_mask_and_statistics(stats_causal):
    q, k, v, rows, expect = _load_toy()
    geo = so.Geometry(8, 4, 2, 2, sink_blocks=1, local_blocks=1, stats_causal=stats_causal)
    qc, sq = so.quantize_blocks(q[None], 2)
    kc, sk = so.quantize_blocks(k[None], 2)
    assert np.all(sq == 1) and np.all(sk == 1)
    np.testing.assert_array_equal(qc[0].astype(np.float32), q)
    a = so.int_products(qc[0], kc[0])
    for r in (4, 5, 6, 7):
        np.testing.assert_array_equal(a[r], rows[f"A{r}"].astype(np.int32))
    mask, margin, mthr, thr, m, l = so.select_head(geo, q, k, qc[0], kc[0], sq[0], sk[0], 0.1)
    np.testing.assert_array_equal(mask, expect)
    e = math.exp
    np.testing.assert_allclose(m[4:8], [4, 4, 2, 2])
    if not stats_causal:
        l_expect = [1 + e(-4) + 2 * e(-6), 1 + e(-4) + e(-6.5) + e(-6), 1 + 3 * e(-2), 1 + 2 * e(-2) + e(-3)]
    else:   # rows see only keys <= their own position inside the diagonal block
        l_expect = [1 + e(-4) + e(-6), 1 + e(-4) + e(-6.5) + e(-6), 1 + 2 * e(-2), 1 + 2 * e(-2) + e(-3)]
    np.testing.assert_allclose(l[4:8], l_expect, rtol=1e-13)
    np.testing.assert_allclose(thr[4], math.log(0.1 * l_expect[0]) + 4, rtol=1e-13)
    # margins: block (2,1) max S~ = 2, block (3,1) max 1, block (3,2) max -1
    np.testing.assert_allclose(margin[2, 1], 2 - (math.log(0.1 * min(l_expect[0], l_expect[1])) + 4), rtol=1e-12)
    assert margin[3, 2] < 0 < margin[3, 1]
    # relative attention scores quoted in the fixture
    if not stats_causal:
        assert abs(e(-2) / l_expect[1] - 0.1324) < 2e-4 or abs(e(-2) / l_expect[0] - 0.1323) < 2e-4
        assert abs(e(-1) / l_expect[3] - 0.2786) < 1e-4
        assert abs(e(-3) / l_expect[3] - 0.0377) < 1e-4


def test_toy_4x4_attention_rows():
    q, k, v, rows, expect = _load_toy()
    geo = so.Geometry(8, 4, 2, 2, sink_blocks=1, local_blocks=1)
    e = math.exp
    o_sparse, _ = so.attention_head(geo, q, k, v, expect)
    o_dense, _ = so.attention_head(geo, q, k, v, so.dense_mask(geo))
    # row 6 sparse: keys 0,1,2,3,6 with weights e^2, 1, 1, e, 1
    w = np.array([e(2), 1, 1, e(1), 1]); keys = [0, 1, 2, 3, 6]
    np.testing.assert_allclose(o_sparse[6], (w[:, None] * v[keys]).sum(0) / w.sum(), rtol=1e-13)
    # row 6 dense: keys 0..6, weights e^2, 1, 1, e, e^-1, e^-1, 1
    w = np.array([e(2), 1, 1, e(1), e(-1), e(-1), 1])
    np.testing.assert_allclose(o_dense[6], (w[:, None] * v[:7]).sum(0) / w.sum(), rtol=1e-13)
    assert abs(o_dense[6, 0] - 0.5914) < 1e-4 and abs(o_sparse[6, 0] - 0.5235) < 1e-4
    # row 7 sparse: keys 0,1,2,3,6,7 with S = 2, 0, -1.5, 1, 0, -1
    w = np.array([e(2), 1, e(-1.5), e(1), 1, e(-1)]); keys = [0, 1, 2, 3, 6, 7]
    np.testing.assert_allclose(o_sparse[7], (w[:, None] * v[keys]).sum(0) / w.sum(), rtol=1e-13)


def _grid_inputs(n, d, b, seed):
    """Inputs on the lossless grid: integers in [-7, 7], every block holds a 7."""
    rng = np.random.default_rng(seed)
    q = rng.integers(-2, 3, size=(n, d)).astype(np.float32)
    k = rng.integers(-1, 2, size=(n, d)).astype(np.float32)
    # a +-7 in a channel whose partner is zero, so logits stay moderate
    q[:, d - 1] = 0; k[:, d - 1] = 0; q[:, d - 2] = 0; k[:, d - 2] = 0
    q[0::b, d - 1] = 7
    k[0::b, d - 2] = 7
    return q, k


@pytest.mark.parametrize("bq,bk,local,tau", [(16, 16, 2, 0.2), (16, 8, 4, 0.2), (8, 8, 1, 0.5)])
def test_lossless_grid_mask_equals_library_logsumexp_rule(bq, bk, local, tau):
    """On the lossless grid S~ = S exactly, so the block rule reduces to
    'some element has S[r,c] - logsumexp_{c' in I_SL} S[r,c'] >= ln(tau)'."""
    n, d = 256, 16
    q, k = _grid_inputs(n, d, min(bq, bk), 11)
    geo = so.Geometry(n, d, bq, bk, sink_blocks=1, local_blocks=local)
    qc, sq = so.quantize_blocks(q[None], bq)
    kc, sk = so.quantize_blocks(k[None], bk)
    assert np.all(sq == 1) and np.all(sk == 1)
    mask, margin, mthr, *_ = so.select_head(geo, q, k, qc[0], kc[0], sq[0], sk[0], tau)

    s = (torch.from_numpy(q).double() @ torch.from_numpy(k).double().T) / math.sqrt(d)
    n_q, n_k = n // bq, n // bk
    expect = np.zeros((n_q, n_k), dtype=bool)
    near = 0
    for i in range(n_q):
        j_last = ((i + 1) * bq - 1) // bk
        isl = sorted(set([0]) | set(range(max(0, j_last - local + 1), j_last + 1)))
        cols = torch.cat([torch.arange(j * bk, (j + 1) * bk) for j in isl])
        rows = slice(i * bq, (i + 1) * bq)
        lse = torch.logsumexp(s[rows][:, cols], dim=1)
        for j in range(j_last + 1):
            if j in isl:
                expect[i, j] = True
                continue
            rel = s[rows, j * bk:(j + 1) * bk] - lse[:, None] - math.log(tau)
            expect[i, j] = bool((rel >= 0).any())
            near += int(rel.abs().min() < 1e-9)
    assert near == 0
    np.testing.assert_array_equal(mask, expect)
    assert 0.1 < mask.sum() / so.dense_mask(geo).sum() < 0.95   # the case is not trivial


def _random_case(n=512, d=128, seed=3):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(n, d, generator=g)
    k = torch.randn(n, d, generator=g)
    q += 0.25 * k + 0.4
    k[0] += 1.5
    return q.bfloat16().float().numpy(), k.bfloat16().float().numpy()


def test_eq3_and_eq4_agree():
    """max P~ >= tau (Eq. 3) and the log-domain compare (Eq. 4) give the same
    decision for every middle block."""
    q, k = _random_case()
    geo = so.Geometry(512, 128, 64, 64, 1, 2)
    qc, sq = so.quantize_blocks(q[None], 64)
    kc, sk = so.quantize_blocks(k[None], 64)
    tau = 0.06
    mask, margin, mthr, thr, m, l = so.select_head(geo, q, k, qc[0], kc[0], sq[0], sk[0], tau)
    checked = 0
    for i in range(geo.n_q):
        rs = slice(i * 64, (i + 1) * 64)
        for j in range(geo.j_last(i) + 1):
            if j in geo.sink_local(i):
                continue
            a = so.int_products(qc[0][rs], kc[0][j * 64:(j + 1) * 64])
            p = so.relative_attention_score(so.dequantize(a, sq[0, i], sk[0, j], 128), m[rs], l[rs])
            if abs(p.max() / tau - 1) < 1e-9:
                continue
            assert bool(p.max() >= tau) == bool(mask[i, j])
            checked += 1
    assert checked > 10


def test_mask_invariants_and_tau_monotonicity():
    q, k = _random_case(seed=4)
    geo = so.Geometry(512, 128, 64, 32, 1, 4)      # b_k != b_q exercises j_last
    qc, sq = so.quantize_blocks(q[None], 64)
    kc, sk = so.quantize_blocks(k[None], 32)
    masks = {}
    for tau in (1e-30, 0.03, 0.07, 0.2):
        masks[tau], *_ = so.select_head(geo, q, k, qc[0], kc[0], sq[0], sk[0], tau)
    dm = so.dense_mask(geo)
    for tau, mk in masks.items():
        assert not np.any(mk & ~dm)                        # never above the causal boundary
        for i in range(geo.n_q):
            jl = ((i + 1) * 64 - 1) // 32
            assert mk[i, 0] and mk[i, max(0, jl - 3):jl + 1].all()   # sink, local, diagonal
    np.testing.assert_array_equal(masks[1e-30], dm)        # tau -> 0+ keeps every causal block
    assert np.all(masks[0.03] >= masks[0.07]) and np.all(masks[0.07] >= masks[0.2])
    assert masks[0.03].sum() > masks[0.07].sum() > masks[0.2].sum()


def test_sink_local_set_and_word_packing():
    geo = so.Geometry(64 * 10, 128, 64, 64, 1, 4)
    assert geo.sink_local(0) == [0]
    assert geo.sink_local(2) == [0, 1, 2]
    assert geo.sink_local(9) == [0, 6, 7, 8, 9]
    geo2 = so.Geometry(64 * 10, 128, 64, 32, 1, 8)
    assert geo2.j_last(0) == 1 and geo2.j_last(9) == 19
    assert geo2.sink_local(9) == [0] + list(range(12, 20))
    row = np.zeros(130, dtype=bool); row[[0, 63, 64, 129]] = True
    w = so.pack_mask_words(row)
    assert w.dtype == np.uint64 and list(w) == [(1 << 63) | 1, 1, 2]


@pytest.mark.parametrize("bq,bk,local,tau", [(64, 64, 2, 0.12), (64, 32, 4, 0.15)])
def test_16bit_estimate_equals_library_logsumexp_rule_on_any_input(bq, bk, local, tau):
    """Appendix E variant ("w/o QK Quant"): with S~ = S the rule is 'some element of the block has
    S[r,c] - logsumexp_{c' in I_SL} S[r,c'] >= ln(tau)' for arbitrary inputs."""
    q, k = _random_case(n=512, seed=8)
    n, d = q.shape
    geo = so.Geometry(n, d, bq, bk, sink_blocks=1, local_blocks=local)
    mask, *_ = so.select_head(geo, q, k, None, None, None, None, tau, estimate="16bit")
    s = (torch.from_numpy(q).double() @ torch.from_numpy(k).double().T) / math.sqrt(d)
    expect = np.zeros((geo.n_q, geo.n_k), dtype=bool)
    for i in range(geo.n_q):
        j_last = ((i + 1) * bq - 1) // bk
        isl = sorted(set([0]) | set(range(max(0, j_last - local + 1), j_last + 1)))
        cols = torch.cat([torch.arange(j * bk, (j + 1) * bk) for j in isl])
        rows = slice(i * bq, (i + 1) * bq)
        lse = torch.logsumexp(s[rows][:, cols], dim=1)
        for j in range(j_last + 1):
            rel = s[rows, j * bk:(j + 1) * bk] - lse[:, None] - math.log(tau)
            expect[i, j] = j in isl or bool((rel >= 0).any())
            assert j in isl or rel.abs().min() > 1e-9
    np.testing.assert_array_equal(mask, expect)
    dm = so.dense_mask(geo)
    assert 0.2 < mask.sum() / dm.sum() < 0.95


def test_16bit_and_int4_estimates_coincide_on_the_lossless_grid():
    q, k = _grid_inputs(256, 16, 8, 21)
    geo = so.Geometry(256, 16, 16, 8, 1, 4)
    qc, sq = so.quantize_blocks(q[None], 16)
    kc, sk = so.quantize_blocks(k[None], 8)
    m4, *_ = so.select_head(geo, q, k, qc[0], kc[0], sq[0], sk[0], 0.2)
    m16, *_ = so.select_head(geo, q, k, None, None, None, None, 0.2, estimate="16bit")
    np.testing.assert_array_equal(m4, m16)


def _segment_walk(j_last, sink, base_local, seg):
    """Appendix C's local area, by walking the row instead of a formula: after the sink blocks, whole
    segments are peeled off from the left for as long as `seg` middle blocks remain before the
    base_local blocks at the diagonal; whatever is left is the local area."""
    blocks = list(range(j_last + 1))
    pos = min(sink, len(blocks))
    while len(blocks) - pos - base_local >= seg:
        pos += seg
    return sorted(set(blocks[:sink]) | set(blocks[max(pos, 0):] if len(blocks) - sink > base_local else blocks))


def test_segment_rule_local_area_matches_walk_and_paper_bounds():
    """Paper shape (Sec. 4.1, Appendix C): b_q = 64, b_k = 32, sink 1 block, local at least 128 tokens =
    4 blocks, segments of 4 blocks: the local area holds at least 128 and fewer than 256 tokens and
    the middle blocks split into whole segments."""
    geo = so.Geometry(64 * 40, 128, 64, 32, sink_blocks=1, local_blocks=4, segment=4)
    plain = so.Geometry(64 * 40, 128, 64, 32, sink_blocks=1, local_blocks=4)
    seen = set()
    for i in range(geo.n_q):
        jl = geo.j_last(i)
        isl = geo.sink_local(i)
        assert isl == _segment_walk(jl, 1, 4, 4)
        assert set(plain.sink_local(i)) <= set(isl)
        middle = [j for j in range(jl + 1) if j not in isl]
        assert len(middle) % 4 == 0
        if middle:
            assert middle == list(range(1, 1 + len(middle)))            # contiguous, right after the sink
            local_tokens = (jl + 1 - middle[-1] - 1) * 32
            assert 128 <= local_tokens < 256
            assert geo.local_count(i) * 32 == local_tokens
            seen.add(geo.local_count(i))
        else:
            assert isl == list(range(jl + 1))
    assert len(seen) >= 2                                               # the remainder really varies
    # other segment sizes and bases, against the same walk
    for sink, base, seg, bk in [(2, 3, 4, 32), (1, 4, 2, 64), (0, 1, 3, 32)]:
        g2 = so.Geometry(64 * 24, 128, 64, bk, sink_blocks=sink, local_blocks=base, segment=seg)
        for i in range(g2.n_q):
            assert g2.sink_local(i) == _segment_walk(g2.j_last(i), sink, base, seg), (sink, base, seg, i)


def test_segment_rule_mask_is_the_plain_mask_with_the_remainder_kept():
    """On the lossless grid the segment variant equals the library logsumexp rule taken over the
    enlarged sink-local set; and every block it adds to I_SL is kept."""
    n, d, bq, bk = 512, 16, 16, 8
    q, k = _grid_inputs(n, d, bk, 21)
    geo = so.Geometry(n, d, bq, bk, sink_blocks=1, local_blocks=2, segment=4)
    qc, sq = so.quantize_blocks(q[None], bq)
    kc, sk = so.quantize_blocks(k[None], bk)
    tau = 0.2
    mask, *_ = so.select_head(geo, q, k, qc[0], kc[0], sq[0], sk[0], tau)
    s = (torch.from_numpy(q).double() @ torch.from_numpy(k).double().T) / math.sqrt(d)
    expect = np.zeros_like(mask)
    for i in range(geo.n_q):
        jl = ((i + 1) * bq - 1) // bk
        isl = _segment_walk(jl, 1, 2, 4)
        cols = torch.cat([torch.arange(j * bk, (j + 1) * bk) for j in isl])
        rows = slice(i * bq, (i + 1) * bq)
        lse = torch.logsumexp(s[rows][:, cols], dim=1)
        for j in range(jl + 1):
            rel = s[rows, j * bk:(j + 1) * bk] - lse[:, None] - math.log(tau)
            assert j in isl or rel.abs().min() > 1e-9
            expect[i, j] = j in isl or bool((rel >= 0).any())
    np.testing.assert_array_equal(mask, expect)
    assert 0.1 < mask.sum() / so.dense_mask(geo).sum() < 0.95


def test_is_borderline_band_is_1e5_relative_to_max_1_thr():
    """The band that excuses GPU / oracle mask differences (spec: decisions within 1e-5 relative of the
    threshold), fixed by literal cases: |margin| <= 1e-5 * max(1, |thr|), both signs, nothing else."""
    # |thr| <= 1: the band is 1e-5 absolute, whatever thr is
    for thr in (0.0, 0.5, -0.5, 1.0, -1.0):
        for sign in (1.0, -1.0):
            assert bool(so.is_borderline(np.float64(sign * 0.9e-5), np.float64(thr)))
            assert not bool(so.is_borderline(np.float64(sign * 1.1e-5), np.float64(thr)))
    # |thr| > 1: the band scales with |thr| (thr = +-10 -> 1e-4; thr = 100 -> 1e-3), not with thr's sign
    for thr, band in ((10.0, 1e-4), (-10.0, 1e-4), (100.0, 1e-3)):
        for sign in (1.0, -1.0):
            assert bool(so.is_borderline(np.float64(sign * 0.9 * band), np.float64(thr)))
            assert not bool(so.is_borderline(np.float64(sign * 1.1 * band), np.float64(thr)))
    # exactly on the edge counts as borderline; zero margin always does
    assert bool(so.is_borderline(np.float64(1e-5), np.float64(0.0)))
    assert bool(so.is_borderline(np.float64(0.0), np.float64(123.0)))
    # element-wise over arrays, thr broadcast per element
    got = so.is_borderline(np.array([0.9e-5, 0.9e-4, 0.9e-4, -2.0]), np.array([0.0, 0.0, 10.0, 1e6]))
    assert got.tolist() == [True, False, True, True]
    # a NaN margin (no decision was taken for that block: sink / local / beyond the diagonal) is never borderline,
    # neither raw nor after the substitution the parity helper applies (margin -> 1e30, thr -> 0)
    assert not bool(so.is_borderline(np.float64("nan"), np.float64(0.0)))
    assert not bool(so.is_borderline(np.float64("nan"), np.float64("nan")))
    assert not bool(so.is_borderline(np.nan_to_num(np.float64("nan"), nan=1e30), np.nan_to_num(np.float64("nan"), nan=0.0)))
    # the explicit rel argument replaces the 1e-5
    assert bool(so.is_borderline(np.float64(0.9e-3), np.float64(0.0), 1e-3))
    assert not bool(so.is_borderline(np.float64(1.1e-3), np.float64(0.0), 1e-3))


def test_parity_helper_forgives_only_differences_inside_the_band():
    """compare_mask_row (what every GPU mask test and the smoke check use) counts a differing decision as hard
    unless its oracle margin is inside the band; blocks without a decision (NaN margin) are always hard."""
    from parity_utils import compare_mask_row
    ora = np.array([True, False, True, False, True])
    gpu = np.array([False, True, True, True, False])              # differs at 0, 1, 3, 4
    margin = np.array([0.5e-5, -3e-5, 0.0, np.nan, 2e-4])
    thr = np.array([0.3, 0.3, 0.3, np.nan, 50.0])                 # band: 1e-5, 1e-5, -, never, 5e-4
    hard, soft = compare_mask_row(gpu, ora, margin, thr)
    assert (hard, soft) == (2, 2)
    assert compare_mask_row(ora, ora, margin, thr) == (0, 0)

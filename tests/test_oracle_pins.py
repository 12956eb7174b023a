"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests calls the GPU library.  Each checks the oracle against
something other than itself: published known-answer vectors, constants the
paper prints, closed forms, invariants, library routines (numpy) or brute
force written independently in Python.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _constants():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_constants.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, val = line.split()[:2]
        out[name] = float(val)
    return out


# ----------------------------------------------------------------------------
# RNG
# ----------------------------------------------------------------------------

def test_philox_known_answer_vectors():
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        out = oracle.philox4x32_10(w[0:4], w[4:6])
        assert [int(x) for x in out] == w[6:10]
        n += 1
    assert n == 3


def test_uniform24_counter_layout():
    # key = (seed lo, seed hi), counter = (row lo, row hi, iteration, 0); stream picks word 0 / 1
    seed = 0x299F31D0A4093822
    row = 0x85A308D3243F6A88
    it = 0x13198A2E
    out = oracle.philox4x32_10([row & 0xFFFFFFFF, row >> 32, it, 0], [seed & 0xFFFFFFFF, seed >> 32])
    for s in (0, 1):
        assert oracle.uniform24(seed, it, row, s) == (int(out[s]) >> 8) / 2.0 ** 24


def test_uniform24_is_uniform_and_streams_uncorrelated():
    n = 40000
    u0 = np.array([oracle.uniform24(7, 3, i, 0) for i in range(n)])
    u1 = np.array([oracle.uniform24(7, 3, i, 1) for i in range(n)])
    u2 = np.array([oracle.uniform24(7, 4, i, 0) for i in range(n)])
    assert u0.min() >= 0.0 and u0.max() < 1.0
    for u in (u0, u1, u2):
        cnt, _ = np.histogram(u, bins=64, range=(0, 1))
        chi2 = ((cnt - n / 64) ** 2 / (n / 64)).sum()
        assert chi2 < 120.0          # 63 dof: mean 63, P(chi2 > 120) ~ 1e-5
    for a, b in ((u0, u1), (u0, u2), (u0[:-1], u0[1:])):
        assert abs(np.corrcoef(a, b)[0, 1]) < 4.0 / math.sqrt(n)


# ----------------------------------------------------------------------------
# Scales, levels, rounding
# ----------------------------------------------------------------------------

def test_delta_h_worked_example_and_levels():
    c = _constants()
    rng = np.random.default_rng(0)
    p = rng.uniform(0.01, 0.99, 1000).astype(np.float32)
    p[17] = 0.5
    g = (p - (rng.random(1000) < 0.5)).astype(np.float32)
    h = (p * (1 - p)).astype(np.float32)
    d = oracle.scales(g, h, 3, 3)
    assert d[1] == np.float32(c["delta_h_binary_3bit"])          # 0.25 / 6 = 1/24
    for B, name in ((2, "levels_2bit"), (3, "levels_3bit")):
        vals_g, vals_h = set(), set()
        for seed in range(4):
            gq, hq, _ = oracle.quantize_gradients(g, h, B, B, seed, 0)
            vals_g |= set(int(x) for x in gq); vals_h |= set(int(x) for x in hq)
        k = int(c[name])
        assert vals_g == set(range(-(k // 2), k // 2 + 1))          # 2^B-1 values, symmetric
        assert vals_h == set(range(0, k))                           # 0 .. 2^B-2


def test_delta_g_definition():
    g = np.array([0.3, -0.7, 0.1], np.float32)
    h = np.array([0.2, 0.1, 0.05], np.float32)
    for B in (2, 3, 4, 5):
        d = oracle.scales(g, h, B, B)
        assert d[0] == np.float32(0.7) / np.float32(2 ** (B - 1) - 1)
        assert d[1] == np.float32(0.2) / np.float32(2 ** B - 2)


def test_sr_takes_floor_or_ceil_and_error_bounded_by_delta():
    rng = np.random.default_rng(1)
    g = rng.normal(size=20000).astype(np.float32)
    h = rng.uniform(0, 1, size=20000).astype(np.float32)
    for B in (2, 3, 5):
        gq, hq, d = oracle.quantize_gradients(g, h, B, B, 11, 5)
        xg = g.astype(np.float64) / float(d[0]); xh = h.astype(np.float64) / float(d[1])
        kg, kh = 2 ** (B - 1) - 1, 2 ** B - 2
        fl = np.floor(np.float32(g / d[0])); ce = np.ceil(np.float32(g / d[0]))
        assert np.all((gq == np.clip(fl, -kg, kg)) | (gq == np.clip(ce, -kg, kg)))
        assert np.all(np.abs(gq - xg) <= 1.0 + 1e-6)                 # |delta_g g~ - g| <= delta_g
        assert np.all(np.abs(hq.astype(np.float64) - xh) <= 1.0 + 1e-6)
        assert gq.min() >= -kg and gq.max() <= kg and hq.max() <= kh


def test_sr_on_grid_inputs_are_deterministic():
    # g, h exact multiples of delta: SR must return them whatever the random numbers are
    k = np.arange(-7, 8)
    g = (k * 0.125).astype(np.float32)          # max|g| = 7/8, B=4 -> delta_g = 1/8
    h = (np.arange(15) % 15 * 0.0625).astype(np.float32)  # max h = 14/16, B=4 -> delta_h = 1/16
    for seed in range(5):
        gq, hq, d = oracle.quantize_gradients(g, h, 4, 4, seed, seed)
        assert d[0] == 0.125 and d[1] == 0.0625
        assert np.array_equal(gq, k) and np.array_equal(hq, np.arange(15))


def test_sr_unbiased_over_seeds_and_seed_changes_result():
    # E[g~] = g / delta_g per row; different seeds give different roundings
    g = np.array([0.9, -0.9, 0.31, -0.52, 0.07, 0.6], np.float32)
    h = np.array([0.25, 0.21, 0.04, 0.13, 0.19, 0.01], np.float32)
    S = 4000
    B = 3
    accg = np.zeros(g.size); acch = np.zeros(g.size)
    seen = set()
    for seed in range(S):
        gq, hq, d = oracle.quantize_gradients(g, h, B, B, seed, 1)
        accg += gq; acch += hq
        seen.add(tuple(gq))
    xg = g / d[0]; xh = h / d[1]
    rg = xg - np.floor(xg); rh = xh - np.floor(xh)
    assert np.all(np.abs(accg / S - xg) <= 4.5 * np.sqrt(rg * (1 - rg) / S) + 1e-9)
    assert np.all(np.abs(acch / S - xh) <= 4.5 * np.sqrt(rh * (1 - rh) / S) + 1e-9)
    assert len(seen) == 8                # three rows are off-grid: all 2^3 outcomes occur


def test_sr_probability_of_ceil_is_fractional_part():
    # one row replicated: rows are independent draws, fraction rounded up ~ x - floor(x)
    n = 200000
    g = np.full(n, 0.25, np.float32); g[0] = 1.0        # B=3: delta_g = 1/3, x = 0.75
    h = np.full(n, 0.1, np.float32); h[0] = 0.6         # delta_h = 0.1, x = 1.0 -> always 1
    gq, hq, d = oracle.quantize_gradients(g, h, 3, 3, 123, 9)
    x = float(np.float32(0.25) / d[0])
    up = (gq[1:] == 1).mean()
    assert abs(up - x) < 5 * math.sqrt(x * (1 - x) / n)
    assert set(np.unique(gq[1:])) == {0, 1}
    xh = float(np.float32(0.1) / d[1])
    assert abs(hq[1:].mean() - xh) < 5 * math.sqrt(0.25 / n)


def test_hoeffding_bound_on_summed_error():
    # P(|sum eps_i| >= delta_g sqrt(2 n ln(4/delta))) <= delta/2   (proof of Thm 5.3)
    rng = np.random.default_rng(5)
    n = 2000
    g = rng.normal(size=n).astype(np.float32); h = np.full(n, 0.25, np.float32)
    dl = 0.1
    viol = 0
    S = 300
    errs = []
    for seed in range(S):
        gq, _, d = oracle.quantize_gradients(g, h, 3, 3, seed, 0)
        e = float((gq.astype(np.float64) * float(d[0]) - g).sum())
        errs.append(e)
        viol += abs(e) >= float(d[0]) * math.sqrt(2 * n * math.log(4 / dl))
    assert viol / S <= dl / 2
    assert abs(np.mean(errs)) < 5 * np.std(errs) / math.sqrt(S)      # E[G~ delta_g] = G


def test_round_to_nearest_mode():
    g = np.array([1.0, 0.49, 0.5, -0.5, -0.51, 0.26, -1.0], np.float32)   # B=3: delta_g = 1/3
    h = np.array([0.6, 0.04, 0.05, 0.06, 0.3, 0.0, 0.14], np.float32)     # delta_h = 0.1
    gq, hq, d = oracle.quantize_gradients(g, h, 3, 3, 0, 0, rounding=1)
    xg = np.float32(g / d[0]); xh = np.float32(h / d[1])
    assert np.array_equal(gq, np.floor(xg.astype(np.float64) + 0.5))      # half rounds up
    assert np.array_equal(hq, np.floor(xh.astype(np.float64) + 0.5))
    # and it ignores the seed
    gq2, hq2, _ = oracle.quantize_gradients(g, h, 3, 3, 99, 7, rounding=1)
    assert np.array_equal(gq, gq2) and np.array_equal(hq, hq2)


def test_all_zero_gradients_quantize_to_zero():
    g = np.zeros(10, np.float32); h = np.zeros(10, np.float32)
    gq, hq, d = oracle.quantize_gradients(g, h, 3, 3, 0, 0)
    assert d[0] == 0 and d[1] == 0 and not gq.any() and not hq.any()


# ----------------------------------------------------------------------------
# Packing and the width rule
# ----------------------------------------------------------------------------

def test_pack_is_gradient_high_signed_hessian_low():
    for w in (16, 32):
        for G, H in ((0, 0), (5, 3), (-5, 3), (-1, (1 << w) - 1), (-(1 << (w - 1)), 0), ((1 << (w - 1)) - 1, 7)):
            word = oracle.pack(G, H, w)
            assert word == (G << w) + H                              # Sec. 6.2 layout
            raw = word & ((1 << (2 * w)) - 1)                        # two's complement bit pattern
            assert raw & ((1 << w) - 1) == H
            hi = raw >> w
            assert (hi - (1 << w) if hi >> (w - 1) else hi) == G
            assert oracle.unpack(word, w) == (G, H)
    with pytest.raises(OverflowError):
        oracle.pack(1 << 15, 0, 16)
    with pytest.raises(OverflowError):
        oracle.pack(0, 1 << 16, 16)


def test_packed_addition_equals_fieldwise_addition():
    rng = np.random.default_rng(2)
    for w in (16, 32):
        G = 0; H = 0; acc = 0
        for _ in range(500):
            g = int(rng.integers(-15, 16)); h = int(rng.integers(0, 31))
            acc += oracle.pack(g, h, w); G += g; H += h
        assert oracle.unpack(acc, w) == (G, H)


def test_width_rule_thresholds():
    for bg, bh in ((2, 2), (3, 3), (4, 4), (5, 5), (3, 8)):
        kg, kh = 2 ** (bg - 1) - 1, 2 ** bh - 2
        for w in (16, 32):
            n = oracle.max_rows_for_width(bg, bh, w)
            fits = lambda m: m * kg <= 2 ** (w - 1) - 1 and m * kh <= 2 ** w - 1
            assert fits(n) and not fits(n + 1)
            oracle.pack(-n * kg, n * kh, w)                          # worst case still packs
    assert [oracle.max_rows_for_width(b, b, 16) for b in (2, 3, 4, 5)] == [32767, 10922, 4681, 2184]
    assert oracle.max_rows_for_width(3, 8, 16) == 258
    assert oracle.max_rows_for_width(3, 8, 32) < 20_000_000          # why cfg 5's root needs the exact-total bound


# ----------------------------------------------------------------------------
# Histogram, subtraction
# ----------------------------------------------------------------------------

def _rand_problem(rng, N, F, nb, B=3):
    bins = rng.integers(0, nb, size=(N, F)).astype(np.uint8)
    kg, kh = 2 ** (B - 1) - 1, 2 ** B - 2
    gq = rng.integers(-kg, kg + 1, size=N).astype(np.int8)
    hq = rng.integers(0, kh + 1, size=N).astype(np.uint8)
    return bins, gq, hq


def test_histogram_matches_numpy_bincount_and_sums_to_leaf_totals():
    rng = np.random.default_rng(3)
    N, F, nb = 5000, 7, 63
    bins, gq, hq = _rand_problem(rng, N, F, nb)
    idx = np.sort(rng.choice(N, 1777, replace=False)).astype(np.int32)
    for rows, kw in ((np.arange(N), {}), (idx, {"row_idx": idx}), (idx[100:900], {"row_idx": idx, "begin": 100, "count": 800}),
                     (np.arange(40, 1040), {"begin": 40, "count": 1000})):
        hist = oracle.build_histograms(bins, nb, gq, hq, **kw)
        for f in range(F):
            eg = np.bincount(bins[rows, f], weights=gq[rows].astype(np.float64), minlength=nb)
            eh = np.bincount(bins[rows, f], weights=hq[rows].astype(np.float64), minlength=nb)
            assert np.array_equal(hist[f, :, 0], eg.astype(np.int64))
            assert np.array_equal(hist[f, :, 1], eh.astype(np.int64))
            assert hist[f, :, 0].sum() == gq[rows].astype(np.int64).sum()
            assert hist[f, :, 1].sum() == hq[rows].astype(np.int64).sum()
    empty = oracle.build_histograms(bins, nb, gq, hq, begin=10, count=0)
    assert not empty.any()


def test_histogram_uint16_bins():
    rng = np.random.default_rng(4)
    N, F, nb = 3000, 3, 700
    bins = rng.integers(0, nb, size=(N, F)).astype(np.uint16)
    gq = rng.integers(-3, 4, N).astype(np.int8); hq = rng.integers(0, 7, N).astype(np.uint8)
    hist = oracle.build_histograms(bins, nb, gq, hq)
    for f in range(F):
        assert np.array_equal(hist[f, :, 0], np.bincount(bins[:, f], weights=gq, minlength=nb).astype(np.int64))


def test_parent_minus_child_is_sibling():
    rng = np.random.default_rng(6)
    N, F, nb = 4000, 5, 32
    bins, gq, hq = _rand_problem(rng, N, F, nb)
    idx = rng.permutation(N).astype(np.int32)[:3000]
    idx.sort()
    left = idx[bins[idx, 2] <= 11]; right = idx[bins[idx, 2] > 11]
    hp = oracle.build_histograms(bins, nb, gq, hq, row_idx=idx)
    hl = oracle.build_histograms(bins, nb, gq, hq, row_idx=left)
    hr = oracle.build_histograms(bins, nb, gq, hq, row_idx=right)
    assert np.array_equal(oracle.subtract_histograms(hp, hl), hr)
    assert np.array_equal(oracle.subtract_histograms(hp, hr), hl)


# ----------------------------------------------------------------------------
# Split search: brute force on tiny inputs
# ----------------------------------------------------------------------------

def _brute_force_split(bins, gq, hq, rows, nb, dg, dh, min_data, min_sum_hess):
    """Every (feature, threshold): physically partition the rows, sum g~, h~ directly
    (no histogram), evaluate eq. (gain); first strictly-largest gain wins."""
    dg = float(dg); dh = float(dh)
    Gs = int(gq[rows].astype(np.int64).sum()); Hs = int(hq[rows].astype(np.int64).sum())
    n = len(rows)
    best = (0.0, -1, -1, None)
    exact = {}
    if Hs <= 0:
        return best, exact
    parent = (Gs * dg) * (Gs * dg) / (2.0 * (Hs * dh))
    for f in range(bins.shape[1]):
        for t in range(nb - 1):
            L = [i for i in rows if bins[i, f] <= t]
            GL = sum(int(gq[i]) for i in L); HL = sum(int(hq[i]) for i in L)
            GR = Gs - GL; HR = Hs - HL
            if HL <= 0 or HR <= 0:
                continue
            cl = int(Fraction(HL * n, Hs) + Fraction(1, 2))            # round half up
            if cl < min_data or n - cl < min_data:
                continue
            if HL * dh < min_sum_hess or HR * dh < min_sum_hess:
                continue
            gain = (GL * dg) * (GL * dg) / (2.0 * (HL * dh)) + (GR * dg) * (GR * dg) / (2.0 * (HR * dh)) - parent
            exact[(f, t)] = Fraction(GL * GL, HL) + Fraction(GR * GR, HR)
            if gain > best[0]:
                best = (gain, f, t, (GL, HL, GR, HR, cl))
    return best, exact


@pytest.mark.parametrize("seed", range(8))
def test_find_best_split_matches_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    N, F, nb = 60, 4, 6
    bins, gq, hq = _rand_problem(rng, N, F, nb, B=3)
    rows = np.sort(rng.choice(N, 45, replace=False)).astype(np.int32)
    dg, dh = np.float32(0.3), np.float32(0.04)
    min_data = [0, 5, 12][seed % 3]
    msh = [0.0, 0.0, 0.0, 1.5][seed % 4]
    hist = oracle.build_histograms(bins, nb, gq, hq, row_idx=rows)
    Gs = int(gq[rows].astype(np.int64).sum()); Hs = int(hq[rows].astype(np.int64).sum())
    got = oracle.find_best_split(hist, len(rows), Gs, Hs, dg, dh, min_data, msh)
    (gain, f, t, st), exact = _brute_force_split(bins, gq, hq, list(rows), nb, dg, dh, min_data, msh)
    assert (got.feature, got.bin) == (f, t)
    if f >= 0:
        assert got.gain == gain
        assert (got.GL, got.HL, got.GR, got.HR, got.cnt_left) == st
        # the winner maximises the exact rational criterion GL^2/HL + GR^2/HR, and is the
        # first (feature, bin) in scan order among the exact maximisers
        mx = max(exact.values())
        assert exact[(f, t)] == mx
        assert (f, t) == min(k for k, v in exact.items() if v == mx)
    else:
        assert got.gain == 0.0


def test_find_best_split_tie_goes_to_lowest_feature_then_bin():
    # two identical features, and empty bins that repeat the same left sums
    bins = np.array([[0, 0], [0, 0], [3, 3], [3, 3], [5, 5], [5, 5]], np.uint8)
    gq = np.array([-3, -3, 1, 1, 3, 3], np.int8); hq = np.full(6, 2, np.uint8)
    hist = oracle.build_histograms(bins, 6, gq, hq)
    s = oracle.find_best_split(hist, 6, 2, 12, 0.5, 0.125)
    assert (s.feature, s.bin) == (0, 0)          # thresholds 0,1,2 tie on feature 0 and on feature 1
    assert (s.GL, s.HL, s.GR, s.HR, s.cnt_left) == (-6, 4, 8, 8, 2)
    assert s.gain == pytest.approx(((-6 * .5) ** 2 / (2 * 4 * .125) + (8 * .5) ** 2 / (2 * 8 * .125) - (2 * .5) ** 2 / (2 * 12 * .125)))


def test_no_valid_split_cases():
    bins = np.zeros((10, 2), np.uint8)           # every row in one bin: HR = 0 everywhere
    gq = np.ones(10, np.int8); hq = np.ones(10, np.uint8)
    hist = oracle.build_histograms(bins, 4, gq, hq)
    assert oracle.find_best_split(hist, 10, 10, 10, 1.0, 1.0).feature == -1
    bins[5:, 0] = 2
    hist = oracle.build_histograms(bins, 4, gq, hq * 0)     # all hessians zero
    assert oracle.find_best_split(hist, 10, 10, 0, 1.0, 1.0).feature == -1
    gq2 = np.array([1] * 5 + [-1] * 5, np.int8)
    hist = oracle.build_histograms(bins, 4, gq2, hq)
    assert oracle.find_best_split(hist, 10, 0, 10, 1.0, 1.0, min_data=6).feature == -1
    assert oracle.find_best_split(hist, 10, 0, 10, 1.0, 1.0, min_data=5).feature == 0


# ----------------------------------------------------------------------------
# Partition, refit
# ----------------------------------------------------------------------------

def test_partition_is_stable_filter():
    rng = np.random.default_rng(8)
    N, F, nb = 3000, 6, 20
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    idx = np.sort(rng.choice(N, 2000, replace=False)).astype(np.int32)
    out, nl = oracle.partition_rows(bins, idx, 300, 1200, 4, 7)
    seg = idx[300:1500]
    left = seg[bins[seg, 4] <= 7]; right = seg[bins[seg, 4] > 7]
    assert nl == left.size
    assert np.array_equal(out[300:300 + nl], left) and np.array_equal(out[300 + nl:1500], right)
    assert np.array_equal(out[:300], idx[:300]) and np.array_equal(out[1500:], idx[1500:])
    out0, nl0 = oracle.partition_rows(bins, idx, 5, 0, 0, 0)
    assert nl0 == 0 and np.array_equal(out0, idx)


def test_refit_closed_forms():
    rng = np.random.default_rng(9)
    n = 5000
    y = (rng.random(n) < 0.3).astype(np.float32)
    g = (np.float32(0.5) - y).astype(np.float32); h = np.full(n, 0.25, np.float32)    # log-loss at score 0
    idx = np.arange(n, dtype=np.int32)
    w = oracle.refit_leaves(g, h, idx, [0], [n])
    assert w[0] == pytest.approx(4.0 * (y.mean(dtype=np.float64) - 0.5), rel=1e-12)
    # squared loss: h = 1, g = prediction - target  ->  w = mean residual (target - prediction)
    res = rng.normal(size=n).astype(np.float32)
    w = oracle.refit_leaves(-res, np.ones(n, np.float32), idx, [0, 2000], [2000, 3000])
    assert w[0] == pytest.approx(res[:2000].astype(np.float64).mean(), rel=1e-12)
    assert w[1] == pytest.approx(res[2000:].astype(np.float64).mean(), rel=1e-12)
    # zero hessian sum -> 0
    assert oracle.refit_leaves(g, np.zeros(n, np.float32), idx, [0], [n])[0] == 0.0
    # gathers through the index list
    perm = rng.permutation(n).astype(np.int32)
    w = oracle.refit_leaves(-res, np.ones(n, np.float32), perm, [0], [100])
    assert w[0] == pytest.approx(res[perm[:100]].astype(np.float64).mean(), rel=1e-12)


def test_quantized_leaf_value_formula():
    assert oracle.quantized_leaf_value(-6, 4, 0.5, 0.125) == 6 * 0.5 / (4 * 0.125)
    assert oracle.quantized_leaf_value(3, 0, 0.5, 0.125) == 0.0


def test_appendix_d_worked_number():
    c = _constants()
    d_h = float(oracle.scales(np.zeros(2, np.float32), np.array([0.25, 0.1], np.float32), 3, 3)[1])
    val = 8 * d_h ** 2 * math.log(8 / 0.01) / 0.01 ** 2
    assert round(val) == int(c["min_rows_example"])


# ----------------------------------------------------------------------------
# loss derivatives and score update (the steps around the tree)
# ----------------------------------------------------------------------------

def test_logistic_gradients_closed_forms():
    # score 0: p = 1/2, so g = 1/2 - y and h = 1/4 exactly
    y = np.array([0.0, 1.0, 0.0, 1.0], np.float32)
    g, h = oracle.logistic_gradients(np.zeros(4, np.float32), y)
    assert np.array_equal(g, np.array([0.5, -0.5, 0.5, -0.5], np.float32))
    assert np.array_equal(h, np.full(4, 0.25, np.float32))
    # symmetry sigma(-s) = 1 - sigma(s): g(s, 0) + g(-s, 0) = 1, h even in s
    s = np.linspace(-12, 12, 97).astype(np.float32)
    g0, h0 = oracle.logistic_gradients(s, np.zeros_like(s))
    g1, h1 = oracle.logistic_gradients(-s, np.zeros_like(s))
    assert np.allclose(g0 + g1, 1.0, atol=2e-7)
    assert np.allclose(h0, h1, rtol=1e-6, atol=1e-12)
    # g is the derivative of the loss, h the derivative of g (central differences in fp64)
    def loss(sv, yv):
        p = 1.0 / (1.0 + np.exp(-sv)); return -(yv * np.log(p) + (1 - yv) * np.log(1 - p))
    sv = np.linspace(-4, 4, 33); eps = 1e-4
    for yv in (0.0, 1.0):
        gg, hh = oracle.logistic_gradients(sv.astype(np.float32), np.full(sv.size, yv, np.float32))
        sv32 = sv.astype(np.float32).astype(np.float64)
        num_g = (loss(sv32 + eps, yv) - loss(sv32 - eps, yv)) / (2 * eps)
        num_h = (loss(sv32 + eps, yv) - 2 * loss(sv32, yv) + loss(sv32 - eps, yv)) / eps ** 2
        assert np.allclose(gg, num_g, atol=1e-6)
        assert np.allclose(hh, num_h, atol=1e-5)
    # saturation: bounded in [-1, 1] (Sec. 5 remark on cross-entropy), h -> 0
    g, h = oracle.logistic_gradients(np.array([80.0, -80.0], np.float32), np.array([0.0, 1.0], np.float32))
    assert g[0] == 1.0 and g[1] == -1.0 and h[0] >= 0.0 and h[0] < 1e-30 and h[1] < 1e-30


def test_update_scores_adds_each_rows_leaf_value_once():
    rng = np.random.default_rng(2)
    N, L = 1000, 7
    perm = rng.permutation(N).astype(np.int32)
    cuts = np.sort(rng.choice(np.arange(1, N), L - 1, replace=False))
    begin = np.concatenate([[0], cuts]).astype(np.int64); count = np.diff(np.concatenate([begin, [N]])).astype(np.int64)
    value = rng.normal(size=L)
    score = rng.normal(size=N).astype(np.float32)
    out = oracle.update_scores(score, perm, begin, count, value, 0.1)
    leaf_of_row = np.empty(N, np.int64)
    for l in range(L):
        leaf_of_row[perm[begin[l]: begin[l] + count[l]]] = l
    exp = score + (0.1 * value[leaf_of_row]).astype(np.float32)      # one fp32 addition per row
    assert np.array_equal(out, exp)
    assert np.array_equal(oracle.update_scores(score, perm, begin, count, np.zeros(L), 0.1), score)


def test_lambdarank_gradients_pins():
    # two documents, relevance 1 and 0, equal scores: ranks 0 and 1, gains 1 and 0, maxDCG = 1,
    # |disc_0 - disc_1| = 1 - 1/log2(3), rho = 1/2
    d = 1.0 - 1.0 / np.log2(3.0)
    g, h = oracle.lambdarank_gradients(np.zeros(2, np.float32), np.array([1.0, 0.0], np.float32), 2)
    assert np.allclose(g, [-0.5 * d, 0.5 * d], rtol=1e-7) and np.allclose(h, [0.25 * d, 0.25 * d], rtol=1e-7)
    # ... and with the relevant document scored s higher: rho = 1 / (1 + e^s)
    s = 1.5
    g, h = oracle.lambdarank_gradients(np.array([s, 0.0], np.float32), np.array([1.0, 0.0], np.float32), 2)
    rho = 1.0 / (1.0 + np.exp(s))
    assert np.allclose(g, [-rho * d, rho * d], rtol=1e-7) and np.allclose(h, [rho * (1 - rho) * d] * 2, rtol=1e-7)
    # brute force in numpy on random queries (independent of the C loops: vectorised over pairs)
    rng = np.random.default_rng(4)
    Q, gs = 7, 13
    sc = rng.normal(size=Q * gs).astype(np.float32); rel = rng.integers(0, 5, Q * gs).astype(np.float32)
    sc[3] = sc[5]                                                  # a tie inside the first query: ranked by position
    g, h = oracle.lambdarank_gradients(sc, rel, gs)
    for q in range(Q):
        s64 = sc[q * gs:(q + 1) * gs].astype(np.float64); r = rel[q * gs:(q + 1) * gs]
        order = np.lexsort((np.arange(gs), -s64)); rank = np.empty(gs, int); rank[order] = np.arange(gs)
        disc = 1.0 / np.log2(rank + 2.0); gain = 2.0 ** r - 1.0
        max_dcg = (np.sort(gain)[::-1] / np.log2(np.arange(gs) + 2.0)).sum()
        better = r[:, None] > r[None, :]
        rho = 1.0 / (1.0 + np.exp(s64[:, None] - s64[None, :]))
        w = np.abs(gain[:, None] - gain[None, :]) * np.abs(disc[:, None] - disc[None, :]) / max_dcg
        lam = np.where(better, rho * w, 0.0); hes = np.where(better, rho * (1 - rho) * w, 0.0)
        assert np.allclose(g[q * gs:(q + 1) * gs], -lam.sum(1) + lam.sum(0), rtol=1e-6, atol=1e-9)
        assert np.allclose(h[q * gs:(q + 1) * gs], hes.sum(1) + hes.sum(0), rtol=1e-6, atol=1e-9)
        assert abs(g[q * gs:(q + 1) * gs].astype(np.float64).sum()) < 1e-6          # every pair adds +x and -x
    assert (h >= 0).all()
    # a common offset of a query's scores changes nothing; a query of equal relevance has no pairs
    g2, h2 = oracle.lambdarank_gradients(sc + np.float32(2.0), rel, gs)
    assert np.allclose(g2, g, rtol=1e-4, atol=1e-7)
    g0, h0 = oracle.lambdarank_gradients(sc[:gs], np.full(gs, 2.0, np.float32), gs)
    assert not g0.any() and not h0.any()
    # a shorter last query
    g3, h3 = oracle.lambdarank_gradients(sc[:gs + 5], rel[:gs + 5], gs)
    assert np.array_equal(g3[:gs], g[:gs]) and abs(g3[gs:].astype(np.float64).sum()) < 1e-6

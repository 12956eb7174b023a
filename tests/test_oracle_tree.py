"""Whole-tree pins of the CPU oracle.

The end-to-end pin is the on-grid special case: when every g_i and h_i is an
exact multiple of the quantization interval, stochastic rounding changes
nothing (g~ delta_g = g), so the quantized tree must equal the textbook
exact-histogram GBDT tree grown from the floating-point g, h with the split
criterion of Sec. 3.  That reference grower is written here, independently, in
numpy / Python.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _exact_gbdt_tree(bins, nb, g, h, num_leaves, min_data):
    """Leaf-wise GBDT from fp64 g, h (Sec. 3, eq. (leaf), eq. (split_criterion)).
    Row counts for min_data are the hessian-share estimate, rounded half up."""
    g = g.astype(np.float64); h = h.astype(np.float64)
    N, F = bins.shape
    leaves = [np.arange(N)]
    best = {}

    def evaluate(rows):
        Gs = g[rows].sum(); Hs = h[rows].sum(); n = len(rows)
        res = (0.0, -1, -1)
        if Hs <= 0:
            return res
        parent = Gs * Gs / (2.0 * Hs)
        for f in range(F):
            cg = np.cumsum(np.bincount(bins[rows, f], weights=g[rows], minlength=nb))
            ch = np.cumsum(np.bincount(bins[rows, f], weights=h[rows], minlength=nb))
            for t in range(nb - 1):
                GL, HL = cg[t], ch[t]; GR, HR = Gs - GL, Hs - HL
                if HL <= 0 or HR <= 0:
                    continue
                cl = int(Fraction(HL) * n / Fraction(Hs) + Fraction(1, 2))
                if cl < min_data or n - cl < min_data:
                    continue
                gain = GL * GL / (2.0 * HL) + GR * GR / (2.0 * HR) - parent
                if gain > res[0]:
                    res = (gain, f, t)
        return res

    best[0] = evaluate(leaves[0])
    splits = []
    while len(leaves) < num_leaves:
        s = -1; bg = 0.0
        for l in range(len(leaves)):
            if best[l][1] >= 0 and best[l][0] > bg:
                bg = best[l][0]; s = l
        if s < 0:
            break
        gain, f, t = best[s]
        rows = leaves[s]
        left = rows[bins[rows, f] <= t]; right = rows[bins[rows, f] > t]
        splits.append((s, f, t, gain, len(left)))
        leaves[s] = left; leaves.append(right)
        best[s] = evaluate(left); best[len(leaves) - 1] = evaluate(right)
    values = [(-g[r].sum() / h[r].sum()) if h[r].sum() > 0 else 0.0 for r in leaves]
    return splits, leaves, values


def _on_grid_problem(seed, N, F, nb, const_h):
    rng = np.random.default_rng(seed)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    signal = (bins[:, 0].astype(np.float64) / nb - 0.5) + 0.5 * (bins[:, 1] > nb // 3) - 0.25
    kq = np.clip(np.round(4 * signal + rng.normal(scale=2.0, size=N)), -7, 7)
    kq[0] = 7
    g = (kq * 0.125).astype(np.float32)                       # B=4: delta_g = (7/8)/7 = 1/8
    if const_h:
        h = np.full(N, 0.875, np.float32)                     # h~ = 14 everywhere, delta_h = 1/16
    else:
        m = rng.integers(1, 15, N); m[1] = 14
        h = (m * 0.0625).astype(np.float32)
    return bins, g, h


@pytest.mark.parametrize("seed,const_h,min_data", [(0, True, 20), (1, True, 1), (2, False, 0), (3, False, 25)])
def test_on_grid_quantized_tree_equals_exact_gbdt_tree(seed, const_h, min_data):
    N, F, nb, L = 2500, 5, 12, 12
    bins, g, h = _on_grid_problem(seed, N, F, nb, const_h)
    for sr_seed in (0, 12345):                                # the result must not depend on the RNG
        t = oracle.grow_tree(bins, nb, g, h, 4, 4, sr_seed, 3, L, min_data=min_data, verify_sibling=True)
        assert t.delta[0] == 0.125 and t.delta[1] == 0.0625
        splits, leaves, values = _exact_gbdt_tree(bins, nb, g, h, L, min_data)
        assert t.n_leaves == len(leaves) and t.n_leaves > 4
        for k, (s, f, b, gain, nl) in enumerate(splits):
            assert (t.split_leaf[k], t.split_feature[k], t.split_bin[k]) == (s, f, b)
            assert t.split_gain[k] == gain                   # same operations on the same exact values
            assert t.split_n_left[k] == nl
        for l, rows in enumerate(leaves):
            mine = t.row_idx[t.leaf_begin[l]: t.leaf_begin[l] + t.leaf_count[l]]
            assert np.array_equal(mine, rows)                # ascending = stable partition
            assert t.leaf_value[l] == pytest.approx(values[l], rel=1e-12)
            assert t.leaf_value_quant[l] == pytest.approx(values[l], rel=1e-12)   # on grid: no refit error


def test_tree_invariants_off_grid():
    rng = np.random.default_rng(7)
    N, F, nb, L = 20000, 8, 63, 31
    X = rng.normal(size=(N, F))
    bins = np.clip(((X + 3) / 6 * nb).astype(int), 0, nb - 1).astype(np.uint8)
    y = (rng.random(N) < 1 / (1 + np.exp(-(X[:, 0] - X[:, 1] * X[:, 2])))).astype(np.float32)
    score = rng.normal(scale=0.3, size=N)
    p = 1 / (1 + np.exp(-score))
    g = (p - y).astype(np.float32); h = (p * (1 - p)).astype(np.float32)
    t = oracle.grow_tree(bins, nb, g, h, 3, 3, 42, 0, L, min_data=20, verify_sibling=True)
    assert t.n_leaves == L
    # leaves tile the index array, each ascending, together all rows once
    order = np.argsort(t.leaf_begin)
    pos = 0
    for l in order:
        assert t.leaf_begin[l] == pos
        rows = t.row_idx[pos: pos + t.leaf_count[l]]
        assert np.all(np.diff(rows) > 0)
        assert t.leaf_G[l] == t.gq[rows].astype(np.int64).sum()
        assert t.leaf_H[l] == t.hq[rows].astype(np.int64).sum()
        Gf = g[rows].astype(np.float64).sum(); Hf = h[rows].astype(np.float64).sum()
        assert t.leaf_value[l] == pytest.approx(-Gf / Hf, rel=1e-12)
        pos += t.leaf_count[l]
    assert pos == N and np.array_equal(np.sort(t.row_idx), np.arange(N))
    # sum over leaves of refit numerators = total gradient
    tot = sum(-t.leaf_value[l] * h[t.row_idx[t.leaf_begin[l]: t.leaf_begin[l] + t.leaf_count[l]]].astype(np.float64).sum()
              for l in range(L))
    assert tot == pytest.approx(g.astype(np.float64).sum(), rel=1e-9, abs=1e-9)
    # gains of the chosen splits are positive; children's quantized sums add up to the parent's
    assert np.all(t.split_gain > 0)
    assert t.hist_units >= N * F and t.hist_units <= N * F * (1 + (L - 1) / 2)
    # replay: every split's (GL,HL,GR,HR) equal direct sums over the physically partitioned rows
    members = {0: np.arange(N)}
    for k in range(L - 1):
        s = int(t.split_leaf[k]); rows = members[s]
        left = rows[bins[rows, t.split_feature[k]] <= t.split_bin[k]]
        right = rows[bins[rows, t.split_feature[k]] > t.split_bin[k]]
        assert len(left) == t.split_n_left[k]
        assert tuple(t.split_stats[k]) == (t.gq[left].astype(np.int64).sum(), t.hq[left].astype(np.int64).sum(),
                                           t.gq[right].astype(np.int64).sum(), t.hq[right].astype(np.int64).sum())
        members[s] = left; members[k + 1] = right
    # best-first: at every step the split leaf has the largest best-gain among all open leaves
    # (ties: lowest id), each leaf's best split re-derived from a histogram of its own rows
    members = {0: np.arange(N)}
    for k in range(L - 1):
        cand = {}
        for l, rows in members.items():
            hist = oracle.build_histograms(bins, nb, t.gq, t.hq, row_idx=rows.astype(np.int32))
            sp = oracle.find_best_split(hist, len(rows), int(t.gq[rows].astype(np.int64).sum()),
                                        int(t.hq[rows].astype(np.int64).sum()), t.delta[0], t.delta[1], 20, 0.0)
            if sp.feature >= 0:
                cand[l] = sp
        top = max(v.gain for v in cand.values())
        s = min(l for l, v in cand.items() if v.gain == top)
        assert s == t.split_leaf[k]
        assert (cand[s].feature, cand[s].bin, cand[s].gain) == (t.split_feature[k], t.split_bin[k], t.split_gain[k])
        rows = members[s]
        members[s] = rows[bins[rows, cand[s].feature] <= cand[s].bin]
        members[k + 1] = rows[bins[rows, cand[s].feature] > cand[s].bin]


def test_single_leaf_and_stopping():
    rng = np.random.default_rng(3)
    N = 500
    bins = rng.integers(0, 8, (N, 3)).astype(np.uint8)
    y = (rng.random(N) < 0.3).astype(np.float32)
    g = (0.5 - y).astype(np.float32); h = np.full(N, 0.25, np.float32)
    t = oracle.grow_tree(bins, 8, g, h, 3, 3, 0, 0, 1)
    assert t.n_leaves == 1 and t.leaf_count[0] == N
    assert t.leaf_value[0] == pytest.approx(4 * (y.mean(dtype=np.float64) - 0.5), rel=1e-12)
    # min_data larger than half the rows: the root cannot be split
    t = oracle.grow_tree(bins, 8, g, h, 3, 3, 0, 0, 8, min_data=300)
    assert t.n_leaves == 1
    # all-zero gradients: delta = 0, single leaf, value 0
    t = oracle.grow_tree(bins, 8, np.zeros(N, np.float32), np.zeros(N, np.float32), 3, 3, 0, 0, 8)
    assert t.n_leaves == 1 and t.leaf_value[0] == 0.0


def test_constant_hessians_not_quantized():
    """bits_h = 0 (Sec. 4.1: constant hessians need no quantization): h~ = 1, delta_h = the constant,
    so the integer hessian sums are row counts, the count estimate is the true count, and on on-grid
    gradients the tree is the exact-histogram tree of the constant-hessian loss."""
    N, F, nb, L = 2500, 5, 12, 12
    bins, g, _ = _on_grid_problem(5, N, F, nb, True)
    h = np.full(N, 0.75, np.float32)
    gq, hq, delta = oracle.quantize_gradients(g, h, 4, 0, 9, 1)
    assert np.all(hq == 1) and delta[1] == np.float32(0.75) and delta[0] == 0.125
    t = oracle.grow_tree(bins, nb, g, h, 4, 0, 9, 1, L, min_data=20, verify_sibling=True)
    splits, leaves, values = _exact_gbdt_tree(bins, nb, g, h, L, 20)
    assert t.n_leaves == len(leaves) and t.n_leaves > 4
    for k, (s, f, b, gain, nl) in enumerate(splits):
        assert (t.split_leaf[k], t.split_feature[k], t.split_bin[k]) == (s, f, b)
        assert t.split_gain[k] == pytest.approx(gain, rel=1e-12)
        assert t.split_n_left[k] == nl
        assert t.split_stats[k][1] == nl                      # H~ of the left child is its row count
    assert np.array_equal(t.leaf_H[: t.n_leaves], t.leaf_count[: t.n_leaves])
    for l, rows in enumerate(leaves):
        assert np.array_equal(t.row_idx[t.leaf_begin[l]: t.leaf_begin[l] + t.leaf_count[l]], rows)
        assert t.leaf_value[l] == pytest.approx(values[l], rel=1e-12)
    # the width rule with k_h = 1
    assert oracle.max_rows_for_width(2, 0, 16) == 32767 and oracle.max_rows_for_width(5, 0, 16) == 32767 // 15
    # all-zero hessians: nothing to split on
    t0 = oracle.grow_tree(bins, nb, g, np.zeros(N, np.float32), 4, 0, 9, 1, L)
    assert t0.n_leaves == 1


def test_uint16_bins_on_grid_tree_with_thresholds_beyond_8_bits():
    # 16-bit bins: the on-grid special case again, with 700 bins per feature, so that bin ids and thresholds
    # above 255 are in play (a reader that took one byte per bin would fail), and the partition against its
    # plain definition
    rng = np.random.default_rng(21)
    N, F, nb = 600, 2, 700
    bins = rng.integers(0, nb, (N, F)).astype(np.uint16)
    kq = np.clip(np.round(6.0 * (bins[:, 0].astype(np.float64) / nb - 0.5) + rng.normal(scale=1.5, size=N)), -7, 7)
    kq[0] = 7
    g = (kq * 0.125).astype(np.float32)
    h = np.full(N, 0.875, np.float32)
    t = oracle.grow_tree(bins, nb, g, h, 4, 4, 3, 0, 6, min_data=5)
    splits, leaves, values = _exact_gbdt_tree(bins, nb, g, h, 6, 5)
    assert t.n_leaves == len(leaves)
    assert [(int(a), int(b), int(c)) for a, b, c in zip(t.split_leaf, t.split_feature, t.split_bin)] == \
           [(s, f, th) for s, f, th, _, _ in splits]
    assert max(int(b) for b in t.split_bin) > 255
    for l, rows in enumerate(leaves):
        assert np.array_equal(t.row_idx[t.leaf_begin[l]: t.leaf_begin[l] + t.leaf_count[l]], rows)
    idx = np.sort(rng.choice(N, 400, replace=False)).astype(np.int32)
    out, nl = oracle.partition_rows(bins, idx, 10, 300, 1, 300)
    part = idx[10:310]
    exp = np.concatenate([part[bins[part, 1] <= 300], part[bins[part, 1] > 300]])
    assert nl == int((bins[part, 1] <= 300).sum())
    assert np.array_equal(out[10:310], exp) and np.array_equal(out[:10], idx[:10]) and np.array_equal(out[310:], idx[310:])

"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on the same seeded inputs.  Integers, partitions and chosen splits must be
bit-exact; gains and leaf values within 1e-9 relative (fp64)."""
import numpy as np
import pytest
import torch

import oracle
import workloads

pytestmark = pytest.mark.gpu

RTOL = 1e-9


def _ctx(N, F, nb, L=255):
    from paper_2207_09682_amd import Context
    return Context(N, F, nb, max_leaves=L)


def _pack_gh(gq, hq):
    return ((gq.astype(np.int16) << 8) | hq.astype(np.int16)).astype(np.int16)


def _pack_hist(hist):
    """oracle hist [F, nb, 2] -> packed 32|32 words in the library's [nb, F] layout."""
    return np.ascontiguousarray(((hist[..., 0].astype(np.int64) << 32) + hist[..., 1].astype(np.int64)).T)


def _rand_gh(rng, N, bits_g, bits_h, dev):
    kg, kh = 2 ** (bits_g - 1) - 1, 2 ** bits_h - 2
    gq = rng.integers(-kg, kg + 1, N).astype(np.int8)
    hq = rng.integers(0, kh + 1, N).astype(np.uint8)
    return gq, hq, torch.from_numpy(_pack_gh(gq, hq)).to(dev)


# ----------------------------------------------------------------------------
# quantize
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 1000, 100003])
@pytest.mark.parametrize("bits", [(2, 2), (3, 3), (4, 4), (5, 5), (3, 8)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_quantize_bit_exact(n, bits, rounding):
    rng = np.random.default_rng(n + bits[0] * 7 + rounding)
    p = rng.uniform(0.001, 0.999, n).astype(np.float32)
    y = (rng.random(n) < 0.4).astype(np.float32)
    g = (p - y).astype(np.float32); h = (p * (1 - p)).astype(np.float32)
    if n > 10:
        g[3] = 0.0; h[5] = 0.0; g[7] = np.float32(1e-30); h[8] = np.float32(1e-42)   # tiny and denormal inputs
    ctx = _ctx(n, 4, 16)
    gq, hq, d = oracle.quantize_gradients(g, h, bits[0], bits[1], 1234567890123, 17, rounding)
    gh, delta = ctx.quantize_gradients(torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), bits[0], bits[1],
                                       1234567890123, 17, rounding)
    assert np.array_equal(delta.cpu().numpy(), d)
    assert np.array_equal(gh.cpu().numpy(), _pack_gh(gq, hq))


def test_quantize_first_tree_logistic_and_zero_inputs():
    n = 50000
    rng = np.random.default_rng(0)
    y = (rng.random(n) < 0.5).astype(np.float32)
    g = (0.5 - y).astype(np.float32); h = np.full(n, 0.25, np.float32)     # score 0: g = +-1/2, h = 1/4
    ctx = _ctx(n, 4, 16)
    for g_, h_ in ((g, h), (np.zeros(n, np.float32), np.zeros(n, np.float32)), (g, np.zeros(n, np.float32))):
        gq, hq, d = oracle.quantize_gradients(g_, h_, 3, 3, 5, 0)
        gh, delta = ctx.quantize_gradients(torch.from_numpy(g_).cuda(), torch.from_numpy(h_).cuda(), 3, 3, 5, 0)
        assert np.array_equal(delta.cpu().numpy(), d)
        assert np.array_equal(gh.cpu().numpy(), _pack_gh(gq, hq))


# ----------------------------------------------------------------------------
# histogram
# ----------------------------------------------------------------------------

HIST_SHAPES = [
    # N, F, nb, bits_g, bits_h
    (50000, 28, 255, 3, 3),
    (50000, 28, 255, 5, 5),      # 16|16 chunks of 2184 rows: many merges
    (30011, 28, 63, 2, 2),
    (20000, 200, 255, 3, 8),     # tiled features, 8-bit hessians
    (6000, 2000, 63, 3, 3),      # wide
    (9000, 5, 16, 3, 3),         # feature count not a multiple of 4: unaligned rows, partial last dword
    (4000, 3, 256, 3, 3),        # rows narrower than a dword: one byte load per bin
    (8000, 90, 255, 3, 3),       # two ragged tiles
    (6000, 30, 63, 4, 4),
    (5000, 65, 255, 3, 3),       # 64 + 1 features: the tiles are cut so that none is narrower than a dword
    (5000, 7, 255, 2, 2),
    (7000, 64, 256, 4, 4),
    (5000, 36, 100, 3, 3),
]


@pytest.mark.parametrize("N,F,nb,bg,bh", HIST_SHAPES)
@pytest.mark.parametrize("acc", [0, 16, 32])
def test_histogram_bit_exact(N, F, nb, bg, bh, acc):
    rng = np.random.default_rng(N + F)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    bins[:, 0] = np.where(rng.random(N) < 0.7, 0, bins[:, 0])          # one heavily skewed feature
    gq, hq, gh = _rand_gh(rng, N, bg, bh, "cuda")
    ctx = _ctx(N, F, nb)
    dbins = torch.from_numpy(bins).cuda()
    idx = np.sort(rng.choice(N, N // 3, replace=False)).astype(np.int32)
    didx = torch.from_numpy(idx).cuda()
    cases = [
        dict(),                                                          # root: all rows, contiguous
        dict(begin=17, count=N - 40),                                    # contiguous slice, ragged
        dict(row_idx=idx),                                               # gathered leaf
        dict(row_idx=idx, begin=5, count=idx.size // 2),
        dict(row_idx=idx, begin=3, count=1),
        dict(begin=9, count=0),                                          # empty
    ]
    for kw in cases:
        exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, **kw))
        gkw = dict(kw)
        if "row_idx" in gkw:
            gkw["row_idx"] = didx
        got = ctx.build_histograms(dbins, gh, bits_g=bg, bits_h=bh, acc_width=acc, **gkw).cpu().numpy().reshape(nb, F)
        assert np.array_equal(got, exp), (kw.keys(), acc)


def test_histogram_worst_case_first_tree_values():
    # every row carries the extreme values (g~ = +-k_g, h~ = k_h): the overflow bound is tight
    N, F, nb = 200000, 28, 255
    rng = np.random.default_rng(1)
    bins = rng.integers(0, 4, (N, F)).astype(np.uint8)                    # few bins: large sums per bin
    # equal bit widths (16|16 fields) and unequal ones, where a 32-bit word is split unevenly (13|19 for (3, 8),
    # 17|15 for un-quantized constant hessians, 19|13 for (8, 2)): the chunk length is exactly what the fields hold
    for bg, bh in ((3, 3), (5, 5), (3, 8), (3, 0), (4, 0), (2, 5), (8, 2), (6, 3)):
        kg, kh = 2 ** (bg - 1) - 1, (2 ** bh - 2 if bh else 1)
        hq = np.full(N, kh, np.uint8)
        ctx = _ctx(N, F, nb)
        bins[:, 0] = 0                                                    # one feature: every row in one bin
        for gq in (np.where(rng.random(N) < 0.9, kg, -kg).astype(np.int8), np.full(N, kg, np.int8),
                   np.full(N, -kg, np.int8)):                             # the last two fill a field to its last row
            gh = torch.from_numpy(_pack_gh(gq, hq)).cuda()
            exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq))
            for acc in (16, 32):
                got = ctx.build_histograms(torch.from_numpy(bins).cuda(), gh, bits_g=bg, bits_h=bh, acc_width=acc)
                assert np.array_equal(got.cpu().numpy().reshape(nb, F), exp), (bg, bh, acc)


def test_histogram_worst_case_multi_chunk_groups_with_unaligned_head():
    # A contiguous slice that starts at an odd row (its first rows up to a 16-byte aligned row start are taken
    # on top of the first chunk) and is long enough that the row groups of forced 32-bit words span several
    # chunks; every row carries the extreme 4-bit values and feature 0 keeps all rows in one bin: a chunk that
    # took even one row more than the fields hold would overflow.
    N, F, nb = 9_400_003, 28, 255
    gen = torch.Generator(device="cuda").manual_seed(3)
    dbins = torch.randint(0, 4, (N, F), dtype=torch.uint8, device="cuda", generator=gen)
    dbins[:, 0] = 0
    bins = dbins.cpu().numpy()
    ctx = _ctx(N, F, nb, L=15)
    for gval in (7, -7):
        gq = np.full(N, gval, np.int8); hq = np.full(N, 14, np.uint8)
        gh = torch.from_numpy(_pack_gh(gq, hq)).cuda()
        for begin in (1, 2, 3):
            exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, begin=begin, count=N - begin))
            got = ctx.build_histograms(dbins, gh, begin=begin, count=N - begin, bits_g=4, bits_h=4, acc_width=16)
            assert np.array_equal(got.cpu().numpy().reshape(nb, F), exp), (gval, begin)
    del ctx, dbins
    torch.cuda.empty_cache()


@pytest.mark.parametrize("F", [16, 40, 48])
def test_histogram_two_level_byte_stream_other_row_widths(F):
    # long contiguous builds of narrow matrices take the byte-stream kernel's two-level form (32-bit working words
    # folded into 64-bit words in LDS): here for rows of 16, 40 and 48 bytes (64, 60 and 63 lanes per iteration), slices
    # that start on and off a 16-byte boundary, 4- and 5-bit values with every row at the extremes and one feature
    # that keeps all rows in one bin -- a fold that came one row late would overflow a field
    N, nb = 2_600_003, 255
    from paper_2207_09682_amd.binding import describe_hist_plan
    gen = torch.Generator(device="cuda").manual_seed(F)
    dbins = torch.randint(0, 5, (N, F), dtype=torch.uint8, device="cuda", generator=gen)
    dbins[:, 1] = 3
    bins = dbins.cpu().numpy()
    ctx = _ctx(N, F, nb, L=15)
    rng = np.random.default_rng(F)
    for bg, bh in ((5, 5), (4, 4)):
        kg, kh = 2 ** (bg - 1) - 1, 2 ** bh - 2
        assert describe_hist_plan(N, F, nb, 15, 1, bg, bh, 16, False, rows=N - 3)["two_level"] == 1
        gq = np.where(rng.random(N) < 0.97, kg, -kg).astype(np.int8); hq = np.full(N, kh, np.uint8)
        gh = torch.from_numpy(_pack_gh(gq, hq)).cuda()
        for begin in (0, 1, 3):
            exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, begin=begin, count=N - begin))
            got = ctx.build_histograms(dbins, gh, begin=begin, count=N - begin, bits_g=bg, bits_h=bh, acc_width=16)
            assert np.array_equal(got.cpu().numpy().reshape(nb, F), exp), (bg, begin)
    del ctx, dbins
    torch.cuda.empty_cache()


def test_subtract_bit_exact():
    N, F, nb = 40000, 28, 255
    rng = np.random.default_rng(2)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    gq, hq, gh = _rand_gh(rng, N, 4, 4, "cuda")
    idx = np.arange(N, dtype=np.int32)
    left = idx[bins[:, 3] <= 100]
    ctx = _ctx(N, F, nb)
    dbins = torch.from_numpy(bins).cuda()
    hp = ctx.build_histograms(dbins, gh, bits_g=4, bits_h=4)
    hl = ctx.build_histograms(dbins, gh, row_idx=torch.from_numpy(left).cuda(), bits_g=4, bits_h=4)
    hr = ctx.subtract_histograms(hp, hl)
    exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, row_idx=idx[bins[:, 3] > 100]))
    assert np.array_equal(hr.cpu().numpy().reshape(nb, F), exp)
    ctx.subtract_histograms(hp, hl, out=hp)                                # aliasing the parent
    assert np.array_equal(hp.cpu().numpy().reshape(nb, F), exp)


# ----------------------------------------------------------------------------
# split search
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("F,nb", [(28, 255), (28, 63), (200, 255), (2000, 63), (5, 16), (3, 256), (70, 33), (300, 64),
                                  (70, 65), (90, 100), (130, 129), (64, 256)])   # tile search with 2 and 4 bins per lane
def test_find_best_splits_matches_oracle(F, nb):
    from paper_2207_09682_amd import unpack_splits
    rng = np.random.default_rng(F * nb)
    N = 30000
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    bins[:, F // 2] = bins[:, 0]                                          # duplicated feature: ties
    bins[bins == 7] = 8                                                   # an empty bin: repeated prefix sums
    signal = (bins[:, 0] > nb // 2).astype(np.float32) - 0.5
    g = (signal + rng.normal(scale=1.0, size=N)).astype(np.float32); h = rng.uniform(0.01, 0.25, N).astype(np.float32)
    gq, hq, d = oracle.quantize_gradients(g, h, 3, 3, 9, 1)
    leaves = [np.arange(N, dtype=np.int32), np.arange(0, N, 3, dtype=np.int32), np.arange(50, dtype=np.int32),
              np.arange(100, 141, dtype=np.int32), np.arange(5, dtype=np.int32)]
    hists = [oracle.build_histograms(bins, nb, gq, hq, row_idx=r) for r in leaves]
    stats = np.array([[len(r), gq[r].astype(np.int64).sum(), hq[r].astype(np.int64).sum()] for r in leaves], np.int64)
    ctx = _ctx(N, F, nb)
    dh = torch.from_numpy(np.stack([_pack_hist(x).reshape(-1) for x in hists])).cuda()
    for min_data, msh in ((20, 0.0), (0, 0.0), (1, 1.5)):
        raw = ctx.find_best_splits(dh, torch.from_numpy(stats).cuda(), torch.from_numpy(d).cuda(), min_data, msh)
        got = unpack_splits(raw)
        for k, r in enumerate(leaves):
            e = oracle.find_best_split(hists[k], len(r), int(stats[k, 1]), int(stats[k, 2]), d[0], d[1], min_data, msh)
            assert (got[k]["feature"], got[k]["bin"]) == (e.feature, e.bin), (k, min_data)
            assert got[k]["gain"] == pytest.approx(e.gain, rel=RTOL, abs=0.0)
            if e.feature >= 0:
                assert (got[k]["GL"], got[k]["HL"], got[k]["GR"], got[k]["HR"], got[k]["cnt_left"]) == \
                       (e.GL, e.HL, e.GR, e.HR, e.cnt_left)


# ----------------------------------------------------------------------------
# partition, refit
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("N,F", [(100000, 28), (5000, 2000), (300, 5)])
def test_partition_bit_exact(N, F):
    rng = np.random.default_rng(N)
    nb = 64
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    idx = np.sort(rng.choice(N, N // 2, replace=False)).astype(np.int32)
    ctx = _ctx(N, F, nb)
    dbins = torch.from_numpy(bins).cuda()
    for begin, count, f, b in ((0, idx.size, F - 1, 20), (37, idx.size - 100, 0, 0), (5, 1, 1, 63), (10, 0, 0, 5),
                               (0, idx.size, 2, 63), (0, min(777, idx.size), 1, 31)):
        exp, nl = oracle.partition_rows(bins, idx, begin, count, f, b)
        didx = torch.from_numpy(idx.copy()).cuda()
        got_nl = ctx.partition_rows(dbins, didx, begin, count, f, b)
        assert int(got_nl.item()) == nl
        assert np.array_equal(didx.cpu().numpy(), exp)


def test_refit_matches_oracle():
    rng = np.random.default_rng(3)
    N, L = 200000, 37
    g = rng.normal(size=N).astype(np.float32); h = rng.uniform(0, 0.25, N).astype(np.float32)
    perm = rng.permutation(N).astype(np.int32)
    cuts = np.sort(rng.choice(np.arange(1, N), L - 1, replace=False))
    begin = np.concatenate([[0], cuts]).astype(np.int64); count = np.diff(np.concatenate([begin, [N]])).astype(np.int64)
    count[5] = 0                                                           # an empty leaf
    h2 = h.copy(); h2[perm[begin[7]: begin[7] + count[7]]] = 0.0           # a leaf with zero hessian sum
    ctx = _ctx(N, 4, 16, L=64)
    for hh in (h, h2):
        exp = oracle.refit_leaves(g, hh, perm, begin, count)
        got = ctx.refit_leaves(torch.from_numpy(g).cuda(), torch.from_numpy(hh).cuda(), torch.from_numpy(perm).cuda(),
                               torch.from_numpy(begin).cuda(), torch.from_numpy(count).cuda()).cpu().numpy()
        assert np.allclose(got, exp, rtol=RTOL, atol=1e-13)
    assert got[5] == 0.0 and got[7] == 0.0


# ----------------------------------------------------------------------------
# whole trees
# ----------------------------------------------------------------------------

def _compare_tree(t, e, N):
    n = int(t.n_leaves.item())
    assert n == e.n_leaves
    ns = n - 1
    assert np.array_equal(t.delta.cpu().numpy(), e.delta)
    assert np.array_equal(t.split_leaf.cpu().numpy()[:ns], e.split_leaf)
    assert np.array_equal(t.split_feature.cpu().numpy()[:ns], e.split_feature)
    assert np.array_equal(t.split_bin.cpu().numpy()[:ns], e.split_bin)
    assert np.array_equal(t.split_stats.cpu().numpy()[:ns * 4].reshape(ns, 4), e.split_stats)
    assert np.array_equal(t.split_n_left.cpu().numpy()[:ns], e.split_n_left)
    assert np.allclose(t.split_gain.cpu().numpy()[:ns], e.split_gain, rtol=RTOL, atol=0.0)
    assert np.array_equal(t.leaf_begin.cpu().numpy()[:n], e.leaf_begin)
    assert np.array_equal(t.leaf_count.cpu().numpy()[:n], e.leaf_count)
    assert np.array_equal(t.leaf_sum_g.cpu().numpy()[:n], e.leaf_G)
    assert np.array_equal(t.leaf_sum_h.cpu().numpy()[:n], e.leaf_H)
    assert np.array_equal(t.row_idx.cpu().numpy(), e.row_idx)
    assert np.allclose(t.leaf_value.cpu().numpy()[:n], e.leaf_value, rtol=RTOL, atol=1e-13)
    assert np.allclose(t.leaf_value_quant.cpu().numpy()[:n], e.leaf_value_quant, rtol=RTOL, atol=0.0)
    assert int(t.hist_units.item()) == e.hist_units


def _lockstep(cfg, N, F, n_trees, num_leaves, acc=0, bits=None, device="cpu"):
    """Boosting in lock step: every tree of both sides is grown from the same fp32 g, h
    (computed from the GPU side's scores), then compared.  `device` is where the inputs are
    generated (the full-size cases generate on the GPU and copy to the host for the oracle)."""
    wl = workloads.make_workload(cfg, n_rows=N, n_features=F, device=device)
    N = wl.n_rows
    bins_np = workloads.to_numpy(wl.bins)
    dbins = wl.bins.cuda()
    score = torch.zeros(N, device=device)
    ctx = _ctx(N, F, cfg.n_bins, L=num_leaves)
    if device == "cuda":
        ctx.bind_bins(dbins)                               # the full-size cases run as bench.py does: matrix bound
    bg, bh = bits or (cfg.bits_g, cfg.bits_h)
    for it in range(n_trees):
        g, h = workloads.gradients(wl, score)
        t = ctx.grow_tree(dbins, g.cuda(), h.cuda(), bg, bh, cfg.seed, it, num_leaves,
                          min_data_in_leaf=cfg.min_data_in_leaf, acc_width=acc)
        e = oracle.grow_tree(bins_np, cfg.n_bins, workloads.to_numpy(g), workloads.to_numpy(h), bg, bh, cfg.seed, it,
                             num_leaves, min_data=cfg.min_data_in_leaf)
        _compare_tree(t, e, N)
        # score update with the GPU's leaf values (the caller's step, outside the path)
        n = int(t.n_leaves.item())
        leaf_of_row = torch.empty(N, dtype=torch.int64)
        ridx = t.row_idx.cpu().long(); lb = t.leaf_begin.cpu(); lc = t.leaf_count.cpu()
        for l in range(n):
            leaf_of_row[ridx[lb[l]: lb[l] + lc[l]]] = l
        score = score + (cfg.learning_rate * t.leaf_value.cpu()[leaf_of_row].float()).to(score.device)
    return ctx


def test_grow_tree_cfg1_full():
    cfg = workloads.CONFIGS[0]
    _lockstep(cfg, cfg.n_rows, cfg.n_features, 1, cfg.num_leaves)


@pytest.mark.parametrize("acc", [0, 16, 32])
def test_grow_tree_cfg2_reduced_multi_tree(acc):
    cfg = workloads.CONFIGS[1]
    _lockstep(cfg, 150_000, cfg.n_features, 3, 255, acc=acc)


@pytest.mark.parametrize("bits", [(2, 2), (4, 4), (5, 5)])
def test_grow_tree_cfg3_reduced_bit_sweep(bits):
    cfg = workloads.CONFIGS[2]
    _lockstep(cfg, 120_000, cfg.n_features, 2, 255, bits=bits)


def test_grow_tree_cfg4_reduced_wide():
    cfg = workloads.CONFIGS[3]
    _lockstep(cfg, 20_000, cfg.n_features, 2, 63)


def test_grow_tree_cfg5_reduced_ranking():
    cfg = workloads.CONFIGS[4]
    _lockstep(cfg, 60_000, cfg.n_features, 2, 127)


# The five configurations at their full sizes, in the launch configuration bench.py times
# (same context shape, same entry point): whole trees against the oracle, every split, every
# row position and every leaf.

@pytest.mark.parametrize("F,bits,acc", [(16, (4, 4), 0), (40, (5, 5), 16), (48, (4, 4), 0)])
def test_grow_tree_long_narrow_matrices_of_other_widths(F, bits, acc):
    # whole trees whose root build takes the byte-stream kernel's two-level form at row widths other than
    # configuration 3's 28 bytes (2.6 M rows: every CU's share spans several chunks of 4- or 5-bit values)
    cfg = workloads.CONFIGS[2]
    _lockstep(cfg, 2_600_000, F, 2, 31, acc=acc, bits=bits, device="cuda")
    torch.cuda.empty_cache()


def test_full_size_cfg2():
    cfg = workloads.CONFIGS[1]
    _lockstep(cfg, cfg.n_rows, cfg.n_features, 3, cfg.num_leaves, device="cuda")


# Configuration 3 is a grid: 2- to 5-bit gradients x local accumulator words of 32 bits (16|16 fields, handed over
# every n16 rows) or 64 bits (32|32), plus the automatic choice.  Every cell grows the same two trees at full size
# (10.5 M rows, matrix bound, as bench.py times it) and is compared with the oracle's trees for its bit width; the
# oracle's trees and the derivatives they were grown from are shared by the cells of a bit width.
_CFG3_CACHE = {}


def _cfg3_workload():
    if "wl" not in _CFG3_CACHE:
        cfg = workloads.CONFIGS[2]
        wl = workloads.make_workload(cfg, device="cuda")
        ctx = _ctx(wl.n_rows, cfg.n_features, cfg.n_bins, L=cfg.num_leaves)
        dbins = wl.bins.cuda()
        ctx.bind_bins(dbins)
        _CFG3_CACHE.update(wl=wl, ctx=ctx, dbins=dbins, bins_np=workloads.to_numpy(wl.bins))
    return _CFG3_CACHE


def _score_update(t, score, lr):
    """score += lr * leaf value of the row's leaf (the caller's step, outside the path)."""
    n = int(t.n_leaves.item())
    order = torch.argsort(t.leaf_begin[:n], stable=True)      # leaves in the order of their slices
    leaf_at_pos = torch.repeat_interleave(order, t.leaf_count[:n][order])
    upd = (lr * t.leaf_value[leaf_at_pos]).float()
    return score.index_add(0, t.row_idx.long(), upd)


def _cfg3_reference(bits, n_trees):
    """Derivatives of the first n_trees boosting iterations at this bit width and the oracle's trees for them."""
    key = ("ref", bits)
    c = _cfg3_workload()
    have = _CFG3_CACHE.setdefault(key, {"g": [], "h": [], "e": [], "score": None})
    cfg = workloads.CONFIGS[2]
    wl, ctx = c["wl"], c["ctx"]
    if have["score"] is None:
        have["score"] = torch.zeros(wl.n_rows, device="cuda")
    while len(have["e"]) < n_trees:
        it = len(have["e"])
        g, h = workloads.gradients(wl, have["score"])
        e = oracle.grow_tree(c["bins_np"], cfg.n_bins, workloads.to_numpy(g), workloads.to_numpy(h), bits[0], bits[1],
                             cfg.seed, it, cfg.num_leaves, min_data=cfg.min_data_in_leaf)
        t = ctx.grow_tree(c["dbins"], g, h, bits[0], bits[1], cfg.seed, it, cfg.num_leaves,
                          min_data_in_leaf=cfg.min_data_in_leaf)
        _compare_tree(t, e, wl.n_rows)
        have["g"].append(g); have["h"].append(h); have["e"].append(e)
        have["score"] = _score_update(t, have["score"], cfg.learning_rate)
    return have


@pytest.mark.parametrize("acc", [16, 32, 0], ids=["acc16", "acc32", "auto"])
@pytest.mark.parametrize("bits", [(2, 2), (3, 3), (4, 4), (5, 5)], ids=["2bit", "3bit", "4bit", "5bit"])
def test_full_size_cfg3(bits, acc):
    cfg = workloads.CONFIGS[2]
    c = _cfg3_workload()
    ref = _cfg3_reference(bits, 2)
    for it in range(2):
        t = c["ctx"].grow_tree(c["dbins"], ref["g"][it], ref["h"][it], bits[0], bits[1], cfg.seed, it, cfg.num_leaves,
                               min_data_in_leaf=cfg.min_data_in_leaf, acc_width=acc)
        _compare_tree(t, ref["e"][it], c["wl"].n_rows)


def test_full_size_cfg3_ten_trees_lock_step():
    # the headline cell (3-bit, automatic width) over the ten trees the configuration names
    cfg = workloads.CONFIGS[2]
    ref = _cfg3_reference((3, 3), 10)       # every tree is compared with the oracle's as it is grown
    assert len(ref["e"]) == 10
    _CFG3_CACHE.clear()
    torch.cuda.empty_cache()


def test_full_size_cfg4():
    cfg = workloads.CONFIGS[3]
    _lockstep(cfg, cfg.n_rows, cfg.n_features, 2, cfg.num_leaves, device="cuda")


def test_full_size_cfg5():
    cfg = workloads.CONFIGS[4]
    _lockstep(cfg, cfg.n_rows, cfg.n_features, 1, cfg.num_leaves, device="cuda")
    torch.cuda.empty_cache()


@pytest.mark.parametrize("N,F,nb,L", [(160_000_000, 28, 255, 15), (2_400_000, 2000, 63, 7)])
def test_rows_times_features_beyond_2_to_32(N, F, nb, L):
    # Byte offsets into the bin matrix exceed 32 bits.  160 M x 28 (rows kept in leaf order): the partition has
    # 156 K segments, and with forced 32-bit local words every row group spans several chunks (merged through
    # atomics).  2.4 M x 2000 (rows gathered through row ids, 16 feature tiles).  One first-iteration tree
    # (g = +-1/2, h = 1/4: the extreme quantized values) per accumulator setting.
    gen = torch.Generator(device="cuda").manual_seed(5)
    bins = torch.randint(0, nb, (N, F), dtype=torch.uint8, device="cuda", generator=gen)
    z = (bins[:, 3].float() - nb / 2) / (nb / 6) + (bins[:, F - 1] > (3 * nb) // 4).float() - (bins[:, 11] < nb // 8).float()
    y = (torch.rand(N, generator=gen, device="cuda") < torch.sigmoid(z)).float()
    del z
    g = 0.5 - y; h = torch.full((N,), 0.25, device="cuda")
    bins_np = bins.cpu().numpy(); g_np = g.cpu().numpy(); h_np = h.cpu().numpy()
    e = oracle.grow_tree(bins_np, nb, g_np, h_np, 3, 3, 11, 0, L, min_data=20)
    del bins_np
    ctx = _ctx(N, F, nb, L=L)
    for acc in (0, 16):
        t = ctx.grow_tree(bins, g, h, 3, 3, 11, 0, L, min_data_in_leaf=20, acc_width=acc)
        _compare_tree(t, e, N)
    del ctx, bins
    torch.cuda.empty_cache()


def test_constant_hessian_regression_full_size():
    # squared error on a 463,715 x 90 matrix: bits_h = 0 (hessians not quantized), F % 4 == 2 takes the
    # byte-wise histogram kernel; three trees in lock step
    cfg = workloads.EXTRA_CONFIGS[0]
    _lockstep(cfg, cfg.n_rows, cfg.n_features, 3, cfg.num_leaves, device="cuda")


def test_grow_tree_cfg5_full_leaf_budget():
    # 511 leaves: the growth bookkeeping needs more than 64 KB of LDS
    cfg = workloads.CONFIGS[4]
    _lockstep(cfg, 150_000, 40, 1, 511)


def test_grow_tree_bushy_tree_near_the_leaf_limit():
    # 658 leaves (the most the LDS of the growth bookkeeping holds) on twelve two-valued features of about equal
    # weight: nodes of one depth have about the same gain, the tree grows level by level, and the late rounds expand
    # a hundred nodes and more at once -- so many scanned histograms that the plan kernel's feature reduce gives each
    # of them one or two lanes only
    N, F, nb, L = 300_000, 12, 2, 658
    rng = np.random.default_rng(77)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    w = 1.0 - 0.03 * np.arange(F)
    logit = ((bins.astype(np.float64) - 0.5) * w).sum(axis=1)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-logit))).astype(np.float32)
    g = (0.5 - y).astype(np.float32); h = np.full(N, 0.25, np.float32)
    ctx = _ctx(N, F, nb, L=L)
    t = ctx.grow_tree(torch.from_numpy(bins).cuda(), torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), 3, 3, 5, 0, L,
                      min_data_in_leaf=1)
    e = oracle.grow_tree(bins, nb, g, h, 3, 3, 5, 0, L, min_data=1)
    _compare_tree(t, e, N)
    rounds, expanded, committed, _ = ctx.tree_stats()
    assert committed == L - 1 and expanded >= committed
    # the first eight rounds can expand 255 nodes at most (a node's parent is expanded in an earlier round)
    assert rounds <= 16 and (expanded - 255) / (rounds - 8) >= 64, (rounds, expanded)


def test_quantize_unaligned_pointers():
    # g, h that do not start on a 16-byte boundary take the scalar kernels
    N = 70_001
    rng = np.random.default_rng(11)
    g = rng.normal(size=N + 1).astype(np.float32); h = rng.random(N + 1).astype(np.float32)
    ctx = _ctx(N, 8, 32)
    dg = torch.from_numpy(g).cuda(); dh = torch.from_numpy(h).cuda()
    gh, delta = ctx.quantize_gradients(dg[1:], dh[1:], 4, 3, 5, 2)
    gq, hq, d = oracle.quantize_gradients(g[1:], h[1:], 4, 3, 5, 2)
    assert np.array_equal(delta.cpu().numpy(), d)
    assert np.array_equal(gh.cpu().numpy(), _pack_gh(gq, hq))


def test_grow_tree_degenerate_cases():
    N, F, nb = 3000, 8, 32
    rng = np.random.default_rng(4)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    y = (rng.random(N) < 0.3).astype(np.float32)
    g = (0.5 - y).astype(np.float32); h = np.full(N, 0.25, np.float32)
    ctx = _ctx(N, F, nb, L=16)
    dbins = torch.from_numpy(bins).cuda()
    cases = [
        (g, h, 1, 20),                                     # a single leaf
        (g, h, 16, 2000),                                  # min_data forbids every split
        (np.zeros(N, np.float32), np.zeros(N, np.float32), 16, 20),   # all-zero gradients
        (g, h, 16, 20),
    ]
    for g_, h_, L, md in cases:
        t = ctx.grow_tree(dbins, torch.from_numpy(g_).cuda(), torch.from_numpy(h_).cuda(), 3, 3, 1, 0, L, min_data_in_leaf=md)
        e = oracle.grow_tree(bins, nb, g_, h_, 3, 3, 1, 0, L, min_data=md)
        _compare_tree(t, e, N)


@pytest.mark.parametrize("N,F,nb,L", [(1, 1, 2, 4), (2, 1, 2, 4), (64, 3, 4, 8), (1000, 5, 16, 15), (3000, 30, 63, 31),
                                      (5000, 65, 32, 31), (4000, 17, 255, 63), (2500, 130, 8, 15),
                                      (3000, 4096, 16, 7), (2000, 255, 256, 7), (4000, 124, 255, 15), (4000, 132, 200, 15),
                                      (1500, 2, 2, 4), (6000, 16, 256, 31)])
def test_grow_tree_small_and_ragged_shapes(N, F, nb, L):
    # every kernel variant of the tree path at small sizes: rows narrower than a dword, ragged rows,
    # tiles cut so that none is narrower than a dword, a single row, leaves of one row
    rng = np.random.default_rng(N * 131 + F)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-(bins[:, 0].astype(np.float64) - nb / 2) * 4.0 / nb))).astype(np.float32)
    score = np.zeros(N, np.float32)
    ctx = _ctx(N, F, nb, L=L)
    dbins = torch.from_numpy(bins).cuda()
    for it in range(2):
        p = 1.0 / (1.0 + np.exp(-score.astype(np.float64)))
        g = (p - y).astype(np.float32); h = (p * (1 - p)).astype(np.float32)
        t = ctx.grow_tree(dbins, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), 4, 4, 99, it, L, min_data_in_leaf=1)
        e = oracle.grow_tree(bins, nb, g, h, 4, 4, 99, it, L, min_data=1)
        _compare_tree(t, e, N)
        for l in range(e.n_leaves):
            rows = e.row_idx[e.leaf_begin[l]: e.leaf_begin[l] + e.leaf_count[l]]
            score[rows] += np.float32(0.3 * e.leaf_value[l])


def test_errors_are_reported_not_crashes():
    from paper_2207_09682_amd import QgbdtError
    ctx = _ctx(1000, 8, 32, L=8)
    g = torch.zeros(1000, device="cuda"); bins = torch.zeros((1000, 8), dtype=torch.uint8, device="cuda")
    with pytest.raises(QgbdtError):
        ctx.quantize_gradients(g, g, 1, 3, 0, 0)                         # bits out of range
    with pytest.raises(QgbdtError):
        ctx.grow_tree(bins, g, g, 3, 3, 0, 0, 9)                         # more leaves than the context holds
    gh = torch.zeros(1000, dtype=torch.int16, device="cuda")
    with pytest.raises(QgbdtError):
        ctx.build_histograms(bins, gh, begin=10, count=995)              # slice outside the rows
    with pytest.raises(QgbdtError):
        ctx.build_histograms(bins, gh, acc_width=8)
    with pytest.raises(QgbdtError):
        ctx.grow_tree(bins, g, g, 3, 3, 0, 0, 8, row_layout=4)           # no such layout
    with pytest.raises(QgbdtError):
        ctx.grow_tree(bins, g, g, 3, 3, 0, 0, 8, row_layout=3)           # ordered rows need 16..64 features


def test_workspace_is_the_callers():
    # The library allocates no device memory: every buffer is carved from one block the caller hands over.
    from paper_2207_09682_amd import Context, QgbdtError
    from paper_2207_09682_amd import binding as b
    N, F, nb, L = 30000, 28, 63, 15
    rng = np.random.default_rng(9)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-(bins[:, 2].astype(np.float64) - nb / 2) * 6.0 / nb))).astype(np.float32)
    g = (0.5 - y).astype(np.float32); h = np.full(N, 0.25, np.float32)
    e = oracle.grow_tree(bins, nb, g, h, 3, 3, 4, 0, L, min_data=5)
    dbins = torch.from_numpy(bins).cuda(); dg = torch.from_numpy(g).cuda(); dh = torch.from_numpy(h).cuda()
    need0 = Context.workspace_bytes_for(N, F, nb, L, flags=0)
    ctx = Context(N, F, nb, max_leaves=L, workspace_flags=0)
    assert ctx.workspace_bytes == need0
    # a block that is one byte short, or misaligned, is refused, and the context is left without one
    small = torch.empty(need0 - 1, dtype=torch.uint8, device="cuda")
    with pytest.raises(QgbdtError) as ei:
        ctx.set_workspace(small, flags=0)
    assert ei.value.code == b.E_WORKSPACE
    with pytest.raises(QgbdtError) as ei:
        ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5)   # no workspace: refused, nothing launched
    assert ei.value.code == b.E_WORKSPACE
    odd = torch.empty(need0 + 512, dtype=torch.uint8, device="cuda")
    with pytest.raises(QgbdtError):
        ctx.set_workspace(odd[8:], flags=0)
    # a block without optional sections: the steps that need one say so, the others run
    ws = torch.empty(need0 + 4096, dtype=torch.uint8, device="cuda")
    ctx.set_workspace(ws, flags=0)
    for call in (lambda: ctx.bind_bins(dbins),
                 lambda: ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5, row_layout=b.ROWS_ORDERED),
                 lambda: ctx.boost_iteration(dbins, dg, dh.clone(), 3, 3, 4, 0, L, 0.1)):
        with pytest.raises(QgbdtError) as ei:
            call()
        assert ei.value.code == b.E_WORKSPACE
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e, N)   # row ids move
    # the caller may hand over a larger block with more sections later; results do not change
    need_all = Context.workspace_bytes_for(N, F, nb, L)
    ws_all = torch.empty(need_all, dtype=torch.uint8, device="cuda")
    ws_all.fill_(0xA5)                                                     # nothing relies on zeroed memory
    ctx.set_workspace(ws_all)
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e, N)   # leaf-ordered copies
    ctx.bind_bins(dbins)
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e, N)   # bound, row ids move
    # the library wrote nothing outside the block it was given
    guard = torch.empty(need0 + 2 * 4096, dtype=torch.uint8, device="cuda")
    guard.fill_(0x5A)
    ctx.set_workspace(guard[4096:4096 + need0], flags=0)
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e, N)
    torch.cuda.synchronize()
    assert bool((guard[:4096] == 0x5A).all()) and bool((guard[4096 + need0:] == 0x5A).all())


# ----------------------------------------------------------------------------
# around the tree: loss derivatives, score update, one boosting iteration on the device
# ----------------------------------------------------------------------------

def _ulp_diff(a, b):
    ia = a.view(np.int32).astype(np.int64); ib = b.view(np.int32).astype(np.int64)
    ia = np.where(ia < 0, -(ia & 0x7fffffff), ia); ib = np.where(ib < 0, -(ib & 0x7fffffff), ib)
    return np.abs(ia - ib)


@pytest.mark.parametrize("n,offset", [(1, 0), (1003, 0), (262147, 0), (70001, 1)])
def test_logistic_gradients_match_oracle(n, offset):
    # both sides evaluate in fp64 and round once; a last-place difference of the two exp routines can
    # at most move the rounded result by one unit in the last place
    rng = np.random.default_rng(n)
    s = (rng.normal(size=n + offset) * 4).astype(np.float32); y = (rng.random(n + offset) < 0.4).astype(np.float32)
    s[: min(n, 4)] = np.array([0.0, 90.0, -90.0, 1e-20], np.float32)[: min(n, 4)]
    ctx = _ctx(n, 4, 16)
    g, h = ctx.logistic_gradients(torch.from_numpy(s).cuda()[offset:], torch.from_numpy(y).cuda()[offset:])
    eg, eh = oracle.logistic_gradients(s[offset:], y[offset:])
    assert _ulp_diff(g.cpu().numpy(), eg).max() <= 1
    assert _ulp_diff(h.cpu().numpy(), eh).max() <= 1
    assert (g.cpu().numpy() != eg).mean() < 1e-3 and (h.cpu().numpy() != eh).mean() < 1e-3


def test_update_scores_bit_exact():
    rng = np.random.default_rng(8)
    N, L = 300_000, 33
    perm = rng.permutation(N).astype(np.int32)
    cuts = np.sort(rng.choice(np.arange(1, N), L - 1, replace=False))
    begin = np.concatenate([[0], cuts]).astype(np.int64); count = np.diff(np.concatenate([begin, [N]])).astype(np.int64)
    count[3] = 0
    value = rng.normal(size=L)
    score = rng.normal(size=N).astype(np.float32)
    ctx = _ctx(N, 4, 16, L=64)
    d = torch.from_numpy(score.copy()).cuda()
    ctx.update_scores(d, torch.from_numpy(perm).cuda(), torch.from_numpy(begin).cuda(), torch.from_numpy(count).cuda(),
                      torch.from_numpy(value).cuda(), 0.1)
    # rows of the emptied leaf keep their score on both sides
    assert np.array_equal(d.cpu().numpy(), oracle.update_scores(score, perm, begin, count, value, 0.1))


def test_boost_iterations_on_device_lock_step():
    # three iterations run entirely by the library; the oracle follows in lock step from the library's
    # own derivatives of every iteration (the exp routines may differ in the last place)
    cfg = workloads.CONFIGS[1]
    N, F, L, lr = 200_000, cfg.n_features, 63, 0.1
    wl = workloads.make_workload(cfg, n_rows=N, n_features=F)
    bins_np = workloads.to_numpy(wl.bins); dbins = wl.bins.cuda(); label = wl.label.cuda()
    ctx = _ctx(N, F, cfg.n_bins, L=L)
    score = torch.zeros(N, device="cuda")
    for it in range(3):
        before = score.clone()
        g, h = ctx.logistic_gradients(before, label)            # what the iteration will compute internally
        t = ctx.boost_iteration(dbins, label, score, 3, 3, cfg.seed, it, L, lr, min_data_in_leaf=cfg.min_data_in_leaf)
        e = oracle.grow_tree(bins_np, cfg.n_bins, g.cpu().numpy(), h.cpu().numpy(), 3, 3, cfg.seed, it, L,
                             min_data=cfg.min_data_in_leaf)
        _compare_tree(t, e, N)
        n = int(t.n_leaves.item())
        exp = oracle.update_scores(before.cpu().numpy(), e.row_idx, e.leaf_begin, e.leaf_count,
                                   t.leaf_value.cpu().numpy()[:n], lr)
        assert np.array_equal(score.cpu().numpy(), exp)


@pytest.mark.parametrize("n,gs", [(13, 13), (1300, 100), (1037, 100), (4096, 1024), (50, 1)])
def test_lambdarank_gradients_match_oracle(n, gs):
    # both sides sum fp64 terms (in different orders) and round once to fp32
    rng = np.random.default_rng(n + gs)
    s = rng.normal(size=n).astype(np.float32); rel = rng.integers(0, 5, n).astype(np.float32)
    if n > 8:
        s[3] = s[6]                                       # a tie in score: ranked by position on both sides
    ctx = _ctx(n, 4, 16)
    g, h = ctx.lambdarank_gradients(torch.from_numpy(s).cuda(), torch.from_numpy(rel).cuda(), gs)
    eg, eh = oracle.lambdarank_gradients(s, rel, gs)
    scale = max(float(np.abs(eg).max()), 1e-30)
    assert np.allclose(g.cpu().numpy(), eg, rtol=1e-6, atol=1e-7 * scale)
    assert np.allclose(h.cpu().numpy(), eh, rtol=1e-6, atol=1e-7 * scale)


def test_lambdarank_gradients_extreme_score_ranges():
    # a query whose score range is far beyond what exp() of half the range can hold takes the direct form;
    # one near the switch takes the factored form with large factors
    rng = np.random.default_rng(8)
    n, gs = 400, 100
    s = rng.normal(size=n).astype(np.float32); rel = rng.integers(0, 5, n).astype(np.float32)
    s[:100] *= 2000.0                                   # range of several thousand
    s[100:200] *= 100.0                                 # range of ~550: still the factored form, products up to e^550
    s[200:300] = 3.0                                    # all scores equal
    ctx = _ctx(n, 4, 16)
    g, h = ctx.lambdarank_gradients(torch.from_numpy(s).cuda(), torch.from_numpy(rel).cuda(), gs)
    eg, eh = oracle.lambdarank_gradients(s, rel, gs)
    assert np.all(np.isfinite(g.cpu().numpy())) and np.all(np.isfinite(h.cpu().numpy()))
    scale = max(float(np.abs(eg).max()), 1e-30)
    assert np.allclose(g.cpu().numpy(), eg, rtol=1e-6, atol=1e-7 * scale)
    assert np.allclose(h.cpu().numpy(), eh, rtol=1e-6, atol=1e-7 * scale)


def test_boost_iterations_lambdarank_lock_step():
    cfg = workloads.CONFIGS[4]
    N, F, L, lr = 60_000, 40, 63, 0.1
    wl = workloads.make_workload(cfg, n_rows=N, n_features=F)
    N = wl.n_rows
    gs = wl.extra["group_size"]
    bins_np = workloads.to_numpy(wl.bins); dbins = wl.bins.cuda(); rel = wl.label.cuda()
    ctx = _ctx(N, F, cfg.n_bins, L=L)
    score = torch.zeros(N, device="cuda")
    for it in range(2):
        before = score.clone()
        g, h = ctx.lambdarank_gradients(before, rel, gs)
        t = ctx.boost_iteration(dbins, rel, score, cfg.bits_g, cfg.bits_h, cfg.seed, it, L, lr,
                                min_data_in_leaf=cfg.min_data_in_leaf, group_size=gs)
        e = oracle.grow_tree(bins_np, cfg.n_bins, g.cpu().numpy(), h.cpu().numpy(), cfg.bits_g, cfg.bits_h, cfg.seed, it,
                             L, min_data=cfg.min_data_in_leaf)
        _compare_tree(t, e, N)
        n = int(t.n_leaves.item())
        exp = oracle.update_scores(before.cpu().numpy(), e.row_idx, e.leaf_begin, e.leaf_count,
                                   t.leaf_value.cpu().numpy()[:n], lr)
        assert np.array_equal(score.cpu().numpy(), exp)


def test_work_runs_on_torchs_current_stream():
    # the library enqueues on the stream torch considers current: inputs produced by torch kernels on a side
    # stream (default priority) are consumed without a synchronisation in between, and torch kernels that
    # follow on that stream see the tree
    N, F, nb, L = 200_000, 28, 63, 31
    rng = np.random.default_rng(12)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-(bins[:, 3].astype(np.float64) - nb / 2) * 6.0 / nb))).astype(np.float32)
    dbins = torch.from_numpy(bins).cuda(); dy = torch.from_numpy(y).cuda()
    ctx = _ctx(N, F, nb, L=L)
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        score = torch.zeros(N, device="cuda")
        for _ in range(20):                                 # a queue of torch work in front of the library's
            score = score * 0.5 + 0.0
        p = torch.sigmoid(score)
        g = (p - dy).contiguous(); h = (p * (1 - p)).contiguous()
        t = ctx.grow_tree(dbins, g, h, 3, 3, 8, 0, L, min_data_in_leaf=20)
        n_leaves_dev = t.n_leaves.clone()                   # a torch kernel behind the library's work
        split_feature = t.split_feature.clone()
    side.synchronize()
    e = oracle.grow_tree(bins, nb, g.cpu().numpy(), h.cpu().numpy(), 3, 3, 8, 0, L, min_data=20)
    _compare_tree(t, e, N)
    assert int(n_leaves_dev.item()) == e.n_leaves
    assert np.array_equal(split_feature.cpu().numpy()[: e.n_leaves - 1], e.split_feature)


def test_create_rejects_leaf_budgets_beyond_the_bookkeeping():
    from paper_2207_09682_amd import QgbdtError
    with pytest.raises(QgbdtError):
        _ctx(1000, 8, 32, L=4096)
    ctx = _ctx(1000, 8, 32, L=600)            # fits
    assert ctx.workspace_bytes > 0


def test_measured_stream_read_is_plausible():
    from paper_2207_09682_amd import QgbdtError
    ctx = _ctx(1000, 8, 32, L=8)
    buf = torch.zeros(64 << 20, dtype=torch.uint8, device="cuda")
    gbps = ctx.measure_stream_read(buf, reps=5)
    assert 200.0 < gbps < 40000.0                                  # 64 MiB may be served by the on-die caches
    v = ctx.stream_read_variant                                     # the best of the swept launch shapes
    assert v["loads_in_flight"] in (4, 8, 16) and v["workgroups"] >= 1 and v["non_temporal"] in (False, True)
    assert ctx.measure_stream_read(buf[:16], reps=1) > 0.0
    with pytest.raises(QgbdtError):
        ctx.measure_stream_read(buf[8:8 + 64], reps=1)              # not 16-byte aligned


def test_tree_stats_after_a_tree():
    cfg = workloads.CONFIGS[0]
    wl = workloads.make_workload(cfg)
    ctx = _ctx(wl.n_rows, cfg.n_features, cfg.n_bins, L=cfg.num_leaves)
    g, h = workloads.gradients(wl, torch.zeros(wl.n_rows))
    t = ctx.grow_tree(wl.bins.cuda(), g.cuda(), h.cuda(), 2, 2, 0, 0, cfg.num_leaves)
    rounds, expanded, committed, nodes = ctx.tree_stats()
    n = int(t.n_leaves.item())
    assert committed == n - 1 and expanded >= committed and nodes == 2 * expanded + 1 and 1 <= rounds <= expanded + 1


def test_profile_separates_root_builds_from_the_rounds_builds():
    # with profiling on, every histogram launch is timed; those that are a tree's root build are reported apart
    cfg = workloads.CONFIGS[0]
    wl = workloads.make_workload(cfg)
    ctx = _ctx(wl.n_rows, cfg.n_features, cfg.n_bins, L=cfg.num_leaves)
    g, h = workloads.gradients(wl, torch.zeros(wl.n_rows))
    dbins, dg, dh = wl.bins.cuda(), g.cuda(), h.cuda()
    ctx.set_profiling(True)
    ctx.read_profile()
    rounds = 0
    for it in range(3):
        ctx.grow_tree(dbins, dg, dh, 2, 2, 0, it, cfg.num_leaves)
        rounds += ctx.tree_stats()[0]
    gh, _ = ctx.quantize_gradients(dg, dh, 2, 2, 0, 0)
    ctx.build_histograms(dbins, gh, bits_g=2, bits_h=2)            # a stand-alone build is not a tree's root
    root_ms, root_n = ctx.read_profile_roots()
    ms, n, nbytes = ctx.read_profile()
    ctx.set_profiling(False)
    assert root_n == 3 and 0.0 < root_ms < ms
    assert n >= 3 + rounds + 1 and nbytes > 3 * wl.n_rows * (cfg.n_features + 2)
    assert ctx.read_profile_roots() == (0.0, 0)                     # read_profile has reset the timers


# ----------------------------------------------------------------------------
# 16-bit bins (more than 256 bins per feature)
# ----------------------------------------------------------------------------

def _ctx16(N, F, nb, L=63):
    from paper_2207_09682_amd import Context
    return Context(N, F, nb, max_leaves=L, bin_bytes=2)


@pytest.mark.parametrize("N,F,nb,bg,bh", [(20000, 10, 600, 3, 3), (9000, 33, 1024, 4, 4), (5000, 100, 300, 3, 8),
                                          (3000, 1, 1000, 2, 2)])
@pytest.mark.parametrize("acc", [0, 16, 32])
def test_histogram_uint16_bins_bit_exact(N, F, nb, bg, bh, acc):
    rng = np.random.default_rng(N + F + nb)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint16)
    bins[:, 0] = np.where(rng.random(N) < 0.5, nb - 1, bins[:, 0])
    gq, hq, gh = _rand_gh(rng, N, bg, bh, "cuda")
    ctx = _ctx16(N, F, nb)
    dbins = torch.from_numpy(bins).cuda()
    idx = np.sort(rng.choice(N, N // 3, replace=False)).astype(np.int32)
    didx = torch.from_numpy(idx).cuda()
    for kw in (dict(), dict(begin=11, count=N - 30), dict(row_idx=idx), dict(row_idx=idx, begin=2, count=1),
               dict(begin=4, count=0)):
        exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, **kw))
        gkw = dict(kw)
        if "row_idx" in gkw:
            gkw["row_idx"] = didx
            gkw.setdefault("count", idx.size)
        got = ctx.build_histograms(dbins, gh, bits_g=bg, bits_h=bh, acc_width=acc, **gkw).cpu().numpy().reshape(nb, F)
        assert np.array_equal(got, exp), (kw.keys(), acc)


def test_find_best_splits_and_partition_uint16_bins():
    from paper_2207_09682_amd import unpack_splits
    rng = np.random.default_rng(77)
    N, F, nb = 30000, 6, 1000
    bins = rng.integers(0, nb, (N, F)).astype(np.uint16)
    bins[:, 3] = bins[:, 0]                                                # duplicated feature: ties
    g = ((bins[:, 0] > 700).astype(np.float32) - 0.5 + rng.normal(size=N)).astype(np.float32)
    h = rng.uniform(0.01, 0.25, N).astype(np.float32)
    gq, hq, d = oracle.quantize_gradients(g, h, 3, 3, 9, 1)
    leaves = [np.arange(N, dtype=np.int32), np.arange(0, N, 7, dtype=np.int32), np.arange(30, dtype=np.int32)]
    hists = [oracle.build_histograms(bins, nb, gq, hq, row_idx=r) for r in leaves]
    stats = np.array([[len(r), gq[r].astype(np.int64).sum(), hq[r].astype(np.int64).sum()] for r in leaves], np.int64)
    ctx = _ctx16(N, F, nb)
    dh = torch.from_numpy(np.stack([_pack_hist(x).reshape(-1) for x in hists])).cuda()
    got = unpack_splits(ctx.find_best_splits(dh, torch.from_numpy(stats).cuda(), torch.from_numpy(d).cuda(), 5, 0.0))
    for k, r in enumerate(leaves):
        e = oracle.find_best_split(hists[k], len(r), int(stats[k, 1]), int(stats[k, 2]), d[0], d[1], 5, 0.0)
        assert (got[k]["feature"], got[k]["bin"]) == (e.feature, e.bin)
        assert got[k]["gain"] == pytest.approx(e.gain, rel=RTOL, abs=0.0)
    idx = np.sort(rng.choice(N, N // 2, replace=False)).astype(np.int32)
    dbins = torch.from_numpy(bins).cuda()
    for begin, count, f, b in ((0, idx.size, 5, 600), (9, idx.size - 20, 0, 255), (0, idx.size, 1, 256), (3, 0, 0, 5)):
        exp, nl = oracle.partition_rows(bins, idx, begin, count, f, b)
        didx = torch.from_numpy(idx.copy()).cuda()
        assert int(ctx.partition_rows(dbins, didx, begin, count, f, b).item()) == nl
        assert np.array_equal(didx.cpu().numpy(), exp)


def test_grow_tree_uint16_bins():
    rng = np.random.default_rng(5)
    N, F, nb, L = 60000, 12, 800, 63
    x = rng.normal(size=(N, F)).astype(np.float32)
    edges = np.quantile(x[:, :], np.linspace(0, 1, nb + 1)[1:-1], axis=0)
    bins = np.stack([np.searchsorted(edges[:, f], x[:, f]) for f in range(F)], axis=1).astype(np.uint16)
    w = rng.normal(size=F)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-(x @ w)))).astype(np.float32)
    score = np.zeros(N, np.float32)
    ctx = _ctx16(N, F, nb, L=L)
    dbins = torch.from_numpy(bins).cuda()
    for it in range(2):
        p = 1.0 / (1.0 + np.exp(-score.astype(np.float64)))
        g = (p - y).astype(np.float32); h = (p * (1 - p)).astype(np.float32)
        t = ctx.grow_tree(dbins, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), 3, 3, 21, it, L,
                          min_data_in_leaf=20)
        e = oracle.grow_tree(bins, nb, g, h, 3, 3, 21, it, L, min_data=20)
        _compare_tree(t, e, N)
        assert int(np.max(e.split_bin)) > 255                               # thresholds beyond 8 bits are in play
        n = e.n_leaves
        for l in range(n):
            rows = e.row_idx[e.leaf_begin[l]: e.leaf_begin[l] + e.leaf_count[l]]
            score[rows] += np.float32(0.1 * e.leaf_value[l])


def test_uint16_context_rejects_wrong_bin_type_and_too_many_bins():
    from paper_2207_09682_amd import Context, QgbdtError
    with pytest.raises(QgbdtError):
        Context(100, 4, 1025, max_leaves=7, bin_bytes=2)
    with pytest.raises(QgbdtError):
        Context(100, 4, 257, max_leaves=7, bin_bytes=1)
    ctx = _ctx16(100, 4, 300, L=7)
    with pytest.raises(TypeError):
        ctx.build_histograms(torch.zeros((100, 4), dtype=torch.uint8, device="cuda"),
                             torch.zeros(100, dtype=torch.int16, device="cuda"), bits_g=3, bits_h=3)


# ----------------------------------------------------------------------------
# bound bin matrix: feature-major copy for the partition of wide or ragged matrices
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("N,F,nb,L,bb", [(30000, 200, 255, 31, 1), (20000, 2000, 63, 15, 1), (9000, 33, 40, 15, 1),
                                         (12000, 12, 800, 15, 2), (50000, 28, 255, 31, 1)])
def test_grow_tree_with_bound_bins(N, F, nb, L, bb):
    from paper_2207_09682_amd import Context
    rng = np.random.default_rng(N + F)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint16 if bb == 2 else np.uint8)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-(bins[:, 1].astype(np.float64) - nb / 2) * 6.0 / nb))).astype(np.float32)
    g = (0.5 - y).astype(np.float32); h = np.full(N, 0.25, np.float32)
    e = oracle.grow_tree(bins, nb, g, h, 3, 3, 4, 0, L, min_data=5)
    ctx = Context(N, F, nb, max_leaves=L, bin_bytes=bb)
    dbins = torch.from_numpy(bins).cuda()
    dg, dh = torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda()
    ctx.bind_bins(dbins)
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e, N)
    other = dbins.clone()                                     # another matrix object: the copy is not used
    _compare_tree(ctx.grow_tree(other, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e, N)
    bins2 = bins.copy(); bins2[:, 1] = bins[::-1, 1]          # new contents, bound again
    e2 = oracle.grow_tree(bins2, nb, g, h, 3, 3, 4, 0, L, min_data=5)
    dbins.copy_(torch.from_numpy(bins2))
    ctx.bind_bins(dbins)
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e2, N)
    ctx.bind_bins(None)                                       # forgotten: the next tree does not use the copy
    _compare_tree(ctx.grow_tree(dbins, dg, dh, 3, 3, 4, 0, L, min_data_in_leaf=5), e2, N)


# Every choice of what a partition moves (row ids; row ids and packed gradients; those and the bin rows) grows the
# oracle's tree, bound or not: shapes that reach each gathered histogram kernel (dword per lane with one and with
# several tiles, ragged feature counts, 8- and 16-byte pieces of wide rows, 16-bit bins) and 64-bit local words.
@pytest.mark.parametrize("N,F,nb,L,bb,bits", [(70000, 28, 255, 63, 1, (3, 3)), (40000, 64, 255, 31, 1, (3, 8)),
                                              (30000, 30, 100, 31, 1, (3, 3)), (30000, 200, 255, 31, 1, (3, 8)),
                                              (9000, 2000, 63, 15, 1, (3, 3)), (20000, 20, 600, 31, 2, (4, 4)),
                                              (25000, 3, 16, 15, 1, (2, 2))])
def test_row_layouts_grow_the_same_tree(N, F, nb, L, bb, bits):
    from paper_2207_09682_amd import Context, ROWS_IDS, ROWS_IDS_GH, ROWS_ORDERED
    rng = np.random.default_rng(N * 7 + F)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint16 if bb == 2 else np.uint8)
    sig = (bins[:, F // 2].astype(np.float64) / nb - 0.5) * 4 + (bins[:, 0] > nb // 2) * 0.8
    y = (rng.random(N) < 1 / (1 + np.exp(-sig))).astype(np.float32)
    pr = 1 / (1 + np.exp(-rng.normal(scale=0.7, size=N)))
    g = (pr - y).astype(np.float32); h = (pr * (1 - pr)).astype(np.float32)
    e = oracle.grow_tree(bins, nb, g, h, bits[0], bits[1], 21, 0, L, min_data=5)
    dbins = torch.from_numpy(bins).cuda()
    dg, dh = torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda()
    layouts = [ROWS_IDS, ROWS_IDS_GH] + ([ROWS_ORDERED] if (bb == 1 and F % 4 == 0 and 16 <= F <= 64) else [])
    ctx = Context(N, F, nb, max_leaves=L, bin_bytes=bb)
    for bound in (False, True):
        if bound:
            ctx.bind_bins(dbins)
        for layout in layouts + layouts[:1]:                 # and back to the first one on the same context
            t = ctx.grow_tree(dbins, dg, dh, bits[0], bits[1], 21, 0, L, min_data_in_leaf=5, row_layout=layout)
            try:
                _compare_tree(t, e, N)
            except AssertionError as err:
                raise AssertionError(f"bound={bound} layout={layout}: {err}") from err


# ----------------------------------------------------------------------------
# seeded sweep over valid configurations
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_valid_configurations(seed):
    # 100 seeded draws per seed of (rows, features, bins, bin type, leaf budget, bit widths, accumulator setting,
    # bound matrix or not, rounding, minimum rows per leaf, what moves in a partition): two trees each, every output against the oracle
    from paper_2207_09682_amd import Context
    rng = np.random.default_rng(seed)
    for case in range(100):
        bb = 2 if rng.random() < 0.15 else 1
        N = int(rng.choice([1, 2, 3, 17, 100, 1000, 5000, 20000, 60000, 150000]))
        F = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 20, 28, 30, 32, 33, 48, 63, 64, 65, 72, 100, 128, 130, 200, 256, 300]))
        if N * F > 12_000_000:
            F = max(1, 12_000_000 // N)
        nb = int(rng.choice([2, 3, 4, 16, 63, 64, 100, 255, 256])) if bb == 1 else int(rng.choice([257, 300, 700, 1024]))
        L = int(rng.choice([2, 3, 7, 15, 31, 63]))
        bits = [(2, 2), (3, 3), (4, 4), (5, 5), (3, 8), (8, 2), (3, 0), (6, 3)][int(rng.integers(0, 8))]
        acc = int(rng.choice([0, 16, 32]))
        bind = bool(rng.random() < 0.5)
        rounding = int(rng.random() < 0.2)
        md = int(rng.choice([0, 1, 5, 20]))
        can_order = bb == 1 and F % 4 == 0 and 16 <= F <= 64
        layout = int(rng.choice([0, 0, 1, 2, 3] if can_order else [0, 0, 1, 2]))
        bins = rng.integers(0, nb, (N, F)).astype(np.uint16 if bb == 2 else np.uint8)
        if rng.random() < 0.3:
            bins[:, 0] = np.where(rng.random(N) < 0.8, 0, bins[:, 0])
        sig = (bins[:, F // 2].astype(np.float64) / nb - 0.5) * 3 + (bins[:, 0] > nb // 3) * 0.7
        y = (rng.random(N) < 1 / (1 + np.exp(-sig))).astype(np.float32)
        pr = 1 / (1 + np.exp(-rng.normal(scale=0.5, size=N)))
        g = (pr - y).astype(np.float32)
        h = (pr * (1 - pr)).astype(np.float32) if bits[1] != 0 else np.full(N, 1.0, np.float32)
        what = dict(case=case, N=N, F=F, nb=nb, bb=bb, L=L, bits=bits, acc=acc, bind=bind, rounding=rounding, md=md,
                    layout=layout)
        ctx = Context(N, F, nb, max_leaves=L, bin_bytes=bb)
        dbins = torch.from_numpy(bins).cuda()
        if bind:
            ctx.bind_bins(dbins)
        for it in range(2):
            t = ctx.grow_tree(dbins, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), bits[0], bits[1], 77, it, L,
                              min_data_in_leaf=md, acc_width=acc, rounding=rounding, row_layout=layout)
            e = oracle.grow_tree(bins, nb, g, h, bits[0], bits[1], 77, it, L, min_data=md, rounding=rounding)
            try:
                _compare_tree(t, e, N)
            except AssertionError as err:
                raise AssertionError(f"{what}: {err}") from err
        del ctx


@pytest.mark.parametrize("seed", [21, 22])
def test_random_histogram_slices(seed):
    # seeded draws of shape, bit widths, accumulator setting and row set (contiguous slice or gathered slice of a
    # sorted row list) for the stand-alone build; bit-exact against the oracle
    from paper_2207_09682_amd import Context
    rng = np.random.default_rng(seed)
    for case in range(120):
        bb = 2 if rng.random() < 0.15 else 1
        N = int(rng.choice([1, 5, 64, 1000, 4097, 30000, 120000]))
        F = int(rng.choice([1, 3, 4, 6, 9, 16, 28, 31, 40, 64, 66, 96, 136, 200, 272, 520]))
        if N * F > 10_000_000:
            F = max(1, 10_000_000 // N)
        nb = int(rng.choice([2, 5, 16, 63, 128, 255, 256])) if bb == 1 else int(rng.choice([300, 1024]))
        bg, bh = [(2, 2), (3, 3), (4, 4), (5, 5), (3, 8), (8, 8), (2, 7), (3, 0)][int(rng.integers(0, 8))]
        acc = int(rng.choice([0, 16, 32]))
        bins = rng.integers(0, nb, (N, F)).astype(np.uint16 if bb == 2 else np.uint8)
        kg, kh = 2 ** (bg - 1) - 1, (2 ** bh - 2 if bh else 1)
        gq = rng.integers(-kg, kg + 1, N).astype(np.int8)
        hq = rng.integers(0, kh + 1, N).astype(np.uint8) if bh else np.ones(N, np.uint8)
        gh = torch.from_numpy(_pack_gh(gq, hq)).cuda()
        ctx = Context(N, F, nb, max_leaves=4, bin_bytes=bb)
        dbins = torch.from_numpy(bins).cuda()
        kw = {}
        if rng.random() < 0.5:
            m = int(rng.integers(1, N + 1))
            idx = np.sort(rng.choice(N, m, replace=False)).astype(np.int32)
            b = int(rng.integers(0, m)); c = int(rng.integers(0, m - b + 1))
            kw = dict(row_idx=idx, begin=b, count=c)
        else:
            b = int(rng.integers(0, N)); c = int(rng.integers(0, N - b + 1))
            kw = dict(begin=b, count=c)
        exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, **kw))
        gkw = dict(kw)
        if "row_idx" in gkw:
            gkw["row_idx"] = torch.from_numpy(gkw["row_idx"]).cuda()
        got = ctx.build_histograms(dbins, gh, bits_g=bg, bits_h=bh, acc_width=acc, **gkw).cpu().numpy().reshape(nb, F)
        assert np.array_equal(got, exp), dict(case=case, N=N, F=F, nb=nb, bb=bb, bits=(bg, bh), acc=acc,
                                              begin=kw["begin"], count=kw["count"], gathered="row_idx" in kw)
        del ctx


# ----------------------------------------------------------------------------
# most-frequent-bin skipping (bound, skewed wide matrices)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("N,F,nb,bits", [(40000, 200, 255, (3, 8)), (25000, 2000, 63, (3, 3)), (30000, 72, 256, (4, 4)),
                                         (20000, 136, 100, (3, 8))])
def test_frequent_bin_skipping_on_skewed_wide_matrices(N, F, nb, bits):
    # most features have one bin that holds most rows (a different bin per feature), some have none: the wide-row
    # kernels leave that bin out, the stand-alone build fills it in afterwards, the split search of grow_tree
    # rebuilds it from the leaf totals; everything bit-exact against the oracle
    from paper_2207_09682_amd import Context
    rng = np.random.default_rng(N + F)
    bins = rng.integers(0, nb, (N, F)).astype(np.uint8)
    fav = rng.integers(0, nb, F)
    for f in range(F):
        if f % 5 != 4:                                        # four features in five are skewed
            bins[rng.random(N) < 0.75, f] = fav[f]
    bg, bh = bits
    gq, hq, gh = _rand_gh(rng, N, bg, bh, "cuda")
    ctx = Context(N, F, nb, max_leaves=31)
    dbins = torch.from_numpy(bins).cuda()
    ctx.bind_bins(dbins)
    idx = np.sort(rng.choice(N, N // 3, replace=False)).astype(np.int32)
    didx = torch.from_numpy(idx).cuda()
    for acc in (0, 16, 32):
        for kw in (dict(), dict(begin=13, count=N - 50), dict(row_idx=idx), dict(row_idx=idx, begin=7, count=idx.size // 2),
                   dict(begin=3, count=1)):
            exp = _pack_hist(oracle.build_histograms(bins, nb, gq, hq, **kw))
            gkw = dict(kw)
            if "row_idx" in gkw:
                gkw["row_idx"] = didx
                gkw.setdefault("count", idx.size)
            got = ctx.build_histograms(dbins, gh, bits_g=bg, bits_h=bh, acc_width=acc, **gkw).cpu().numpy().reshape(nb, F)
            assert np.array_equal(got, exp), (kw.keys(), acc)
    y = (rng.random(N) < 1.0 / (1.0 + np.exp(-((bins[:, 0] == fav[0]) * 1.5 - (bins[:, 1] > nb // 2) * 1.0)))).astype(np.float32)
    score = np.zeros(N, np.float32)
    for it in range(2):
        pr = 1.0 / (1.0 + np.exp(-score.astype(np.float64)))
        g = (pr - y).astype(np.float32); h = (pr * (1 - pr)).astype(np.float32)
        for acc in (0, 32):
            t = ctx.grow_tree(dbins, torch.from_numpy(g).cuda(), torch.from_numpy(h).cuda(), bg, bh, 5, it, 31,
                              min_data_in_leaf=10, acc_width=acc)
            e = oracle.grow_tree(bins, nb, g, h, bg, bh, 5, it, 31, min_data=10)
            _compare_tree(t, e, N)
        for l in range(e.n_leaves):
            rows = e.row_idx[e.leaf_begin[l]: e.leaf_begin[l] + e.leaf_count[l]]
            score[rows] += np.float32(0.3 * e.leaf_value[l])

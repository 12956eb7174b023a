"""Host-side checks of the histogram launch plans (no GPU): the index arithmetic of the histogram kernels, of the
hand-over of a row group's local bins to its slot and of the slot reduction is replayed in numpy from the plan the
library reports for a shape (qgbdt_describe_hist_plan), and every address is checked against the sizes of what it
points into -- the matrix, the local bins, the workspace section of the slots, the histogram."""
import itertools

import numpy as np
import pytest

from paper_2207_09682_amd.binding import describe_hist_plan

SHAPES = [  # n_rows, n_features, n_bins, max_leaves, bin_bytes
    (10_500_000, 28, 255, 255, 1), (1_000_000, 28, 255, 255, 1), (10_000, 28, 63, 15, 1),
    (400_000, 2000, 63, 63, 1), (20_000_000, 200, 255, 511, 1), (463_715, 90, 255, 255, 1),
    (5000, 3, 256, 15, 1), (9000, 5, 16, 15, 1), (5000, 65, 255, 31, 1), (7000, 64, 256, 31, 1),
    (5000, 36, 100, 31, 1), (30_000, 72, 256, 31, 1), (100_000, 1, 2, 4, 1), (100_000, 2048, 256, 15, 1),
    (20_000, 10, 600, 31, 2), (9000, 33, 1024, 31, 2), (5000, 100, 300, 31, 2), (3000, 1, 700, 7, 2),
    (2_000_000, 40, 600, 63, 2), (160_000_000, 28, 255, 15, 1), (2_400_000, 2000, 63, 7, 1),
    # edges: very wide rows, many bins of both widths, tile widths around the 128-byte piece, the leaf limit
    (50_000, 4096, 256, 31, 1), (20_000, 10_000, 64, 15, 1), (3000, 2000, 1024, 7, 2), (1000, 7, 2, 658, 1),
    (300, 255, 256, 7, 1), (100_000, 16, 256, 15, 1), (100_000, 124, 255, 15, 1), (100_000, 128, 255, 15, 1),
    (50_000, 132, 200, 15, 1), (8000, 257, 1024, 15, 2),
    # long narrow matrices of other row widths (two-level byte-stream builds)
    (3_000_000, 16, 255, 15, 1), (3_000_000, 40, 255, 15, 1), (3_000_000, 48, 255, 15, 1), (6_000_000, 20, 100, 15, 1),
]
BITS = [(2, 2), (3, 3), (4, 4), (5, 5), (3, 8), (3, 0), (8, 8)]


def _plans(shape):
    N, F, nb, L, bb = shape
    for (bg, bh), acc, skew in itertools.product(BITS, (0, 16, 32), (False, True)):
        yield (bg, bh, acc, skew), describe_hist_plan(N, F, nb, L, bb, bg, bh, acc, skew)


def _rows_fitting_word32(bg, bh, s):
    kg, kh = 2 ** (bg - 1) - 1, (2 ** bh - 2 if bh else 1)
    return min((2 ** (31 - s) - 1) // kg, (2 ** s - 1) // kh)


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"{s[0]}x{s[1]}_nb{s[2]}_L{s[3]}_b{s[4]}")
def test_plan_invariants(shape):
    N, F, nb, L, bb = shape
    for key, p in _plans(shape):
        bg, bh, acc, skew = key
        wbytes = 4 if p["acc_width"] == 16 else 8
        npd = 4 // bb
        # tiles cover the features, local bins fit the LDS, and only the wide-row kernels go beyond 64 KB
        assert p["n_tiles"] == -(-F // p["ft"]) and p["ft"] >= 1
        assert p["lds_bytes"] <= 160 * 1024
        assert p["lds_bytes"] <= 64 * 1024 or p["wide_v"] > 0, key
        assert p["slot_bytes"] >= p["lds_bytes"] and p["slot_bytes"] % 16 == 0
        # the flat grid is cut into (XCD, tile, lane): lanes come in whole groups of 8
        assert p["max_lanes"] % 8 == 0 and p["max_lanes"] >= 8 and p["max_groups"] >= 1
        # the slots of any launch of this shape lie inside the workspace section sized from the shape alone
        assert p["max_items"] * p["n_tiles"] * p["slot_bytes"] <= p["partial_bytes"], key
        # width rule (Sec. 7.4.3): a chunk never holds more rows than the fields of a local word take
        if p["acc_width"] == 16:
            assert p["chunk_rows"] <= _rows_fitting_word32(bg, bh, p["hshift"]), key
            assert p["chunk_rows"] >= max(_rows_fitting_word32(bg, bh, s) for s in range(8, 25)), key   # the best split
        assert 1 <= p["single_rows"] <= p["chunk_rows"]
        last = F - (p["n_tiles"] - 1) * p["ft"]
        if not p["bytewise"]:
            assert p["dpr"] * p["rows_per_it"] <= 64 and p["rows_per_it"] >= 1
            assert last >= min(npd, F), key                          # every tile row holds a whole dword
            if p["wide_v"]:
                assert bb == 1 and F % p["wide_v"] == 0 and p["ft"] % p["wide_v"] == 0 and last % p["wide_v"] == 0
                assert p["ftp"] == (p["ft"] + p["ft"] // 4 if p["pad16"] else p["ft"])
            else:
                assert p["ftp"] >= p["ft"]
            assert p["lds_bytes"] == p["ftp"] * nb * wbytes
        if p["flat_lanes"]:
            assert bb == 1 and p["n_tiles"] == 1 and (16 * p["flat_lanes"]) % F == 0 and p["flat_lanes"] <= 64
            assert p["flat_rows"] * F == 16 * p["flat_lanes"]


def _walk_two_level_groups(p, F, count, begin, groups):
    """The two-level byte-stream kernel's walk over one build of `count` rows from row `begin`: every row lies in
    exactly one group, whole blocks start 16-byte aligned, and no more rows than a chunk holds are added to the 32-bit
    working words between two folds."""
    n_waves, U = 16, 2
    align_rows = 16 // (16 if F % 16 == 0 else 8 if F % 8 == 0 else 4)
    BR = U * p["flat_rows"]
    head = min(count, (align_rows - begin % align_rows) % align_rows)
    rpg = max(BR, -(-(-(-(count - head) // groups)) // BR) * BR)
    fold_rounds = max(1, (p["chunk_rows"] - BR - align_rows) // (n_waves * BR))
    covered = head
    for g in range(groups):
        gbegin = min(count, head + g * rpg)
        gend = min(count, gbegin + rpg)
        grow = gend - gbegin
        n_blocks = grow // BR
        rounds = -(-n_blocks // n_waves)
        if n_blocks:
            assert ((begin + gbegin) * F) % 16 == 0
        since_fold = 0
        for r in range(rounds):
            since_fold += BR * max(0, min(n_waves, n_blocks - r * n_waves))
            if (r + 1) % fold_rounds == 0 and r + 1 < rounds:
                assert since_fold <= p["chunk_rows"]
                since_fold = 0
        since_fold += (grow - n_blocks * BR) + (head if g == 0 else 0)
        assert since_fold <= p["chunk_rows"], (F, count, begin, g)
        assert (begin + gend) * F <= (begin + count) * F                             # the last load ends inside the slice
        covered += grow
    assert covered == count


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"{s[0]}x{s[1]}_nb{s[2]}_L{s[3]}_b{s[4]}")
def test_plan_of_one_long_contiguous_build(shape):
    # the plan of a stand-alone build of all rows: for narrow matrices the byte-stream kernel's two-level form
    # (32-bit working words folded into 64-bit words in LDS), whose slots hold the 64-bit words
    N, F, nb, L, bb = shape
    seen_two = False
    for (bg, bh), acc in itertools.product(BITS, (0, 16, 32)):
        p = describe_hist_plan(N, F, nb, L, bb, bg, bh, acc, False, rows=N, n_builds=1)
        assert p["max_items"] * p["n_tiles"] * p["slot_bytes"] <= p["partial_bytes"]
        assert p["max_lanes"] % 8 == 0 and p["lds_bytes"] <= 160 * 1024
        groups = -(-N // p["target_rows"])
        assert 1 <= groups <= p["max_items"]
        if p["two_level"]:
            seen_two = True
            words = nb * p["ftp"]
            assert acc != 32 and p["acc_width"] == 16 and p["flat_lanes"] > 0 and p["n_tiles"] == 1 and p["threads"] == 1024
            assert p["lds_bytes"] == ((4 * words + 15) // 16) * 16 + 8 * words
            assert p["slot_bytes"] >= 8 * words and p["slot_bytes"] % 16 == 0
            assert groups <= p["max_lanes"] == 256                                   # one group per CU, all resident
            assert p["chunk_rows"] <= _rows_fitting_word32(bg, bh, p["hshift"])      # the working words still follow the width rule
            assert N >= 2 * 256 * p["chunk_rows"]
            for begin in (0, 1, 3):                                                  # a slice that starts off a 16-byte boundary
                _walk_two_level_groups(p, F, N - begin, begin, -(-(N - begin) // p["target_rows"]))
        else:
            # without the fold a group of 32-bit words must not be longer than the item table allows one-chunk groups, or the width is 64
            assert p["acc_width"] == 32 or acc == 16 or N // p["single_rows"] < p["max_items"] - 2
    if bb == 1 and 16 <= F <= 64 and F % 4 == 0 and N >= 2_000_000:
        assert seen_two


def _lane_columns(p, F, bb, tile, dword_kernel=False):
    """(first byte of the lane's load inside the row, bytes loaded, LDS word columns it may update) per active lane of
    one tile, as the dword-per-lane and the wide-row kernels compute them."""
    npd = 4 // bb
    f0 = tile * p["ft"]
    ft = min(p["ft"], F - f0)
    out = []
    if p["wide_v"] and not dword_kernel:
        V = p["wide_v"]
        P = p["ft"] // V
        for lane in range(64):
            c = lane % P
            if V * c >= ft:
                continue                                             # the lane sits out (its load aliases piece 0)
            cols = [20 * c + 4 * i + k for i in range(4) for k in range(4)] if V == 16 else [8 * c + k for k in range(8)]
            out.append((f0 + V * c, V, cols))
        return out, ft
    for lane in range(64):
        q, r = lane % p["dpr"], lane // p["dpr"]
        if not (r < p["rows_per_it"] and npd * q < ft):
            continue
        nval = min(npd, ft - npd * q) if p["ragged"] else npd
        back = npd - nval
        cols = [npd * q + c + (4 * (q >> 2) if p["pad16"] else 0) for c in range(nval)]
        out.append(((f0 + npd * q - back) * bb, 4, cols))
    return out, ft


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"{s[0]}x{s[1]}_nb{s[2]}_L{s[3]}_b{s[4]}")
def test_kernel_addresses_stay_inside_their_buffers(shape):
    N, F, nb, L, bb = shape
    rng = np.random.default_rng(F * 7 + nb)
    for key, p in _plans(shape):
        if p["bytewise"]:
            continue                                                 # one load per bin, indexed by (row, feature) directly
        wbytes = 4 if p["acc_width"] == 16 else 8
        row_bytes = F * bb
        for tile in {0, p["n_tiles"] // 2, p["n_tiles"] - 1}:
            lanes, ft = _lane_columns(p, F, bb, tile)
            assert lanes, key
            if p["wide_v"]:   # a matrix that is not 16-byte aligned takes the dword kernel with the same (padded) plan
                lanes = lanes + _lane_columns(p, F, bb, tile, dword_kernel=True)[0]
            for off, nbytes, cols in lanes:
                assert 0 <= off and off + nbytes <= row_bytes, (key, tile, off)       # no load leaves its row
                for col in cols:
                    assert 0 <= col < p["ftp"], (key, tile, col)                       # LDS word inside the bin row
                    assert (nb - 1) * p["ftp"] * wbytes + col * wbytes + wbytes <= p["lds_bytes"]
        # work items of a batched launch: however the rows are spread over the builds, the items fit the table
        for n_builds in {1, 2, min(L, 17), L}:
            for total in {1, 1000, N // 7 + 1, N}:
                t = describe_hist_plan(N, F, nb, L, bb, key[0], key[1], key[2], key[3], rows=total, n_builds=n_builds)["target_rows"] \
                    if n_builds > 1 else None
                if t is None:
                    continue
                cuts = np.sort(rng.integers(0, total + 1, n_builds - 1))
                rows = np.diff(np.concatenate([[0], cuts, [total]]))
                groups = np.maximum(1, -(-rows // t))
                assert int(groups.sum()) <= p["max_items"], (key, n_builds, total, t)
        # slot of the last item a launch can have, and the reduce kernel's walk over the slots
        slots_end = ((p["max_items"] - 1) * p["n_tiles"] + p["n_tiles"] - 1) * p["slot_bytes"] + p["lds_bytes"]
        assert slots_end <= p["partial_bytes"]
        tile_words = nb * p["ftp"]
        xb = -(-tile_words // 256)
        w = np.arange(xb * 256)
        b, f = w // p["ftp"], w % p["ftp"]
        if p["pad16"]:
            g, o = f // 20, f % 20
            f = np.where(o < 16, 16 * g + o, -1)
        for tile in {0, p["n_tiles"] - 1}:
            ftw = min(p["ft"], F - tile * p["ft"])
            ok = (b < nb) & (f >= 0) & (f < ftw)
            assert ok.any()
            assert int(w[ok].max()) * wbytes + wbytes <= p["slot_bytes"]               # word inside the slot
            hoff = b[ok] * F + tile * p["ft"] + f[ok]
            assert 0 <= int(hoff.min()) and int(hoff.max()) < F * nb                   # word inside the histogram
            assert np.unique(hoff).size == hoff.size                                   # every word reduced once


def test_the_launch_shape_of_an_old_unexplained_fault_is_in_bounds():
    # A stand-alone build of 400,000 x 2000 (63 bins, 3-bit) once faulted on the GPU while a development knob forced
    # 196 row groups (16 tiles).  With today's plan for that shape and the forced group count, every slot the
    # kernels and the reduce kernel address lies inside the slot section, every load inside the matrix.
    N, F, nb, L = 400_000, 2000, 63, 63
    p = describe_hist_plan(N, F, nb, L, 1, 3, 3, 0, False, rows=N)
    groups = 196
    assert groups <= p["max_items"]
    lanes = -(-groups // 8) * 8
    grid = lanes * p["n_tiles"]
    seen = set()
    for wg in range(grid):                                           # workgroup -> (tile, row-group lane)
        xcd, s = wg & 7, wg >> 3
        tile, glane = s % p["n_tiles"], (s // p["n_tiles"]) * 8 + xcd
        if glane >= groups:
            continue
        seen.add((glane, tile))
        slot = (glane * p["n_tiles"] + tile) * p["slot_bytes"]
        assert slot + p["lds_bytes"] <= p["partial_bytes"]
    assert len(seen) == groups * p["n_tiles"]                         # every (group, tile) has exactly one workgroup
    rows_per_group = -(-N // groups)
    for item in (0, groups - 1):
        gbegin = min(N, item * rows_per_group); gend = min(N, gbegin + rows_per_group)
        assert gend - gbegin <= p["chunk_rows"]                      # one chunk: handed over with plain stores
        for tile in (0, p["n_tiles"] - 1):
            for off, nbytes, _ in _lane_columns(p, F, 1, tile)[0]:
                assert (gend - 1) * F + off + nbytes <= N * F

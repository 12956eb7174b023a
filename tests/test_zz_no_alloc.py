"""The entry point that allocates nothing (qgbdt_find_best_splits_static: scratch in a fixed array inside the
library) against the existing qgbdt_find_best_splits, through the C ABI: identical records, on two calls in a row,
the second with a smaller input."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _histograms(rng, n, F, nb, dev):
    """n random packed 32|32 histograms [n][nb][F] with their leaf totals [n][3]."""
    G = rng.integers(-2000, 2000, (n, nb, F)).astype(np.int64)
    H = rng.integers(0, 3000, (n, nb, F)).astype(np.int64)
    H[:, :, 0] = rng.integers(0, 3, (n, nb))                      # a feature with many empty bins
    # every feature of a leaf must sum to the leaf's totals: put the difference into the last bin
    tg = G.sum(axis=1).max(axis=1) + 10; th = H.sum(axis=1).max(axis=1) + 10
    G[:, -1, :] += tg[:, None] - G.sum(axis=1)
    H[:, -1, :] += th[:, None] - H.sum(axis=1)
    hist = (G << 32) + H
    stats = np.stack([th // 2, tg, th], axis=1).astype(np.int64)   # n_rows, sum g~, sum h~
    return torch.from_numpy(hist.reshape(n, nb * F)).to(dev), torch.from_numpy(stats).to(dev)


@pytest.mark.parametrize("F,nb", [(28, 255), (200, 63)])
def test_static_split_search_equals_the_workspace_one(F, nb):
    from paper_2207_09682_amd import Context, QgbdtError
    rng = np.random.default_rng(F)
    ref = Context(1000, F, nb, max_leaves=31)                       # its scratch is part of its workspace
    sta = Context(1000, F, nb, max_leaves=31, workspace_flags=0)
    sta.detach_workspace()                                          # no workspace at all
    delta = torch.tensor([0.25, 0.125], dtype=torch.float32, device="cuda")
    out = torch.empty((300, 56), dtype=torch.uint8, device="cuda")
    for n in (300, 37, 1):                                          # consecutive calls share the array
        hist, stats = _histograms(rng, n, F, nb, "cuda")
        want = ref.find_best_splits(hist, stats, delta, min_data_in_leaf=5)
        out.fill_(0xEE)
        got = sta.find_best_splits_static(hist, stats, delta, out[:n], min_data_in_leaf=5)
        torch.cuda.synchronize()
        assert torch.equal(got, want), n
        assert bool((out[n:] == 0xEE).all())                        # nothing written past the n records
        feats = want[:, 8:12].contiguous().view(torch.int32).cpu().numpy().ravel()
        assert (feats >= 0).sum() > 0                               # the comparison is not of empty results
    # beyond what the fixed array holds: refused with a message, nothing launched
    too_many = (4 << 20) // (48 + 24 * F) + 1
    hist1, stats1 = _histograms(rng, 1, F, nb, "cuda")
    with pytest.raises(QgbdtError) as ei:
        # (the binding derives n from stats: hand it a long stats tensor)
        sta.find_best_splits_static(hist1, stats1.expand(too_many, 3).contiguous(), delta,
                                    torch.empty((too_many, 56), dtype=torch.uint8, device="cuda"))
    assert "scratch" in str(ei.value)

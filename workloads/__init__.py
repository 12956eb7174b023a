"""Seeded synthetic inputs for the five benchmark configurations.

This module only produces *inputs* (bin matrices, labels, per-row gradients and
hessians of the loss).  It holds none of the method's arithmetic (no quantizer,
histogram, split or refit code) and serves both the CPU oracle and the GPU
library, which never see each other.

The generators stand in for the public datasets the paper measures on (their
shapes are taken from its dataset table); no item of any such dataset is
reproduced here.  Everything is drawn from torch's seeded generators.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    n_rows: int
    n_features: int
    n_bins: int
    bits_g: int
    bits_h: int
    num_leaves: int
    n_trees: int
    loss: str            # "logistic" | "lambdarank"
    kind: str            # generator recipe
    learning_rate: float = 0.1
    min_data_in_leaf: int = 20
    seed: int = 0
    group_size: int = 100


CONFIGS = [
    Config("cfg1_10k_x28_63bins_2bit", 10_000, 28, 63, 2, 2, 15, 1, "logistic", "linear_bernoulli"),
    Config("cfg2_1M_x28_255bins_3bit", 1_000_000, 28, 255, 3, 3, 255, 10, "logistic", "linear_noisy"),
    Config("cfg3_10.5M_x28_255bins", 10_500_000, 28, 255, 3, 3, 255, 10, "logistic", "tree_ensemble"),
    Config("cfg4_400k_x2000_63bins_3bit", 400_000, 2000, 63, 3, 3, 63, 10, "logistic", "wide_sparse_linear"),
    Config("cfg5_20M_x200_255bins_rank", 20_000_000, 200, 255, 3, 8, 511, 10, "lambdarank", "skewed_bins_rank"),
]

# Workloads of the rows that widen the path (not benchmark configurations): a regression task with the
# shape of the paper's year-prediction dataset (463,715 x 90), squared error loss, whose hessians are
# constant and therefore not quantized (bits_h = 0).
EXTRA_CONFIGS = [
    Config("regression_464k_x90_255bins_l2", 463_715, 90, 255, 3, 0, 255, 10, "l2", "linear_regression"),
]


@dataclass
class Workload:
    cfg: Config
    bins: torch.Tensor            # uint8 [N, F], row-major, on `device`
    label: torch.Tensor           # float32 [N] (0/1 or relevance 0..4)
    extra: dict = field(default_factory=dict)

    @property
    def n_rows(self) -> int:
        return self.bins.shape[0]


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def quantile_bins(X: torch.Tensor, n_bins: int, sample: int = 200_000) -> torch.Tensor:
    """Per-feature equal-frequency binning; edges are quantiles of the first `sample` rows."""
    N, F = X.shape
    out = torch.empty((N, F), dtype=torch.uint8, device=X.device)
    qs = torch.arange(1, n_bins, device=X.device, dtype=torch.float32) / n_bins
    S = X[: min(N, sample)]
    for f in range(F):
        col = S[:, f].contiguous()
        edges = torch.quantile(col, qs) if col.numel() <= 1_000_000 else torch.quantile(col[:1_000_000], qs)
        out[:, f] = torch.bucketize(X[:, f].contiguous(), edges, right=False).to(torch.uint8)
    return out


def _random_tree_scores(X: torch.Tensor, n_trees: int, depth: int, gen: torch.Generator) -> torch.Tensor:
    N, F = X.shape
    score = torch.zeros(N, dtype=torch.float32, device=X.device)
    for _ in range(n_trees):
        n_int = (1 << depth) - 1
        feat = torch.randint(0, F, (n_int,), generator=gen, device=X.device)
        thr = torch.randn(n_int, generator=gen, device=X.device)
        leaf = torch.randn(1 << depth, generator=gen, device=X.device)
        node = torch.zeros(N, dtype=torch.int64, device=X.device)
        for _d in range(depth):
            f = feat[node]
            x = X.gather(1, f.unsqueeze(1)).squeeze(1)
            node = 2 * node + 1 + (x > thr[node]).to(torch.int64)
        score += leaf[node - n_int]
    return score


def make_workload(cfg: Config, n_rows: int | None = None, n_features: int | None = None,
                  device="cpu") -> Workload:
    """Builds the inputs of `cfg`; n_rows / n_features shrink it for tests."""
    N = n_rows or cfg.n_rows
    F = n_features or cfg.n_features
    dev = torch.device(device)
    gen = _gen(cfg.seed * 7919 + 17, dev)
    if cfg.kind in ("linear_bernoulli", "linear_noisy", "tree_ensemble"):
        X = torch.randn((N, F), generator=gen, device=dev)
        if cfg.kind == "tree_ensemble":
            K = 20
            z = _random_tree_scores(X, K, 6, gen) / math.sqrt(K)
            y = (torch.rand(N, generator=gen, device=dev) < torch.sigmoid(z)).float()
        else:
            w = torch.randn(F, generator=gen, device=dev)
            z = X @ w
            if cfg.kind == "linear_bernoulli":
                y = (torch.rand(N, generator=gen, device=dev) < torch.sigmoid(z)).float()
            else:
                y = (z > 0).float()
                flip = torch.rand(N, generator=gen, device=dev) < 0.10
                y = torch.where(flip, 1.0 - y, y)
        bins = quantile_bins(X, cfg.n_bins)
        return Workload(cfg, bins, y)
    if cfg.kind == "linear_regression":
        X = torch.randn((N, F), generator=gen, device=dev)
        w = torch.randn(F, generator=gen, device=dev) / math.sqrt(F)
        y = torch.tanh(X @ w) + 0.3 * torch.randn(N, generator=gen, device=dev)   # targets of order 1
        bins = quantile_bins(X, cfg.n_bins)
        return Workload(cfg, bins, y.float())
    if cfg.kind == "wide_sparse_linear":
        X = torch.rand((N, F), generator=gen, device=dev)
        nnz = min(50, F)
        pos = torch.randperm(F, generator=gen, device=dev)[:nnz]
        w = torch.zeros(F, device=dev)
        w[pos] = torch.randn(nnz, generator=gen, device=dev)
        z = (X - 0.5) @ w
        z = z / (z.std() + 1e-12)
        y = (torch.rand(N, generator=gen, device=dev) < torch.sigmoid(z)).float()
        bins = quantile_bins(X, cfg.n_bins)
        return Workload(cfg, bins, y)
    if cfg.kind == "skewed_bins_rank":
        gs = cfg.group_size
        N = (N // gs) * gs
        bins = torch.empty((N, F), dtype=torch.uint8, device=dev)
        w = torch.randn(F, generator=gen, device=dev) / math.sqrt(F)
        z = torch.empty(N, device=dev)
        step = max(gs, (4_000_000 // max(F, 1)) // gs * gs * 25)
        for a in range(0, N, step):
            b = min(N, a + step)
            dflt = torch.rand((b - a, F), generator=gen, device=dev) < 0.7
            vals = torch.randint(0, 255, (b - a, F), generator=gen, device=dev, dtype=torch.int32)
            blk = torch.where(dflt, torch.zeros_like(vals), vals)
            bins[a:b] = blk.to(torch.uint8)
            z[a:b] = (blk.float() / 255.0) @ w
        z = z + 0.5 * z.std() * torch.randn(N, generator=gen, device=dev)
        # relevance 0..4 = quantile bucket of the noisy linear score
        qs = torch.tensor([0.5, 0.75, 0.9, 0.97], device=dev)
        edges = torch.quantile(z[: min(N, 1_000_000)], qs)
        rel = torch.bucketize(z, edges).float()
        return Workload(cfg, bins, rel, {"group_size": gs})
    raise ValueError(cfg.kind)


# ----------------------------------------------------------------------------
# Loss derivatives (the inputs g_i, h_i of the hot path), fp32
# ----------------------------------------------------------------------------

def logistic_grad(score: torch.Tensor, y: torch.Tensor):
    """Binary log-loss: g = sigmoid(score) - y, h = sigmoid(score) (1 - sigmoid(score))."""
    p = torch.sigmoid(score.float())
    return (p - y).float().contiguous(), (p * (1.0 - p)).float().contiguous()


def lambdarank_grad(score: torch.Tensor, rel: torch.Tensor, group_size: int, chunk_queries: int = 8192):
    """Textbook LambdaRank with |delta NDCG| pair weights; queries are consecutive
    blocks of `group_size` rows; score ties are ranked by row id."""
    N = score.numel()
    Q = N // group_size
    s_all = score.float().view(Q, group_size)
    r_all = rel.float().view(Q, group_size)
    g = torch.zeros_like(s_all)
    h = torch.zeros_like(s_all)
    pos_discount = 1.0 / torch.log2(torch.arange(group_size, device=score.device, dtype=torch.float32) + 2.0)
    for a in range(0, Q, chunk_queries):
        s = s_all[a:a + chunk_queries]; r = r_all[a:a + chunk_queries]
        order = torch.argsort(s, dim=1, descending=True, stable=True)
        rank = torch.empty_like(order)
        rank.scatter_(1, order, torch.arange(group_size, device=s.device).expand_as(order))
        disc = pos_discount[rank]
        gain = torch.pow(2.0, r) - 1.0
        ideal = torch.sort(gain, dim=1, descending=True).values
        max_dcg = (ideal * pos_discount).sum(1, keepdim=True).clamp_min(1e-12)
        better = (r.unsqueeze(2) > r.unsqueeze(1)).float()                      # i more relevant than j
        rho = torch.sigmoid(-(s.unsqueeze(2) - s.unsqueeze(1)))                 # 1 / (1 + e^{s_i - s_j})
        dndcg = (gain.unsqueeze(2) - gain.unsqueeze(1)).abs() * (disc.unsqueeze(2) - disc.unsqueeze(1)).abs()
        dndcg = dndcg / max_dcg.unsqueeze(2)
        lam = rho * dndcg * better
        hes = rho * (1.0 - rho) * dndcg * better
        g[a:a + chunk_queries] = -lam.sum(2) + lam.sum(1)
        h[a:a + chunk_queries] = hes.sum(2) + hes.sum(1)
    return g.view(-1).contiguous(), h.view(-1).contiguous()


def l2_grad(score: torch.Tensor, y: torch.Tensor):
    """Squared error 1/2 (score - y)^2: g = score - y, h = 1."""
    return (score.float() - y).contiguous(), torch.ones_like(y)


def gradients(wl: Workload, score: torch.Tensor):
    if wl.cfg.loss == "logistic":
        return logistic_grad(score, wl.label)
    if wl.cfg.loss == "l2":
        return l2_grad(score, wl.label)
    return lambdarank_grad(score, wl.label, wl.extra["group_size"])


def to_numpy(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()

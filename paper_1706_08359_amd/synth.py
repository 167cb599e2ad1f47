"""Seeded synthetic inputs shaped like the paper's workloads (Table 1).

This module only draws random data: binned feature matrices, labels, the
gradient/hessian of the logistic loss at random scores, and leaf row sets.  It
contains none of the histogram / subtraction / split arithmetic and is the one
piece shared by the GPU tests, the CPU oracle tests and the benchmark, so that
both sides always consume the same arrays.

All generators use torch so that the large workloads can be drawn on the GPU;
pass device="cpu" (default) for the small ones.  Every function is
deterministic for a given (seed, device type).

The paper's datasets (Higgs, epsilon, Microsoft-LTR, Expo, ...) are not
available; these inputs stand in for them by shape, bin count and value
structure only.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import torch


@dataclass
class Workload:
    name: str
    bins: torch.Tensor          # uint8 [n_rows, n_features], values < n_bins
    n_bins: int
    grad: torch.Tensor          # float32 [n_rows]
    hess: torch.Tensor          # float32 [n_rows]
    lam: float = 1.0
    min_child_hess: float = 1e-3
    leaves: List[Optional[torch.Tensor]] = field(default_factory=list)  # int32 row ids, None = root

    @property
    def n_rows(self) -> int:
        return int(self.bins.shape[0])

    @property
    def n_features(self) -> int:
        return int(self.bins.shape[1])


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def quantile_bins(x: torch.Tensor, n_bins: int) -> torch.Tensor:
    """Bin each column of x into n_bins equal-population bins.

    Edges are the column's empirical quantiles j/n_bins (j = 1..n_bins-1), taken
    as order statistics; a value's bin is the number of edges <= it.
    """
    n = x.shape[0]
    srt, _ = torch.sort(x, dim=0)
    pos = torch.tensor([min(n - 1, (j * n) // n_bins) for j in range(1, n_bins)],
                       device=x.device, dtype=torch.long)
    edges = srt[pos, :]                                   # [n_bins-1, F]
    b = torch.searchsorted(edges.t().contiguous(), x.t().contiguous(), right=True)
    return b.t().contiguous().to(torch.uint8)


def uniform_bins(n_rows, n_features, n_bins, gen, device, chunk_rows=1 << 20) -> torch.Tensor:
    """Bins of quantile-binned i.i.d. continuous data: uniform over 0..n_bins-1.

    (Quantile binning maps any continuous distribution to equal-population bins,
    which is the "random bin number" input of the paper's synthetic benchmark,
    App. C.2.)
    """
    out = torch.empty((n_rows, n_features), dtype=torch.uint8, device=device)
    for r0 in range(0, n_rows, chunk_rows):
        r1 = min(n_rows, r0 + chunk_rows)
        out[r0:r1] = torch.randint(0, n_bins, (r1 - r0, n_features), generator=gen,
                                   device=device, dtype=torch.uint8)
    return out


def logistic_grad_hess(n_rows, gen, device, score_std=0.1):
    """grad = sigmoid(s) - y, hess = sigmoid(s)(1 - sigmoid(s)); y~Bernoulli(.5), s~N(0, score_std)."""
    y = (torch.rand(n_rows, generator=gen, device=device) < 0.5).to(torch.float32)
    if score_std == 0.0:
        p = torch.full((n_rows,), 0.5, device=device)
    else:
        s = torch.randn(n_rows, generator=gen, device=device) * score_std
        p = torch.sigmoid(s)
    return (p - y).to(torch.float32), (p * (1.0 - p)).to(torch.float32)


def labels_with_signal(bins, n_bins, gen):
    """Binary labels that depend on the features (a smooth term, two steps and an interaction on
    five columns, through a logistic link), for measurements on whole trees: with labels drawn
    independently of the features every split is chosen among noise and trees degenerate into
    long chains of tiny leaves.  Returns (grad, hess) of the logistic loss at score 0."""
    n, F = bins.shape
    col = lambda j: bins[:, j % F].to(torch.float32) / float(n_bins - 1)
    z = (2.0 * (col(0) - 0.5) + 1.2 * (col(3) > 0.6).float() - 0.9 * (col(7) < 0.25).float()
         + 1.5 * (col(11) - 0.5) * (col(2) - 0.5) + 0.8 * torch.sin(6.0 * col(5)))
    y = (torch.rand(n, generator=gen, device=bins.device) < torch.sigmoid(z)).to(torch.float32)
    p = torch.full((n,), 0.5, device=bins.device)
    return (p - y).to(torch.float32), (p * (1.0 - p)).to(torch.float32)


def leaf_by_truncated_permutation(n_rows, fraction, gen, device) -> torch.Tensor:
    """App. C.2 recipe: random permutation, truncate to fraction*n_rows, sort."""
    k = max(1, int(round(fraction * n_rows)))
    perm = torch.randperm(n_rows, generator=gen, device=device)[:k]
    return torch.sort(perm).values.to(torch.int32)


def random_split_tree_leaves(bins, n_bins, depth, min_fraction, gen) -> List[torch.Tensor]:
    """Row sets of every node of a tree grown by random splits.

    Each node picks a random feature and a random threshold bin in the middle
    40 % of the bin range; rows with bin <= threshold go left.  Row ids stay
    ascending.  Returns the node row sets (root included, as an explicit index
    list) whose size is at least min_fraction of all rows.
    """
    device = bins.device
    n_rows, n_features = bins.shape
    lo = int(math.floor(0.3 * n_bins))
    hi = max(lo + 1, int(math.ceil(0.7 * n_bins)))
    level = [torch.arange(n_rows, device=device, dtype=torch.int64)]
    out = []
    for _ in range(depth + 1):
        nxt = []
        for rows in level:
            if rows.numel() >= max(1, int(min_fraction * n_rows)):
                out.append(rows.to(torch.int32))
            if rows.numel() < 2:
                continue
            f = int(torch.randint(0, n_features, (1,), generator=gen, device=device).item())
            t = int(torch.randint(lo, hi, (1,), generator=gen, device=device).item())
            go_left = bins[rows, f] <= t
            nxt.append(rows[go_left])
            nxt.append(rows[~go_left])
        level = nxt
    return out


# --------------------------------------------------------------------------- configs


def config1_tiny_dense(seed=0, n_rows=10_000, n_features=28, n_bins=64, device="cpu") -> Workload:
    """Tiny dense: N(0,1) features in 64 quantile bins; grad = sigmoid(0) - y, hess = 0.25."""
    gen = _gen(seed, device)
    x = torch.randn((n_rows, n_features), generator=gen, device=device, dtype=torch.float64)
    bins = quantile_bins(x, n_bins)
    grad, hess = logistic_grad_hess(n_rows, gen, device, score_std=0.0)
    return Workload("tiny_dense", bins, n_bins, grad, hess, lam=1.0, leaves=[None])


def config2_dense_wide(seed=1, n_rows=400_000, n_features=2000, n_bins=63, device="cpu",
                       exact_binning=False, tree_depth=8, min_fraction=0.01,
                       with_leaves=True) -> Workload:
    """Dense wide (epsilon-shaped): 63 quantile bins of N(0,1) values, logistic grad/hess."""
    gen = _gen(seed, device)
    if exact_binning:
        x = torch.randn((n_rows, n_features), generator=gen, device=device)
        bins = quantile_bins(x, n_bins)
    else:
        bins = uniform_bins(n_rows, n_features, n_bins, gen, device)
    grad, hess = logistic_grad_hess(n_rows, gen, device, score_std=0.1)
    leaves: List[Optional[torch.Tensor]] = [None]
    if with_leaves:
        leaves += random_split_tree_leaves(bins, n_bins, tree_depth, min_fraction, gen)[1:]
    return Workload("dense_wide", bins, n_bins, grad, hess, leaves=leaves)


def config3_dense_tall(seed=2, n_rows=10_500_000, n_features=28, n_bins=255, device="cpu",
                       exact_binning=False) -> Workload:
    """Dense tall (Higgs-shaped): even columns N(0,1), odd columns Exp(1), 255 quantile bins."""
    gen = _gen(seed, device)
    if exact_binning:
        x = torch.randn((n_rows, n_features), generator=gen, device=device)
        e = -torch.log1p(-torch.rand((n_rows, n_features), generator=gen, device=device))
        odd = (torch.arange(n_features, device=device) % 2 == 1)
        x = torch.where(odd[None, :], e, x)
        bins = quantile_bins(x, n_bins)
    else:
        bins = uniform_bins(n_rows, n_features, n_bins, gen, device)
    grad, hess = logistic_grad_hess(n_rows, gen, device, score_std=0.1)
    return Workload("dense_tall", bins, n_bins, grad, hess, leaves=[None])


def config4_ranking_sparse(seed=3, n_rows=2_270_000, n_features=137, n_bins=255, device="cpu",
                           zero_prob=0.6, fractions=(1.0, 0.5, 0.25, 0.10, 0.05),
                           chunk_rows=1 << 20) -> Workload:
    """Ranking-shaped (Microsoft-LTR-shaped): 60 % zeros in bin 0, nonzeros (LogNormal,
    quantile binned, hence uniform) in bins 1..n_bins-1; grad~N(0,1), hess~U(0.01,1)."""
    gen = _gen(seed, device)
    bins = torch.empty((n_rows, n_features), dtype=torch.uint8, device=device)
    for r0 in range(0, n_rows, chunk_rows):
        r1 = min(n_rows, r0 + chunk_rows)
        nz = torch.randint(1, n_bins, (r1 - r0, n_features), generator=gen, device=device,
                           dtype=torch.uint8)
        z = torch.rand((r1 - r0, n_features), generator=gen, device=device) < zero_prob
        bins[r0:r1] = torch.where(z, torch.zeros_like(nz), nz)
    grad = torch.randn(n_rows, generator=gen, device=device, dtype=torch.float32)
    hess = (torch.rand(n_rows, generator=gen, device=device) * 0.99 + 0.01).to(torch.float32)
    leaves: List[Optional[torch.Tensor]] = []
    for p in fractions:
        leaves.append(None if p >= 1.0 else leaf_by_truncated_permutation(n_rows, p, gen, device))
    return Workload("ranking_sparse", bins, n_bins, grad, hess, leaves=leaves)


def config5_categorical(seed=4, n_rows=11_000_000, n_features=700, n_bins=16, device="cpu",
                        zipf_s=1.2, chunk_rows=1 << 19) -> Workload:
    """Categorical-heavy (Expo-shaped): each feature has 2..16 levels with Zipf(1.2) frequencies."""
    gen = _gen(seed, device)
    levels = torch.randint(2, 17, (n_features,), generator=gen, device=device)
    j = torch.arange(16, device=device, dtype=torch.float64)
    w = (j + 1.0) ** (-zipf_s)
    w = w[None, :] * (j[None, :] < levels[:, None])            # [F, 16]
    cdf = torch.cumsum(w / w.sum(dim=1, keepdim=True), dim=1).to(torch.float32)
    cdf[:, -1] = 2.0                                            # guard the last edge
    bins = torch.empty((n_rows, n_features), dtype=torch.uint8, device=device)
    for r0 in range(0, n_rows, chunk_rows):
        r1 = min(n_rows, r0 + chunk_rows)
        u = torch.rand((r1 - r0, n_features), generator=gen, device=device)
        # level = number of cdf edges <= u (inverse-cdf draw), per feature
        b = torch.searchsorted(cdf, u.t().contiguous(), right=True).t()
        b = torch.minimum(b, (levels - 1)[None, :])
        bins[r0:r1] = b.to(torch.uint8)
    grad, hess = logistic_grad_hess(n_rows, gen, device, score_std=0.1)
    return Workload("categorical", bins, n_bins, grad, hess, leaves=[None])

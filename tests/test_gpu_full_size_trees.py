"""255-leaf trees (the tree size of the paper's experiments, Sec. 5) grown by gbdt_grow_tree on
the FULL dense_tall (10,500,000 x 28, 255 bins) and categorical (11,000,000 x 700, 16 bins,
4-bit) matrices -- smaller child built, sibling by subtraction -- and replayed with the CPU
oracle.

dense_tall: every node is replayed in full (test_gpu_tree._replay: the oracle rebuilds the
histogram of every node from the node's own rows and must make the same choice, or one inside
the near-tie band; children's rows, counts and sums from the oracle's partition).
categorical: the first 31 splits are replayed in full the same way; after that the integer
facts stay complete (every child's rows, counts, sums, the routing of every row) while the
choice of (feature, bin) is checked on the chosen feature plus a seeded sample of others
(the oracle's gain at the device's choice must not be beaten by any sampled candidate by more
than the band).  Oracle wall times are printed.
"""
import time

import numpy as np
import pytest
import torch

from oracle import gbdt_oracle as orc
from paper_1706_08359_amd import binding as B
from paper_1706_08359_amd import synth

from gpu_util import REL_TOL
from test_gpu_tree import BAND, _check_structure, _replay

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def test_config3_dense_tall_255_leaf_tree_full_size():
    w = synth.config3_dense_tall(device=DEV)
    n, F, nb = w.n_rows, w.n_features, w.n_bins
    _say(f"grow_tree {n}x{F} bins={nb} leaves=255 (full dense_tall)")
    packed = B.gbdt_bins_pack(w.bins, nb)
    nodes, order, _ = B.gbdt_grow_tree(packed, n, F, nb, w.grad, w.hess, 255, w.lam, w.min_child_hess)
    torch.cuda.synchronize()
    bins, grad, hess = w.bins.cpu().numpy(), w.grad.cpu().numpy(), w.hess.cpu().numpy()
    n_leaves = int((nodes["left"] < 0).sum())
    assert n_leaves == 255 and len(nodes) == 509
    t0 = time.perf_counter()
    _check_structure(nodes, order.cpu().numpy(), bins)
    t1 = time.perf_counter()
    _, _, near = _replay(nodes, bins, nb, grad, hess, w.lam, w.min_child_hess)
    _say(f"  255 leaves, deepest node at depth {_max_depth(nodes)}, {near} near-tie decisions; "
         f"routing check {t1 - t0:.1f} s, oracle replay of all 509 nodes {time.perf_counter() - t1:.1f} s")


def _max_depth(nodes):
    depth = np.zeros(len(nodes), np.int32)
    for k, nd in enumerate(nodes):
        if nd["parent"] >= 0:
            depth[k] = depth[nd["parent"]] + 1
    return int(depth.max())


def _replay_partly_sampled(nodes, bins, n_bins, grad, hess, lam, mch, full_splits, n_sample, seed):
    """As test_gpu_tree._replay for the first `full_splits` splits (and every node open during
    them); afterwards integer facts in full, the choice of split on sampled features."""
    g64, h64 = grad.astype(np.float64), hess.astype(np.float64)
    F = bins.shape[1]
    rng = np.random.default_rng(seed)
    rows = {0: np.arange(bins.shape[0], dtype=np.int32)}
    budget = {0: (np.abs(g64).sum(), np.abs(h64).sum())}
    best = {}

    def oracle_best(k):
        if k not in best:
            best[k] = orc.best_split(orc.hist_build(bins, n_bins, grad, hess, rows[k]), lam, mch, return_gains=True)
        return best[k]

    open_leaves = [0]
    order = sorted((int(nd["left"]), k) for k, nd in enumerate(nodes) if nd["left"] >= 0)
    near = 0
    t_full = 0.0
    for s_i, (_, k) in enumerate(order):
        nd = nodes[k]
        f_dev, b_dev = int(nd["feature"]), int(nd["bin"])
        if s_i < full_splits:
            t0 = time.perf_counter()
            s_ref, gains = oracle_best(k)
            assert s_ref["feature"] >= 0, f"node {k}: the oracle finds no admissible split"
            scale = max(1.0, abs(s_ref["gain"]))
            g_at = gains[f_dev, b_dev]
            assert np.isfinite(g_at), f"node {k}: inadmissible threshold chosen"
            if (f_dev, b_dev) != (s_ref["feature"], s_ref["bin"]):
                assert s_ref["gain"] - g_at <= BAND * scale, (k, nd, s_ref, g_at)
                near += 1
            assert abs(nd["gain"] - g_at) <= BAND * scale
            top = max(oracle_best(j)[0]["gain"] for j in open_leaves if oracle_best(j)[0]["feature"] >= 0)
            assert top - s_ref["gain"] <= BAND * max(1.0, abs(top)), f"node {k} was not the best open leaf"
            t_full += time.perf_counter() - t0
        else:
            # the chosen feature and a sample of others, on the node's own rows
            others = rng.choice(F, size=min(n_sample, F), replace=False)
            feats = np.unique(np.concatenate([[f_dev], others]))
            sub = np.ascontiguousarray(bins[np.ix_(rows[k], feats)])
            _, gains = orc.best_split(orc.hist_build(sub, n_bins, grad[rows[k]], hess[rows[k]]), lam, mch,
                                      return_gains=True)
            at = int(np.searchsorted(feats, f_dev))
            g_at = gains[at, b_dev]
            assert np.isfinite(g_at), f"node {k}: inadmissible threshold chosen"
            top = np.nanmax(np.where(np.isfinite(gains), gains, -np.inf))
            scale = max(1.0, abs(top))
            assert top - g_at <= BAND * scale, (k, nd, top, g_at)
            if top > g_at:
                near += 1
            assert abs(nd["gain"] - g_at) <= BAND * scale
            # best-first among the open leaves, by the gains the device recorded for them
            rec_top = max(float(nodes[j]["gain"]) for j in open_leaves if nodes[j]["feature"] >= 0)
            assert rec_top - float(nd["gain"]) <= BAND * max(1.0, abs(rec_top)), f"node {k} was not the best open leaf"
        # the children: the oracle's partition of the node's rows by the device's split
        left, right = orc.partition_rows(bins, f_dev, b_dev, rows[k])
        small_is_left = left.size <= right.size
        small = left if small_is_left else right
        b_small = (np.abs(g64[small]).sum(), np.abs(h64[small]).sum())
        b_large = (budget[k][0] + b_small[0], budget[k][1] + b_small[1])
        for side, kid, r in (("left", int(nd["left"]), left), ("right", int(nd["right"]), right)):
            c = nodes[kid]
            assert c["count"] == r.size, (k, side)
            assert abs(c["sum_grad"] - g64[r].sum()) <= REL_TOL * budget[k][0] + 1e-6 * abs(g64[r].sum())
            assert abs(c["sum_hess"] - h64[r].sum()) <= REL_TOL * budget[k][1] + 1e-6 * abs(h64[r].sum())
            rows[kid] = r
            budget[kid] = b_small if (side == "left") == small_is_left else b_large
        del rows[k]
        open_leaves.remove(k)
        open_leaves += [int(nd["left"]), int(nd["right"])]
    return near, t_full


def test_config5_categorical_255_leaf_tree_full_size():
    w = synth.config5_categorical(device=DEV)
    n, F, nb = w.n_rows, w.n_features, w.n_bins
    _say(f"grow_tree {n}x{F} bins={nb} leaves=255 (full categorical)")
    packed = B.gbdt_bins_pack(w.bins, nb)
    nodes, order, _ = B.gbdt_grow_tree(packed, n, F, nb, w.grad, w.hess, 255, w.lam, w.min_child_hess)
    torch.cuda.synchronize()
    order = order.cpu().numpy()
    del packed
    bins, grad, hess = w.bins.cpu().numpy(), w.grad.cpu().numpy(), w.hess.cpu().numpy()
    n_leaves = int((nodes["left"] < 0).sum())
    assert n_leaves == 255 and len(nodes) == 509
    t0 = time.perf_counter()
    _check_structure(nodes, order, bins)
    t1 = time.perf_counter()
    near, t_full = _replay_partly_sampled(nodes, bins, nb, grad, hess, w.lam, w.min_child_hess,
                                          full_splits=31, n_sample=24, seed=55)
    _say(f"  255 leaves, deepest node at depth {_max_depth(nodes)}, {near} near-tie decisions; routing check "
         f"{t1 - t0:.1f} s, replay {time.perf_counter() - t1:.1f} s of which {t_full:.1f} s for the oracle's full "
         f"histograms of the first 31 splits")


@pytest.mark.parametrize("name", ["dense_tall", "dense_wide"])
def test_255_leaf_tree_on_labels_with_signal_full_size(name):
    """The same matrices with labels that depend on the features: balanced trees, so a round of
    the grower really splits many leaves (32 partitions, one batched build, one split search over
    64 children per round) instead of peeling one small leaf off a chain.  Every node replayed in
    full with the oracle."""
    w = synth.config3_dense_tall(device=DEV) if name == "dense_tall" else \
        synth.config2_dense_wide(device=DEV, with_leaves=False)
    n, F, nb = w.n_rows, w.n_features, w.n_bins
    gen = torch.Generator(device=DEV)
    gen.manual_seed(31)
    w.grad, w.hess = synth.labels_with_signal(w.bins, nb, gen)
    _say(f"grow_tree {n}x{F} bins={nb} leaves=255 (full {name}, labels with signal)")
    packed = B.gbdt_bins_pack(w.bins, nb)
    nodes, order, _ = B.gbdt_grow_tree(packed, n, F, nb, w.grad, w.hess, 255, w.lam, w.min_child_hess)
    torch.cuda.synchronize()
    order = order.cpu().numpy()
    del packed
    bins, grad, hess = w.bins.cpu().numpy(), w.grad.cpu().numpy(), w.hess.cpu().numpy()
    n_leaves = int((nodes["left"] < 0).sum())
    assert n_leaves == 255 and len(nodes) == 509
    assert _max_depth(nodes) <= 16, "labels with signal should give a balanced tree"
    t0 = time.perf_counter()
    _check_structure(nodes, order, bins)
    t1 = time.perf_counter()
    _, _, near = _replay(nodes, bins, nb, grad, hess, w.lam, w.min_child_hess)
    _say(f"  255 leaves, deepest node at depth {_max_depth(nodes)}, {near} near-tie decisions; "
         f"routing check {t1 - t0:.1f} s, oracle replay of all 509 nodes {time.perf_counter() - t1:.1f} s")

"""CPU-only pins of the oracle: each test fixes the oracle to something other
than itself -- a library routine, a closed form, an invariant, brute force from
raw rows, a textbook special case, or a hand-worked fixture -- so that a dropped
term, a wrong sign or index, or a transposed operand fails at least one."""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import gbdt_oracle as orc
from oracle.brute_force import brute_force_best_split, gain_table_from_rows
from paper_1706_08359_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(rng, n_rows, n_features, n_bins, skew=False):
    if skew:
        p = rng.dirichlet(np.full(n_bins, 0.3))
        bins = rng.choice(n_bins, size=(n_rows, n_features), p=p).astype(np.uint8)
    else:
        bins = rng.integers(0, n_bins, size=(n_rows, n_features), dtype=np.uint8)
    grad = rng.normal(size=n_rows).astype(np.float32)
    hess = rng.uniform(0.01, 1.0, size=n_rows).astype(np.float32)
    return bins, grad, hess


# ----------------------------------------------------------------- histogram build


@pytest.mark.parametrize("seed", range(6))
def test_hist_equals_numpy_bincount(seed):
    """Alg. 1 per feature is a weighted bincount (library special case)."""
    rng = np.random.default_rng(seed)
    n_rows, n_features = int(rng.integers(1, 400)), int(rng.integers(1, 9))
    n_bins = int(rng.choice([2, 3, 16, 17, 63, 64, 255, 256]))
    bins, grad, hess = _rand_problem(rng, n_rows, n_features, n_bins, skew=seed % 2 == 1)
    variants = [None,
                np.sort(rng.choice(n_rows, size=max(1, n_rows // 3), replace=False)).astype(np.int32),
                rng.integers(0, n_rows, size=2 * n_rows).astype(np.int32)]  # unsorted, with repeats
    for idx in variants:
        h = orc.hist_build(bins, n_bins, grad, hess, idx)
        rows = np.arange(n_rows) if idx is None else idx
        for f in range(n_features):
            col = bins[rows, f]
            np.testing.assert_array_equal(h["count"][f], np.bincount(col, minlength=n_bins))
            np.testing.assert_allclose(
                h["grad"][f], np.bincount(col, weights=grad[rows].astype(np.float64), minlength=n_bins),
                rtol=0, atol=1e-12 * max(1.0, np.abs(grad[rows]).sum()))
            np.testing.assert_allclose(
                h["hess"][f], np.bincount(col, weights=hess[rows].astype(np.float64), minlength=n_bins),
                rtol=0, atol=1e-12 * max(1.0, np.abs(hess[rows]).sum()))


def test_hist_sum_invariant():
    """Every leaf sample lands in exactly one bin of every feature (Alg. 1 loop body)."""
    rng = np.random.default_rng(10)
    bins, grad, hess = _rand_problem(rng, 5000, 13, 37, skew=True)
    idx = np.sort(rng.choice(5000, size=1234, replace=False)).astype(np.int32)
    h = orc.hist_build(bins, 37, grad, hess, idx)
    G, H = grad[idx].astype(np.float64).sum(), hess[idx].astype(np.float64).sum()
    assert (h["count"].sum(axis=1) == idx.size).all()
    np.testing.assert_allclose(h["grad"].sum(axis=1), G, rtol=0, atol=1e-12 * np.abs(grad[idx]).sum())
    np.testing.assert_allclose(h["hess"].sum(axis=1), H, rtol=0, atol=1e-12 * np.abs(hess[idx]).sum())


def test_hist_uses_row_id_not_leaf_position_for_stats():
    """g and h are indexed by row id (g_{d_ri} in Alg. 1), and the feature index
    selects a column (not a row) of the bin matrix."""
    bins = np.array([[0, 1], [1, 0], [1, 1], [0, 0]], dtype=np.uint8)
    grad = np.array([1.0, 10.0, 100.0, 1000.0], dtype=np.float32)
    hess = np.array([2.0, 20.0, 200.0, 2000.0], dtype=np.float32)
    idx = np.array([2, 3], dtype=np.int32)
    h = orc.hist_build(bins, 2, grad, hess, idx)
    np.testing.assert_array_equal(h["grad"], [[1000.0, 100.0], [1000.0, 100.0]])
    np.testing.assert_array_equal(h["hess"], [[2000.0, 200.0], [2000.0, 200.0]])
    np.testing.assert_array_equal(h["count"], [[1, 1], [1, 1]])
    h = orc.hist_build(bins, 2, grad, hess, np.array([0, 1], dtype=np.int32))
    np.testing.assert_array_equal(h["grad"], [[1.0, 10.0], [10.0, 1.0]])


def test_hist_empty_leaf_and_errors():
    bins = np.zeros((4, 3), dtype=np.uint8)
    g = np.ones(4, dtype=np.float32)
    h = orc.hist_build(bins, 5, g, g, np.zeros(0, dtype=np.int32))
    assert h.shape == (3, 5) and not h["count"].any() and not h["grad"].any()
    with pytest.raises(ValueError):
        orc.hist_build(bins, 5, g, g, np.array([4], dtype=np.int32))      # row id out of range
    bins[1, 1] = 7
    with pytest.raises(ValueError):
        orc.hist_build(bins, 5, g, g)                                      # bin value out of range


def test_hand_worked_example():
    d = json.load(open(os.path.join(GOLDEN, "alg1_hand_example.json")))
    bins = np.array(d["bins"], dtype=np.uint8)
    grad = np.array(d["grad"], dtype=np.float32)
    hess = np.array(d["hess"], dtype=np.float32)
    idx = np.array(d["leaf_row_idx"], dtype=np.int32)
    h = orc.hist_build(bins, d["n_bins"], grad, hess, idx)
    np.testing.assert_array_equal(h["grad"], np.array(d["hist"]["grad"]))
    np.testing.assert_array_equal(h["hess"], np.array(d["hist"]["hess"]))
    np.testing.assert_array_equal(h["count"], np.array(d["hist"]["count"]))
    s, gains = orc.best_split(h, d["lambda"], d["min_child_hess"], return_gains=True)
    terms = d["gain_terms"]
    parent = Fraction(*terms["parent"][0]) / Fraction(*terms["parent"][1])
    for key, v in terms.items():
        if key == "parent":
            continue
        f, t = int(key[1]), int(key[4])
        want = (Fraction(*v["left"][0]) / Fraction(*v["left"][1])
                + Fraction(*v["right"][0]) / Fraction(*v["right"][1]) - parent)
        assert abs(gains[f, t] - float(want)) < 1e-14
    assert np.isnan(gains[:, -1]).all()
    for k, v in d["best"].items():
        assert s[k] == v
    assert abs(s["gain"] - float(Fraction(4, 7) + Fraction(289, 36) - Fraction(81, 132))) < 1e-14


def test_config1_closed_form():
    """Tiny dense config: hess == 0.25 and grad == +-0.5 make every bin a closed form,
    and tie-free quantile binning of 10,000 rows into 64 bins gives 156 or 157 per bin."""
    w = synth.config1_tiny_dense()
    bins, grad, hess = w.bins.numpy(), w.grad.numpy(), w.hess.numpy()
    assert bins.shape == (10_000, 28) and bins.max() == 63
    assert set(np.unique(grad)) == {-0.5, 0.5} and (hess == 0.25).all()
    h = orc.hist_build(bins, 64, grad, hess)
    assert set(np.unique(h["count"])) <= {156, 157}
    assert (h["count"].sum(axis=1) == 10_000).all()
    np.testing.assert_array_equal(h["hess"], 0.25 * h["count"])
    for f in range(28):
        positives = np.bincount(bins[:, f], weights=(grad < 0), minlength=64)   # y = 1 <=> grad = -0.5
        np.testing.assert_array_equal(h["grad"][f], 0.5 * (h["count"][f] - 2.0 * positives))


# -------------------------------------------------------------------- subtraction


def test_parent_equals_left_plus_right_and_subtract():
    rng = np.random.default_rng(3)
    bins, grad, hess = _rand_problem(rng, 3000, 7, 64)
    parent_rows = np.sort(rng.choice(3000, size=2000, replace=False)).astype(np.int32)
    go_left = bins[parent_rows, 4] <= 20
    left_rows, right_rows = parent_rows[go_left], parent_rows[~go_left]
    hp = orc.hist_build(bins, 64, grad, hess, parent_rows)
    hl = orc.hist_build(bins, 64, grad, hess, left_rows)
    hr = orc.hist_build(bins, 64, grad, hess, right_rows)
    np.testing.assert_array_equal(hl["count"] + hr["count"], hp["count"])
    tol_g = 1e-12 * np.abs(grad[parent_rows]).sum()
    np.testing.assert_allclose(hl["grad"] + hr["grad"], hp["grad"], rtol=0, atol=tol_g)
    np.testing.assert_allclose(hl["hess"] + hr["hess"], hp["hess"], rtol=0, atol=tol_g)
    sib = orc.hist_subtract(hp, hl)
    np.testing.assert_array_equal(sib["count"], hr["count"])
    np.testing.assert_allclose(sib["grad"], hr["grad"], rtol=0, atol=tol_g)
    np.testing.assert_allclose(sib["hess"], hr["hess"], rtol=0, atol=tol_g)
    # operand order: parent - child, not child - parent
    assert (sib["hess"] >= -tol_g).all()
    with pytest.raises(ValueError):
        orc.hist_subtract(hl, hp)


# --------------------------------------------------------------------- best split


@pytest.mark.parametrize("seed", range(25))
def test_best_split_equals_brute_force_from_raw_rows(seed):
    rng = np.random.default_rng(100 + seed)
    n_rows = int(rng.integers(1, 200))
    n_features = int(rng.integers(1, 6))
    n_bins = int(rng.integers(2, 9))
    bins, grad, hess = _rand_problem(rng, n_rows, n_features, n_bins, skew=seed % 3 == 0)
    if seed % 5 == 0:
        bins[:, 0] = bins[0, 0]                      # a feature with every row in one bin
    n_leaf = int(rng.integers(1, n_rows + 1))
    rows = np.sort(rng.choice(n_rows, size=n_leaf, replace=False)).astype(np.int32)
    lam = float(rng.choice([0.0, 0.5, 1.0, 10.0]))
    mch = float(rng.choice([0.0, 1e-3, 0.5, 3.0]))
    h = orc.hist_build(bins, n_bins, grad, hess, rows)
    s, gains = orc.best_split(h, lam, mch, return_gains=True)
    bf = gain_table_from_rows(bins, n_bins, grad, hess, rows, lam, mch)
    # same admissible set, same gains
    np.testing.assert_array_equal(np.isnan(gains), np.isnan(bf))
    ok = ~np.isnan(bf)
    np.testing.assert_allclose(gains[ok], bf[ok], rtol=0,
                               atol=1e-9 * max(1.0, np.abs(bf[ok]).max() if ok.any() else 1.0))
    f, t, gain = brute_force_best_split(bins, n_bins, grad, hess, rows, lam, mch)
    if f < 0:
        assert s["feature"] == -1 and s["bin"] == -1 and s["gain"] == 0.0
        return
    # the chosen split is the brute-force one, unless fp noise makes two partitions tie
    top = np.nanmax(bf)
    near = np.argwhere(ok & (bf >= top - 1e-9 * max(1.0, abs(top))))
    assert [s["feature"], s["bin"]] in near.tolist()
    if len(near) == 1:
        assert (s["feature"], s["bin"]) == (f, t)
    assert abs(s["gain"] - gain) <= 1e-9 * max(1.0, abs(gain))
    left = bins[rows, s["feature"]] <= s["bin"]
    assert s["left_count"] == left.sum() and s["right_count"] == (~left).sum()
    assert abs(s["left_grad"] - grad[rows][left].astype(np.float64).sum()) < 1e-9
    assert abs(s["right_hess"] - hess[rows][~left].astype(np.float64).sum()) < 1e-9


def test_best_split_no_admissible_threshold():
    bins = np.full((10, 2), 3, dtype=np.uint8)
    g = np.ones(10, dtype=np.float32)
    h = orc.hist_build(bins, 8, g, g)
    s = orc.best_split(h, 1.0, 1e-3)
    assert (s["feature"], s["bin"], s["gain"]) == (-1, -1, 0.0)
    # single-row leaf
    s = orc.best_split(orc.hist_build(bins, 8, g, g, np.array([5], dtype=np.int32)), 1.0, 0.0)
    assert s["feature"] == -1
    # min_child_hess larger than anything reachable
    rng = np.random.default_rng(0)
    bins, grad, hess = _rand_problem(rng, 50, 3, 4)
    s = orc.best_split(orc.hist_build(bins, 4, grad, hess), 0.0, 1e6)
    assert s["feature"] == -1


def test_best_split_tie_break_smallest_feature_then_bin():
    # two identical features -> feature 0 wins; an empty bin right of the best
    # threshold repeats the same partition -> the smaller bin wins.
    col = np.array([0, 0, 0, 2, 2, 2, 3, 3], dtype=np.uint8)      # bin 1 is empty
    bins = np.stack([col, col], axis=1)
    grad = np.array([1, 1, 1, -1, -1, -1, -1, -1], dtype=np.float32)
    hess = np.ones(8, dtype=np.float32)
    s, gains = orc.best_split(orc.hist_build(bins, 4, grad, hess), 1.0, 0.0, return_gains=True)
    assert gains[0, 0] == gains[0, 1] == gains[1, 0] == gains[1, 1]
    assert (s["feature"], s["bin"]) == (0, 0)


@pytest.mark.parametrize("seed", range(5))
def test_best_split_square_loss_special_case_is_eq4(seed):
    """g = -y, h = 1, lambda = 0: maximising the gain is minimising Eq. (4),
    L(t) = sum y^2 - (sum_{V_r} y)^2/N_r - (sum_{V_l} y)^2/N_l  (Sec. 3.1)."""
    rng = np.random.default_rng(200 + seed)
    n, F, B = 300, 4, 12
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    y = rng.normal(size=n) + 2.0 * (bins[:, 2] > 6)
    grad = (-y).astype(np.float32)
    hess = np.ones(n, dtype=np.float32)
    y = -grad.astype(np.float64)
    s = orc.best_split(orc.hist_build(bins, B, grad, hess), 0.0, 0.0)
    best = None
    for f in range(F):
        for t in range(B - 1):
            l = bins[:, f] <= t
            if l.sum() == 0 or (~l).sum() == 0:
                continue
            L = (y ** 2).sum() - y[~l].sum() ** 2 / (~l).sum() - y[l].sum() ** 2 / l.sum()
            if best is None or L < best[0]:
                best = (L, f, t)
    assert (s["feature"], s["bin"]) == (best[1], best[2])
    # and the gain is exactly the drop of Eq. (4) from the unsplit leaf
    L0 = (y ** 2).sum() - y.sum() ** 2 / n
    assert abs(s["gain"] - (L0 - best[0])) < 1e-8 * L0


def test_best_split_planted():
    rng = np.random.default_rng(7)
    n, F, B = 4000, 10, 32
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    y = (bins[:, 6] > 19).astype(np.float64) + 0.05 * rng.normal(size=n)
    p = 0.5
    grad = (p - y).astype(np.float32)
    hess = np.full(n, 0.25, dtype=np.float32)
    s = orc.best_split(orc.hist_build(bins, B, grad, hess), 1.0, 1e-3)
    assert (s["feature"], s["bin"]) == (6, 19)
    assert s["left_count"] == (bins[:, 6] <= 19).sum()


def test_from_f32_hist_is_exact():
    g = np.array([[1.5, -2.25]], dtype=np.float32)
    c = np.array([[3, 4]], dtype=np.uint32)
    h = orc.from_f32_hist(g, g, c)
    assert h["grad"][0, 1] == -2.25 and h["count"][0, 1] == 4 and h.dtype == orc.BIN_DTYPE


# ------------------------------------------------------------ row partition (App. C.1, Split())

@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_partition_equals_per_row_loop(seed):
    """Pin: a pure-Python walk over the raw matrix, no numpy masking, no C."""
    rng = np.random.default_rng(900 + seed)
    n, F, B = 157, 6, 11
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    rows = np.sort(rng.choice(n, size=int(rng.integers(1, n)), replace=False)).astype(np.int32)
    if seed == 3:
        rows = rng.permutation(rows).astype(np.int32)     # order must be kept, sorted or not
    f, t = int(rng.integers(0, F)), int(rng.integers(0, B - 1))
    left, right = orc.partition_rows(bins, f, t, rows)
    want_l = [int(r) for r in rows if int(bins[int(r)][f]) <= t]
    want_r = [int(r) for r in rows if int(bins[int(r)][f]) > t]
    assert left.tolist() == want_l and right.tolist() == want_r


def test_partition_is_an_ordered_disjoint_cover():
    rng = np.random.default_rng(77)
    n, F, B = 5000, 9, 64
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    rows = np.sort(rng.choice(n, size=3211, replace=False)).astype(np.int32)
    left, right = orc.partition_rows(bins, 4, 20, rows)
    assert left.size + right.size == rows.size
    assert np.array_equal(np.sort(np.concatenate([left, right])), rows)
    assert np.all(np.diff(left) > 0) and np.all(np.diff(right) > 0)
    assert np.all(bins[left, 4] <= 20) and np.all(bins[right, 4] > 20)
    # the feature is the one asked for, not a neighbour, and the comparison is <=, not <
    assert not np.array_equal(left, rows[bins[rows, 3] <= 20])
    assert not np.array_equal(left, rows[bins[rows, 4] < 20])


def test_partition_root_and_degenerate_thresholds():
    rng = np.random.default_rng(5)
    bins = rng.integers(0, 16, size=(300, 3), dtype=np.uint8)
    left, right = orc.partition_rows(bins, 1, 7)                       # NULL index list = all rows
    assert np.array_equal(left, np.nonzero(bins[:, 1] <= 7)[0])
    assert np.array_equal(right, np.nonzero(bins[:, 1] > 7)[0])
    left, right = orc.partition_rows(bins, 1, 7, None, n_leaf_rows=100)  # ... or a prefix of them
    assert np.array_equal(left, np.nonzero(bins[:100, 1] <= 7)[0])
    left, right = orc.partition_rows(bins, 0, 255)
    assert left.size == 300 and right.size == 0
    left, right = orc.partition_rows(bins, 0, -1)
    assert left.size == 0 and right.size == 300
    left, right = orc.partition_rows(bins, 2, 3, np.zeros(0, np.int32))
    assert left.size == 0 and right.size == 0
    with pytest.raises(ValueError):
        orc.partition_rows(bins, 3, 1)                                  # no such feature
    with pytest.raises(ValueError):
        orc.partition_rows(bins, 0, 1, np.array([300], np.int32))       # no such row


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_partition_sizes_and_sums_match_the_split_record(seed):
    """Two routes to the children: the split search derives their counts and sums from the
    parent's histogram; the partition walks the rows.  They must describe the same children,
    and the children's own histograms must add up to the parent's."""
    rng = np.random.default_rng(40 + seed)
    n, F, B = 2000, 7, 32
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.1, 1.0, size=n).astype(np.float32)
    rows = np.sort(rng.choice(n, size=1500, replace=False)).astype(np.int32)
    parent = orc.hist_build(bins, B, grad, hess, rows)
    s = orc.best_split(parent, 1.0, 1e-3)
    assert s["feature"] >= 0
    left, right = orc.partition_rows(bins, s["feature"], s["bin"], rows)
    assert left.size == s["left_count"] and right.size == s["right_count"]
    assert np.isclose(grad[left].astype(np.float64).sum(), s["left_grad"], rtol=0, atol=1e-9)
    assert np.isclose(hess[right].astype(np.float64).sum(), s["right_hess"], rtol=0, atol=1e-9)
    hl = orc.hist_build(bins, B, grad, hess, left)
    hr = orc.hist_build(bins, B, grad, hess, right)
    assert np.array_equal(hl["count"] + hr["count"], parent["count"])
    assert np.allclose(hl["grad"] + hr["grad"], parent["grad"], rtol=0, atol=1e-9)


# ------------------------------------------------------------ leaf-wise tree growth (Sec. 3.1, Sec. 5)

from oracle import tree_oracle  # noqa: E402


def _tree_problem(seed, n=400, F=4, B=8):
    rng = np.random.default_rng(seed)
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.2, 1.0, size=n).astype(np.float32)
    return bins, grad, hess, B


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_tree_every_step_is_the_greedy_choice_by_brute_force(seed):
    """Replays the growth: at every step the node that was split must be the open leaf whose
    best split -- found by exhaustive search over raw rows, no histogram -- has the largest
    gain, and its (feature, bin) must be that exhaustive search's answer."""
    bins, grad, hess, B = _tree_problem(seed)
    lam, mch = 0.5, 1e-3
    nodes = tree_oracle.grow_tree(bins, B, grad, hess, 9, lam, mch)
    assert sum(1 for nd in nodes if nd["left"] < 0) == 9 and len(nodes) == 17
    bf = {}

    def brute(k):
        if k not in bf:
            bf[k] = brute_force_best_split(bins, B, grad, hess, nodes[k]["rows"], lam, mch)
        return bf[k]

    open_leaves = [0]
    # splits were made in the creation order of their children
    order = sorted((nd["left"], k) for k, nd in enumerate(nodes) if nd["left"] >= 0)
    for _, k in order:
        gains = {j: brute(j)[2] for j in open_leaves if brute(j)[0] >= 0}
        assert k in gains
        assert gains[k] >= max(gains.values()) - 1e-9 * max(1.0, abs(gains[k]))
        f, t, _ = brute(k)
        assert (nodes[k]["split"]["feature"], nodes[k]["split"]["bin"]) == (f, t)
        open_leaves.remove(k)
        open_leaves += [nodes[k]["left"], nodes[k]["right"]]


def test_tree_rows_are_where_the_splits_route_them():
    bins, grad, hess, B = _tree_problem(7, n=3000, F=6, B=16)
    nodes = tree_oracle.grow_tree(bins, B, grad, hess, 31, 1.0, 1e-3)
    at = tree_oracle.route_rows(bins, nodes)
    leaves = [k for k, nd in enumerate(nodes) if nd["left"] < 0]
    assert len(leaves) == 31
    total = 0
    for k in leaves:
        assert np.array_equal(np.nonzero(at == k)[0], nodes[k]["rows"])      # ascending, complete
        total += nodes[k]["count"]
    assert total == 3000
    for nd in nodes:
        if nd["left"] >= 0:
            l, r = nodes[nd["left"]], nodes[nd["right"]]
            assert l["parent"] == r["parent"] == nodes.index(nd)
            assert l["count"] == nd["split"]["left_count"] and r["count"] == nd["split"]["right_count"]
            assert np.isclose(l["sum_grad"], nd["split"]["left_grad"], rtol=0, atol=1e-9)
            assert np.isclose(r["sum_hess"], nd["split"]["right_hess"], rtol=0, atol=1e-9)
            assert np.isclose(l["sum_grad"] + r["sum_grad"], nd["sum_grad"], rtol=0, atol=1e-9)


def test_tree_recovers_a_planted_two_level_structure():
    """Labels are a function of (feature 1 > 3) and then, on each side, of a different feature:
    the first three splits must be exactly those."""
    rng = np.random.default_rng(11)
    n, F, B = 4000, 5, 8
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    a = bins[:, 1] > 3
    y = np.where(a, np.where(bins[:, 3] > 5, 4.0, 1.0), np.where(bins[:, 0] > 1, -1.0, -4.0))
    grad = (-y).astype(np.float32)                    # square loss at prediction 0: g = -y, h = 1
    hess = np.ones(n, np.float32)
    nodes = tree_oracle.grow_tree(bins, B, grad, hess, 4, 0.0, 0.0)
    assert (nodes[0]["split"]["feature"], nodes[0]["split"]["bin"]) == (1, 3)
    kids = {(nodes[k]["split"]["feature"], nodes[k]["split"]["bin"]) for k in (1, 2)}
    assert kids == {(0, 1), (3, 5)}
    # with 4 leaves every leaf is pure: its value -G/H is the planted label
    for nd in nodes:
        if nd["left"] < 0:
            val = -nd["sum_grad"] / nd["sum_hess"]
            assert min(abs(val - v) for v in (4.0, 1.0, -1.0, -4.0)) < 1e-9


def test_tree_stops_when_nothing_can_be_split():
    bins = np.zeros((50, 3), np.uint8)               # every feature constant: no admissible threshold
    grad = np.linspace(-1, 1, 50).astype(np.float32)
    hess = np.ones(50, np.float32)
    nodes = tree_oracle.grow_tree(bins, 4, grad, hess, 8, 1.0, 0.0)
    assert len(nodes) == 1 and nodes[0]["split"]["feature"] == -1 and nodes[0]["count"] == 50
    # a gain threshold no split reaches stops growth the same way
    bins, grad, hess, B = _tree_problem(3)
    nodes = tree_oracle.grow_tree(bins, B, grad, hess, 8, 1.0, 1e-3, min_split_gain=1e9)
    assert len(nodes) == 1


def test_depthwise_tree_splits_every_splittable_node_level_by_level():
    bins, grad, hess, B = _tree_problem(5, n=1500, F=5, B=12)
    lam, mch = 0.5, 1e-3
    nodes = tree_oracle.grow_tree_depthwise(bins, B, grad, hess, 4, lam, mch)
    assert nodes[0]["depth"] == 0 and max(nd["depth"] for nd in nodes) <= 4
    # numbering: level by level, children in the order of their parents, left first
    depths = [nd["depth"] for nd in nodes]
    assert depths == sorted(depths)
    for k, nd in enumerate(nodes):
        f, t, gain = brute_force_best_split(bins, B, grad, hess, nd["rows"], lam, mch)
        if nd["left"] >= 0:
            assert nd["right"] == nd["left"] + 1 and nodes[nd["left"]]["depth"] == nd["depth"] + 1
            assert (nd["split"]["feature"], nd["split"]["bin"]) == (f, t)       # exhaustive search agrees
        else:
            # a leaf is either at the depth limit or cannot be split at all
            assert nd["depth"] == 4 or f < 0 or not gain > 0.0
    parents = [k for k, nd in enumerate(nodes) if nd["left"] >= 0]
    assert [nodes[k]["left"] for k in parents] == sorted(nodes[k]["left"] for k in parents)
    # rows are where the splits route them
    at = tree_oracle.route_rows(bins, nodes)
    for k, nd in enumerate(nodes):
        if nd["left"] < 0:
            assert np.array_equal(np.nonzero(at == k)[0], nd["rows"])
    # depth 0 is the root alone; a gain threshold nothing reaches stops at the root too
    assert len(tree_oracle.grow_tree_depthwise(bins, B, grad, hess, 0, lam, mch)) == 1
    assert len(tree_oracle.grow_tree_depthwise(bins, B, grad, hess, 4, lam, mch, min_split_gain=1e9)) == 1


def test_depthwise_tree_recovers_the_planted_two_level_structure():
    rng = np.random.default_rng(12)
    n, F, B = 4000, 5, 8
    bins = rng.integers(0, B, size=(n, F), dtype=np.uint8)
    a = bins[:, 1] > 3
    y = np.where(a, np.where(bins[:, 3] > 5, 4.0, 1.0), np.where(bins[:, 0] > 1, -1.0, -4.0))
    grad, hess = (-y).astype(np.float32), np.ones(n, np.float32)
    nodes = tree_oracle.grow_tree_depthwise(bins, B, grad, hess, 2, 0.0, 0.0)
    assert len(nodes) == 7
    assert (nodes[0]["split"]["feature"], nodes[0]["split"]["bin"]) == (1, 3)
    assert (nodes[1]["split"]["feature"], nodes[1]["split"]["bin"]) == (0, 1)      # left child: bins[:,1] <= 3
    assert (nodes[2]["split"]["feature"], nodes[2]["split"]["bin"]) == (3, 5)
    for nd in nodes[3:]:
        assert min(abs(-nd["sum_grad"] / nd["sum_hess"] - v) for v in (4.0, 1.0, -1.0, -4.0)) < 1e-9

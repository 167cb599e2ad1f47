"""GPU parity of gbdt_grow_tree (through the C ABI): the tree the library grows on the device
is replayed with the CPU oracle.  Integer facts (row lists, counts, structure) must be
identical; each choice that floating point decides (which leaf to split, at which feature and
bin) must be the oracle's own choice, or lie inside the band within which fp32 histogram sums
can reorder two candidates of nearly equal gain."""
import numpy as np
import pytest
import torch

from oracle import gbdt_oracle as orc
from oracle import tree_oracle
from paper_1706_08359_amd import binding as B
from paper_1706_08359_amd import synth

from gpu_util import GpuProblem, REL_TOL

pytestmark = pytest.mark.gpu

BAND = 1e-4   # relative gain band inside which two candidates count as tied (as in check_split)


def _say(msg):
    print(msg, flush=True)


def _as_dicts(nodes):
    """NODE_DTYPE array -> the dict form tree_oracle.route_rows understands."""
    return [dict(left=int(nd["left"]), right=int(nd["right"]),
                 split=dict(feature=int(nd["feature"]), bin=int(nd["bin"]))) for nd in nodes]


def _check_structure(nodes, order, bins):
    n = bins.shape[0]
    assert len(nodes) % 2 == 1
    assert nodes[0]["parent"] == -1 and nodes[0]["row_begin"] == 0 and nodes[0]["count"] == n
    for k, nd in enumerate(nodes):
        if nd["left"] < 0:
            assert nd["right"] == -1
            continue
        l, r = nodes[nd["left"]], nodes[nd["right"]]
        assert nd["right"] == nd["left"] + 1 and nd["left"] > k
        assert l["parent"] == k and r["parent"] == k
        assert l["count"] >= 1 and r["count"] >= 1 and l["count"] + r["count"] == nd["count"]
        assert l["row_begin"] == nd["row_begin"] and r["row_begin"] == nd["row_begin"] + l["count"]
        assert nd["feature"] >= 0
    # every leaf's segment holds exactly the rows the stored splits route to it, ascending
    at = tree_oracle.route_rows(bins, _as_dicts(nodes))
    for k, nd in enumerate(nodes):
        if nd["left"] < 0:
            seg = order[nd["row_begin"]:nd["row_begin"] + nd["count"]]
            assert np.array_equal(seg, np.nonzero(at == k)[0]), f"rows of leaf {k}"


def _replay(nodes, bins, n_bins, grad, hess, lam, mch, min_gain=0.0):
    """Follows the device tree's own splits with the oracle and checks every decision."""
    g64, h64 = grad.astype(np.float64), hess.astype(np.float64)
    rows = {0: np.arange(bins.shape[0], dtype=np.int32)}
    best = {}          # oracle's best split and gain table of every node, on the node's rows

    def oracle_best(k):
        if k not in best:
            best[k] = orc.best_split(orc.hist_build(bins, n_bins, grad, hess, rows[k]), lam, mch, return_gains=True)
        return best[k]

    # Sum of |grad| (|hess|) over every leaf whose build kernel output entered a node's
    # histogram: a built child has its own sum, a subtracted sibling its parent's budget plus
    # the built child's.  The library's bound (1e-5 * sum|g| per build, over all bins of a
    # feature together) adds up to 1e-5 * budget for the sums a split record carries.
    budget = {0: (np.abs(g64).sum(), np.abs(h64).sum())}
    open_leaves = [0]
    order = sorted((int(nd["left"]), k) for k, nd in enumerate(nodes) if nd["left"] >= 0)
    near_ties = 0
    for _, k in order:
        nd = nodes[k]
        s_ref, gains = oracle_best(k)
        assert s_ref["feature"] >= 0, f"node {k}: the oracle finds no admissible split"
        scale = max(1.0, abs(s_ref["gain"]))
        # (1) feature and bin: the oracle's choice for this node, or inside the tie band
        g_at = gains[nd["feature"], nd["bin"]]
        assert np.isfinite(g_at), f"node {k}: inadmissible threshold chosen"
        if (nd["feature"], nd["bin"]) != (s_ref["feature"], s_ref["bin"]):
            assert s_ref["gain"] - g_at <= BAND * scale, (k, nd, s_ref, g_at)
            near_ties += 1
        assert abs(nd["gain"] - g_at) <= BAND * scale
        # (2) the leaf: the open leaf with the largest oracle gain, or inside the band
        top = max(oracle_best(j)[0]["gain"] for j in open_leaves if oracle_best(j)[0]["feature"] >= 0)
        assert top - s_ref["gain"] <= BAND * max(1.0, abs(top)), f"node {k} was not the best open leaf"
        assert nd["gain"] > min_gain
        # (3) the children: the oracle's partition of the node's rows by the device's split
        left, right = orc.partition_rows(bins, nd["feature"], nd["bin"], rows[k])
        small_is_left = left.size <= right.size
        small = left if small_is_left else right
        b_small = (np.abs(g64[small]).sum(), np.abs(h64[small]).sum())
        b_large = (budget[k][0] + b_small[0], budget[k][1] + b_small[1])
        for side, kid, r in (("left", nd["left"], left), ("right", nd["right"], right)):
            c = nodes[kid]
            assert c["count"] == r.size, (k, side)
            # the child's sums were read off the parent's histogram
            assert abs(c["sum_grad"] - g64[r].sum()) <= REL_TOL * budget[k][0] + 1e-6 * abs(g64[r].sum())
            assert abs(c["sum_hess"] - h64[r].sum()) <= REL_TOL * budget[k][1] + 1e-6 * abs(h64[r].sum())
            rows[kid] = r
            budget[int(kid)] = b_small if (side == "left") == small_is_left else b_large
        open_leaves.remove(k)
        open_leaves += [int(nd["left"]), int(nd["right"])]
    # growth stopped for a reason
    return open_leaves, oracle_best, near_ties


def _planted(n, F, nb, seed, noise=0.2):
    rng = np.random.default_rng(seed)
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    y = (bins[:, 1] > nb // 2) ^ (bins[:, F // 2] > nb // 3) ^ (rng.random(n) < noise)
    prob = 1.0 / (1.0 + np.exp(-rng.normal(0, 0.3, size=n)))
    return bins, (prob - y).astype(np.float32), (prob * (1 - prob)).astype(np.float32)


@pytest.mark.parametrize("shape", [(60_000, 28, 255, 63), (40_000, 70, 16, 31), (30_000, 100, 64, 31),
                                   (5_000, 9, 33, 255)])
def test_grown_tree_replayed_with_the_oracle(shape):
    n, F, nb, max_leaves = shape
    _say(f"grow_tree {n}x{F} bins={nb} leaves={max_leaves}")
    bins, grad, hess = _planted(n, F, nb, n + F)
    p = GpuProblem(bins, nb, grad, hess)
    lam, mch = 1.0, 1e-3
    nodes, order, _ = B.gbdt_grow_tree(p.packed, n, F, nb, p.grad, p.hess, max_leaves, lam, mch)
    torch.cuda.synchronize()
    order = order.cpu().numpy()[:n]
    n_leaves = int((nodes["left"] < 0).sum())
    assert len(nodes) == 2 * n_leaves - 1
    _check_structure(nodes, order, bins)
    open_leaves, oracle_best, near = _replay(nodes, bins, nb, grad, hess, lam, mch)
    if n_leaves < max_leaves:          # stopped early: no open leaf may have a split left
        assert all(oracle_best(j)[0]["feature"] < 0 or oracle_best(j)[0]["gain"] <= BAND for j in open_leaves)
    else:
        assert n_leaves == max_leaves
    _say(f"  {n_leaves} leaves, {near} near-tie decisions")


def test_grown_tree_equals_the_oracles_tree_on_separated_gains():
    """Square loss on a noiseless planted piecewise-constant target: every gain is far from the
    next, so the device tree must equal the oracle's tree node for node."""
    rng = np.random.default_rng(5)
    n, F, nb = 20_000, 12, 32
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    y = (np.where(bins[:, 3] > 15, 8.0, -8.0) + np.where(bins[:, 7] > 9, 3.0, -3.0)
         + np.where(bins[:, 0] > 20, 1.0, -1.0))
    grad, hess = (-y).astype(np.float32), np.ones(n, np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    nodes, order, _ = B.gbdt_grow_tree(p.packed, n, F, nb, p.grad, p.hess, 8, 0.0, 1.0)
    ref = tree_oracle.grow_tree(bins, nb, grad, hess, 8, 0.0, 1.0)
    assert len(nodes) == len(ref) == 15
    for k, (a, b) in enumerate(zip(nodes, ref)):
        assert (a["left"], a["right"], a["parent"], a["count"]) == (b["left"], b["right"], b["parent"], b["count"]), k
        if b["left"] >= 0:
            assert (a["feature"], a["bin"]) == (b["split"]["feature"], b["split"]["bin"]), k
        assert abs(a["sum_grad"] - b["sum_grad"]) <= 1e-5 * np.abs(grad).sum()
    order = order.cpu().numpy()
    for k, b in enumerate(ref):
        if b["left"] < 0:
            assert np.array_equal(order[nodes[k]["row_begin"]:nodes[k]["row_begin"] + nodes[k]["count"]], b["rows"])


def test_grow_tree_edge_cases():
    _say("grow_tree edge cases")
    rng = np.random.default_rng(8)
    n, F, nb = 3000, 5, 16
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.1, 1, size=n).astype(np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    # a single leaf: the root only, rows in their own order
    nodes, order, scratch = B.gbdt_grow_tree(p.packed, n, F, nb, p.grad, p.hess, 1, 1.0, 1e-3)
    assert len(nodes) == 1 and nodes[0]["left"] == -1 and nodes[0]["count"] == n
    assert np.array_equal(order.cpu().numpy(), np.arange(n))
    assert abs(nodes[0]["sum_grad"] - grad.astype(np.float64).sum()) <= REL_TOL * np.abs(grad).sum()
    # a gain threshold nothing reaches: same tree
    nodes, order, scratch = B.gbdt_grow_tree(p.packed, n, F, nb, p.grad, p.hess, 15, 1.0, 1e-3,
                                             min_split_gain=1e12, scratch=scratch)
    assert len(nodes) == 1
    # constant features: no admissible threshold; the root's sums still come back
    zeros = np.zeros((n, F), np.uint8)
    pz = GpuProblem(zeros, nb, grad, hess)
    nodes, order, _ = B.gbdt_grow_tree(pz.packed, n, F, nb, pz.grad, pz.hess, 15, 1.0, 1e-3)
    assert len(nodes) == 1 and nodes[0]["feature"] == -1
    assert abs(nodes[0]["sum_hess"] - hess.astype(np.float64).sum()) <= REL_TOL * np.abs(hess).sum()
    # more leaves asked for than rows can give: every leaf ends with one row
    tiny = GpuProblem(bins[:6], nb, grad[:6], hess[:6])
    nodes, order, _ = B.gbdt_grow_tree(tiny.packed, 6, F, nb, tiny.grad, tiny.hess, 31, 0.0, 0.0)
    n_leaves = int((nodes["left"] < 0).sum())
    assert n_leaves <= 6 and len(nodes) == 2 * n_leaves - 1
    _check_structure(nodes, order.cpu().numpy()[:6], bins[:6])
    # scratch too small / misaligned
    lib = B.load()
    small = torch.empty(1024, dtype=torch.uint8, device="cuda:0")
    nd = np.zeros(61, dtype=B.NODE_DTYPE)
    import ctypes
    nn = ctypes.c_int32(0)
    args = [p.packed.data_ptr(), n, F, nb, p.grad.data_ptr(), p.hess.data_ptr(), 31, 1.0, 1e-3, 0.0]
    assert lib.gbdt_grow_tree(*args, small.data_ptr(), 1024, nd.ctypes.data, ctypes.byref(nn), None, None) == -4
    assert lib.gbdt_grow_tree(*args, small.data_ptr() + 4, 1 << 30, nd.ctypes.data, ctypes.byref(nn), None, None) == -1
    assert lib.gbdt_grow_tree(*args, None, 1 << 30, nd.ctypes.data, ctypes.byref(nn), None, None) == -1


def test_grow_tree_255_leaves_on_two_million_rows():
    """The tree size of the paper's experiments on a Higgs-shaped matrix (28 features, 255
    bins), replayed in full with the oracle."""
    n, F, nb = 2_000_000, 28, 255
    _say(f"grow_tree {n}x{F} bins={nb} leaves=255")
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(21)
    bins_d = synth.uniform_bins(n, F, nb, gen, dev)
    bins = bins_d.cpu().numpy()
    rng = np.random.default_rng(22)
    score = (bins[:, 2].astype(np.float32) / nb - 0.5) * 2 + (bins[:, 11] > 100) * 1.0 - (bins[:, 20] < 40) * 0.7
    y = rng.random(n) < 1.0 / (1.0 + np.exp(-score))
    prob = np.full(n, 0.5, np.float32)
    grad, hess = (prob - y).astype(np.float32), (prob * (1 - prob)).astype(np.float32)
    p = GpuProblem(bins_d, nb, grad, hess)
    nodes, order, _ = B.gbdt_grow_tree(p.packed, n, F, nb, p.grad, p.hess, 255, 1.0, 1e-3)
    torch.cuda.synchronize()
    assert int((nodes["left"] < 0).sum()) == 255 and len(nodes) == 509
    order = order.cpu().numpy()
    _check_structure(nodes, order, bins)
    _, _, near = _replay(nodes, bins, nb, grad, hess, 1.0, 1e-3)
    _say(f"  255 leaves, {near} near-tie decisions")


# ------------------------------------------------------------------ level-wise growth

def _replay_depthwise(nodes, bins, n_bins, grad, hess, lam, mch, max_depth, min_gain=0.0):
    """Every node of the device tree against the oracle on the node's own rows: the split chosen
    (or a near-tie), the rule "every splittable node above max_depth is split", the children's
    rows, counts and sums.  Returns the number of near-tie decisions."""
    g64, h64 = grad.astype(np.float64), hess.astype(np.float64)
    rows = {0: np.arange(bins.shape[0], dtype=np.int32)}
    budget = {0: (np.abs(g64).sum(), np.abs(h64).sum())}
    depth = {0: 0}
    near = 0
    for k, nd in enumerate(nodes):                      # parents precede children
        s_ref, gains = orc.best_split(orc.hist_build(bins, n_bins, grad, hess, rows[k]), lam, mch, return_gains=True)
        scale = max(1.0, abs(s_ref["gain"]))
        if nd["left"] < 0:
            # a leaf: at the depth limit, or nothing (worth) splitting
            assert depth[k] == max_depth or s_ref["feature"] < 0 or s_ref["gain"] <= min_gain + BAND * scale, k
            if s_ref["feature"] < 0:
                assert nd["feature"] == -1
            continue
        assert depth[k] < max_depth
        assert s_ref["feature"] >= 0, k
        g_at = gains[nd["feature"], nd["bin"]]
        assert np.isfinite(g_at), k
        if (nd["feature"], nd["bin"]) != (s_ref["feature"], s_ref["bin"]):
            assert s_ref["gain"] - g_at <= BAND * scale, (k, nd, s_ref)
            near += 1
        assert abs(nd["gain"] - g_at) <= BAND * scale
        left, right = orc.partition_rows(bins, nd["feature"], nd["bin"], rows[k])
        small_is_left = left.size <= right.size
        small = left if small_is_left else right
        b_small = (np.abs(g64[small]).sum(), np.abs(h64[small]).sum())
        b_large = (budget[k][0] + b_small[0], budget[k][1] + b_small[1])
        for side, kid, r in (("left", int(nd["left"]), left), ("right", int(nd["right"]), right)):
            c = nodes[kid]
            assert c["count"] == r.size and c["parent"] == k
            assert abs(c["sum_grad"] - g64[r].sum()) <= REL_TOL * budget[k][0] + 1e-6 * abs(g64[r].sum())
            assert abs(c["sum_hess"] - h64[r].sum()) <= REL_TOL * budget[k][1] + 1e-6 * abs(h64[r].sum())
            rows[kid], depth[kid] = r, depth[k] + 1
            budget[kid] = b_small if (side == "left") == small_is_left else b_large
    return near


@pytest.mark.parametrize("shape", [(60_000, 28, 255, 6), (40_000, 70, 16, 5), (30_000, 100, 64, 5),
                                   (3_000, 9, 33, 9)])
def test_depthwise_tree_replayed_with_the_oracle(shape):
    n, F, nb, max_depth = shape
    _say(f"grow_tree_depthwise {n}x{F} bins={nb} depth={max_depth}")
    bins, grad, hess = _planted(n, F, nb, n + F + 3)
    p = GpuProblem(bins, nb, grad, hess)
    lam, mch = 1.0, 1e-3
    nodes, order, _ = B.gbdt_grow_tree_depthwise(p.packed, n, F, nb, p.grad, p.hess, max_depth, lam, mch)
    torch.cuda.synchronize()
    _check_structure(nodes, order.cpu().numpy()[:n], bins)
    # numbered level by level, children of a level in the order of their parents
    parents = [k for k in range(len(nodes)) if nodes[k]["left"] >= 0]
    assert [int(nodes[k]["left"]) for k in parents] == sorted(int(nodes[k]["left"]) for k in parents)
    near = _replay_depthwise(nodes, bins, nb, grad, hess, lam, mch, max_depth)
    _say(f"  {len(nodes)} nodes, {near} near-tie decisions")


def test_depthwise_tree_equals_the_oracles_tree_on_separated_gains():
    rng = np.random.default_rng(6)
    n, F, nb = 20_000, 12, 32
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    y = (np.where(bins[:, 3] > 15, 8.0, -8.0) + np.where(bins[:, 7] > 9, 3.0, -3.0)
         + np.where(bins[:, 0] > 20, 1.0, -1.0))
    grad, hess = (-y).astype(np.float32), np.ones(n, np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    nodes, order, _ = B.gbdt_grow_tree_depthwise(p.packed, n, F, nb, p.grad, p.hess, 3, 0.0, 1.0)
    ref = tree_oracle.grow_tree_depthwise(bins, nb, grad, hess, 3, 0.0, 1.0)
    assert len(nodes) == len(ref) == 15
    order = order.cpu().numpy()
    for k, (a, b) in enumerate(zip(nodes, ref)):
        assert (a["left"], a["right"], a["parent"], a["count"]) == (b["left"], b["right"], b["parent"], b["count"]), k
        assert (a["feature"], a["bin"]) == (b["split"]["feature"], b["split"]["bin"]), k
        if b["left"] < 0:
            assert np.array_equal(order[a["row_begin"]:a["row_begin"] + a["count"]], b["rows"])


def test_depthwise_tree_edge_cases():
    _say("grow_tree_depthwise edge cases")
    rng = np.random.default_rng(9)
    n, F, nb = 3000, 5, 16
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.1, 1, size=n).astype(np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    nodes, order, scratch = B.gbdt_grow_tree_depthwise(p.packed, n, F, nb, p.grad, p.hess, 0, 1.0, 1e-3)
    assert len(nodes) == 1 and nodes[0]["count"] == n and nodes[0]["feature"] >= 0      # depth 0: the root, with its split
    assert np.array_equal(order.cpu().numpy(), np.arange(n))
    nodes, order, _ = B.gbdt_grow_tree_depthwise(p.packed, n, F, nb, p.grad, p.hess, 4, 1.0, 1e-3, min_split_gain=1e12)
    assert len(nodes) == 1
    pz = GpuProblem(np.zeros((n, F), np.uint8), nb, grad, hess)
    nodes, order, _ = B.gbdt_grow_tree_depthwise(pz.packed, n, F, nb, pz.grad, pz.hess, 4, 1.0, 1e-3)
    assert len(nodes) == 1 and nodes[0]["feature"] == -1
    assert abs(nodes[0]["sum_hess"] - hess.astype(np.float64).sum()) <= REL_TOL * np.abs(hess).sum()
    tiny = GpuProblem(bins[:6], nb, grad[:6], hess[:6])
    nodes, order, _ = B.gbdt_grow_tree_depthwise(tiny.packed, 6, F, nb, tiny.grad, tiny.hess, 8, 0.0, 0.0)
    _check_structure(nodes, order.cpu().numpy()[:6], bins[:6])
    assert int((nodes["left"] < 0).sum()) <= 6
    with pytest.raises(B.GbdtError):
        B.gbdt_grow_tree_depthwise(p.packed, n, F, nb, p.grad, p.hess, 17, 1.0, 1e-3)


def test_depthwise_tree_depth_8_on_two_million_rows():
    n, F, nb = 2_000_000, 28, 255
    _say(f"grow_tree_depthwise {n}x{F} bins={nb} depth=8")
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(23)
    bins_d = synth.uniform_bins(n, F, nb, gen, dev)
    bins = bins_d.cpu().numpy()
    rng = np.random.default_rng(24)
    score = (bins[:, 2].astype(np.float32) / nb - 0.5) * 2 + (bins[:, 11] > 100) * 1.0 - (bins[:, 20] < 40) * 0.7
    y = rng.random(n) < 1.0 / (1.0 + np.exp(-score))
    prob = np.full(n, 0.5, np.float32)
    grad, hess = (prob - y).astype(np.float32), (prob * (1 - prob)).astype(np.float32)
    p = GpuProblem(bins_d, nb, grad, hess)
    nodes, order, _ = B.gbdt_grow_tree_depthwise(p.packed, n, F, nb, p.grad, p.hess, 8, 1.0, 1e-3)
    torch.cuda.synchronize()
    assert len(nodes) == 511
    _check_structure(nodes, order.cpu().numpy(), bins)
    near = _replay_depthwise(nodes, bins, nb, grad, hess, 1.0, 1e-3, 8)
    _say(f"  511 nodes, {near} near-tie decisions")

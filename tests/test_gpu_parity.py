"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on seeded synthetic inputs.  Counts bit-exact, fp32 sums within
1e-5 * sum|g| (sum|h|) over the leaf, chosen split identical."""
import numpy as np
import pytest
import torch

from oracle import gbdt_oracle as orc
from paper_1706_08359_amd import binding as B
from paper_1706_08359_amd import synth

from gpu_util import GpuProblem, assert_hist_close, check_split

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def test_config1_tiny_dense_is_bit_exact():
    w = synth.config1_tiny_dense()
    _say("config1 10000x28 64 bins root")
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    h = p.build()
    got, ref = B.hist_to_numpy(h), p.oracle()
    # +-0.5 and 0.25 sum exactly in fp32 in any order
    assert (got["count"] == ref["count"]).all()
    assert (got["grad"].astype(np.float64) == ref["grad"]).all()
    assert (got["hess"].astype(np.float64) == ref["hess"]).all()
    s_gpu, s_ref = check_split(h, ref, w.lam, w.min_child_hess, "config1")
    assert (s_gpu["feature"], s_gpu["bin"]) == (s_ref["feature"], s_ref["bin"])


SMALL = [
    # n_rows, n_features, n_bins
    (1, 1, 2), (5, 3, 2), (63, 4, 16), (64, 5, 16), (65, 7, 17), (1000, 28, 64), (4099, 33, 63),
    (5003, 64, 64), (5003, 65, 65), (3001, 100, 256), (7001, 137, 255), (2500, 129, 16),
    (2500, 257, 15), (6007, 200, 64), (9001, 70, 200), (20011, 150, 32),
]


@pytest.mark.parametrize("n_rows,n_features,n_bins", SMALL)
def test_small_shapes_root_indexed_unsorted(n_rows, n_features, n_bins):
    _say(f"small {n_rows}x{n_features} bins={n_bins}")
    rng = np.random.default_rng(n_rows * 1000 + n_features)
    bins = rng.integers(0, n_bins, size=(n_rows, n_features), dtype=np.uint8)
    bins[:, 0] = n_bins - 1                        # the top bin of the capacity class is reachable
    grad = rng.normal(size=n_rows).astype(np.float32)
    hess = rng.uniform(0.01, 1.0, size=n_rows).astype(np.float32)
    p = GpuProblem(bins, n_bins, grad, hess)
    leaves = [("root", None, None), ("first-rows", None, max(1, n_rows // 3))]
    if n_rows > 2:
        leaves.append(("sorted", np.sort(rng.choice(n_rows, size=n_rows // 2 + 1, replace=False)).astype(np.int32), None))
        leaves.append(("unsorted-repeats", rng.integers(0, n_rows, size=n_rows + 17).astype(np.int32), None))
    leaves.append(("single", np.array([n_rows - 1], dtype=np.int32), None))
    for name, idx, n_leaf in leaves:
        h = p.build(idx, n_leaf)
        ref = p.oracle(idx, n_leaf)
        sg, sh = p.leaf_abs_sums(idx, n_leaf)
        assert_hist_close(B.hist_to_numpy(h), ref, sg, sh, f"{name}")
        check_split(h, ref, 1.0, 1e-3, name)


@pytest.mark.parametrize("n_epochs,n_features,n_bins", [(2053, 28, 255), (3121, 40, 64), (2741, 70, 16)])
def test_single_tile_long_leaf_with_a_short_last_unit(n_epochs, n_features, n_bins):
    """One feature tile and a long leaf: every resident workgroup serves that tile, grouped
    around shared work counters; the group slices do not divide into whole units, so short
    last units occur (a unit worked on twice or skipped shows up in the counts)."""
    n_rows = n_epochs * 512 - 77
    _say(f"single tile {n_rows}x{n_features} bins={n_bins}")
    rng = np.random.default_rng(n_epochs)
    bins = rng.integers(0, n_bins, size=(n_rows, n_features), dtype=np.uint8)
    grad = rng.normal(size=n_rows).astype(np.float32)
    hess = rng.uniform(0.01, 1.0, size=n_rows).astype(np.float32)
    p = GpuProblem(bins, n_bins, grad, hess)
    idx = np.sort(rng.choice(n_rows, size=n_rows - 40_001, replace=False)).astype(np.int32)
    for name, leaf in (("root", None), ("indexed", idx)):
        h, ref = p.build(leaf), p.oracle(leaf)
        assert_hist_close(B.hist_to_numpy(h), ref, *p.leaf_abs_sums(leaf), name)
        check_split(h, ref, 1.0, 1e-3, name)


def test_empty_leaf_gives_zero_histogram_and_no_split():
    rng = np.random.default_rng(0)
    bins = rng.integers(0, 64, size=(100, 9), dtype=np.uint8)
    g = np.ones(100, dtype=np.float32)
    p = GpuProblem(bins, 64, g, g)
    h = torch.full((9, 64, 3), float("nan"), device="cuda:0")
    B.gbdt_hist_build(p.packed, 100, 9, 64, None, 0, p.grad, p.hess, hist_out=h)
    got = B.hist_to_numpy(h)
    assert not got["count"].any() and not got["grad"].any() and not got["hess"].any()
    s = B.split_to_dict(B.gbdt_best_split(h, 1.0, 1e-3))
    assert (s["feature"], s["bin"], s["gain"]) == (-1, -1, 0.0)
    empty_idx = torch.zeros(0, dtype=torch.int32, device="cuda:0")
    h2 = B.gbdt_hist_build(p.packed, 100, 9, 64, empty_idx, 0, p.grad, p.hess)
    assert not B.hist_to_numpy(h2)["count"].any()


def test_skewed_bins_single_value_feature():
    """App. A.3's worst case: a feature whose rows all share one bin, plus 60 % zeros."""
    rng = np.random.default_rng(5)
    n, F, nb = 30011, 70, 255
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    bins[:, 3] = 200
    bins[rng.random((n, F)) < 0.6] = 0
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.01, 1.0, size=n).astype(np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    h, ref = p.build(), p.oracle()
    assert_hist_close(B.hist_to_numpy(h), ref, *p.leaf_abs_sums(), "skew")
    check_split(h, ref, 1.0, 1e-3, "skew")


def test_counts_are_reproducible_and_sums_stable():
    w = synth.config2_dense_wide(n_rows=50_000, n_features=300, with_leaves=False)
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    a = B.hist_to_numpy(p.build())
    sg, sh = p.leaf_abs_sums()
    for _ in range(3):
        b = B.hist_to_numpy(p.build())
        assert (a["count"] == b["count"]).all()
        assert np.abs(a["grad"].astype(np.float64) - b["grad"]).max() <= 1e-5 * sg


def test_deterministic_mode_is_bit_reproducible():
    w = synth.config4_ranking_sparse(n_rows=700_000, fractions=(1.0, 0.5))
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    try:
        B.gbdt_set_deterministic(True)
        for leaf in w.leaves:
            a = B.hist_to_numpy(p.build(leaf))
            ref = p.oracle(leaf)
            assert_hist_close(a, ref, *p.leaf_abs_sums(leaf), "deterministic")
            for _ in range(3):
                b = B.hist_to_numpy(p.build(leaf))
                assert a.tobytes() == b.tobytes()
    finally:
        B.gbdt_set_deterministic(False)
    # the default mode agrees with it to the tolerance (and exactly in the counts)
    c = B.hist_to_numpy(p.build(w.leaves[0]))
    B.gbdt_set_deterministic(True)
    try:
        d = B.hist_to_numpy(p.build(w.leaves[0]))
    finally:
        B.gbdt_set_deterministic(False)
    assert (c["count"] == d["count"]).all()
    sg, sh = p.leaf_abs_sums(w.leaves[0])
    assert np.abs(c["grad"].astype(np.float64) - d["grad"]).max() <= 1e-5 * sg


def test_subtract_matches_oracle_and_may_alias():
    rng = np.random.default_rng(11)
    n, F, nb = 40_000, 90, 64
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.01, 1.0, size=n).astype(np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    parent_rows = np.sort(rng.choice(n, size=30_000, replace=False)).astype(np.int32)
    left = parent_rows[bins[parent_rows, 7] <= 25]
    right = parent_rows[bins[parent_rows, 7] > 25]
    hp, hl = p.build(parent_rows), p.build(left)
    sib = B.gbdt_hist_subtract(hp, hl)
    ref_sib = orc.hist_subtract(p.oracle(parent_rows), p.oracle(left))
    sg, sh = p.leaf_abs_sums(parent_rows)       # sibling inherits the parent's rounding
    assert_hist_close(B.hist_to_numpy(sib), ref_sib, sg, sh, "sibling")
    # it is the histogram of the right child, too
    assert_hist_close(B.hist_to_numpy(sib), p.oracle(right), sg, sh, "sibling-vs-right")
    # elementwise exactness of the subtraction itself on the fp32 inputs
    a, b, c = B.hist_to_numpy(hp), B.hist_to_numpy(hl), B.hist_to_numpy(sib)
    assert (c["grad"] == a["grad"] - b["grad"]).all() and (c["hess"] == a["hess"] - b["hess"]).all()
    assert (c["count"] == a["count"] - b["count"]).all()
    keep = c.copy()
    B.gbdt_hist_subtract(hp, hl, sibling_out=hp)   # alias parent
    assert (B.hist_to_numpy(hp) == keep).all()


def test_user_workspace_and_too_small_workspace():
    w = synth.config2_dense_wide(n_rows=20_000, n_features=200, with_leaves=False)
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    ref = B.hist_to_numpy(p.build())
    need = B.gbdt_workspace_bytes(w.n_rows, w.n_features, w.n_bins)
    buf = torch.empty(need, dtype=torch.uint8, device="cuda:0")
    try:
        B.gbdt_set_workspace(buf)
        got = B.hist_to_numpy(p.build())
        assert (got["count"] == ref["count"]).all()
        tiny = torch.empty(256, dtype=torch.uint8, device="cuda:0")
        B.gbdt_set_workspace(tiny)
        with pytest.raises(B.GbdtError, match="workspace"):
            p.build()
    finally:
        B.gbdt_set_workspace(None)
    assert (B.hist_to_numpy(p.build())["count"] == ref["count"]).all()


def test_graph_capture_replays_match_eager():
    """build + subtract + best split captured into one graph and replayed with changing
    inputs; every replay is checked against the eager result (the calls clear memory with
    fill kernels, not memset nodes)."""
    w = synth.config2_dense_wide(n_rows=80_000, n_features=300, with_leaves=False)
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    n, F, nb = p.n_rows, p.n_features, p.n_bins
    idx = torch.arange(0, n, 3, dtype=torch.int32, device="cuda:0")
    parent = p.build()
    hist, sib = torch.empty_like(parent), torch.empty_like(parent)
    split = torch.empty(9, dtype=torch.int32, device="cuda:0")

    def step(h, s_, sp):
        B.gbdt_hist_build(p.packed, n, F, nb, idx, idx.numel(), p.grad, p.hess, hist_out=h)
        B.gbdt_hist_subtract(parent, h, sibling_out=s_)
        B.gbdt_best_split(h, w.lam, w.min_child_hess, split_out=sp)

    B.gbdt_set_deterministic(True)          # so that replays can be compared bit for bit
    try:
        step(hist, sib, split)              # warm-up: workspace and occupancy query outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step(hist, sib, split)
        e_hist, e_sib = torch.empty_like(parent), torch.empty_like(parent)
        e_split = torch.empty_like(split)
        for trial in range(4):
            p.grad.mul_(-1.25).add_(0.01 * trial)      # the program's own eager work between replays
            p.hess.mul_(0.9).add_(0.05)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            step(e_hist, e_sib, e_split)
            torch.cuda.synchronize()
            assert torch.equal(hist.view(torch.int32), e_hist.view(torch.int32)), trial
            assert torch.equal(sib.view(torch.int32), e_sib.view(torch.int32)), trial
            assert torch.equal(split, e_split), trial
        # and the last replay against the oracle
        ref = orc.hist_build(p.bins_cpu.numpy(), nb, p.grad.cpu().numpy(), p.hess.cpu().numpy(), idx.cpu().numpy())
        g64, h64 = p.grad[idx.long()].double(), p.hess[idx.long()].double()
        assert_hist_close(B.hist_to_numpy(hist), ref, g64.abs().sum().item(), h64.abs().sum().item(), "graph")
    finally:
        B.gbdt_set_deterministic(False)


def test_unit_counters_stay_consistent_across_scratch_buffers_and_graphs():
    """The run-time hand-out of work keeps its counters at the head of the scratch buffer and
    expects them zero between calls.  Buffers that arrive full of garbage, switching between
    caller and library scratch, and a captured graph replayed between eager calls must all
    leave every histogram right (a wrong counter would skip or repeat units: counts off)."""
    n, F, nb = 300_000, 40, 64
    rng = np.random.default_rng(77)
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.1, 1.0, size=n).astype(np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    idx = torch.arange(0, n, 2, dtype=torch.int32, device="cuda:0")
    ref_root, ref_leaf = p.oracle(), p.oracle(idx)
    sg, sh = p.leaf_abs_sums()
    lg, lh = p.leaf_abs_sums(idx)

    def check(tag):
        assert_hist_close(B.hist_to_numpy(p.build()), ref_root, sg, sh, tag + " root")
        assert_hist_close(B.hist_to_numpy(p.build(idx)), ref_leaf, lg, lh, tag + " leaf")

    need = B.gbdt_workspace_bytes(n, F, nb)
    ws_a = torch.full((need,), 0xAB, dtype=torch.uint8, device="cuda:0")
    ws_b = torch.full((need,), 0xFF, dtype=torch.uint8, device="cuda:0")
    try:
        check("library scratch")
        B.gbdt_set_workspace(ws_a)
        check("caller scratch A (garbage)")
        check("caller scratch A again")
        B.gbdt_set_workspace(None)
        check("library scratch again")
        B.gbdt_set_workspace(ws_b)
        check("caller scratch B (garbage)")
        ws_b.fill_(0x5C)                      # the caller overwrote its buffer and registers it anew
        B.gbdt_set_workspace(ws_b)
        check("caller scratch B refilled")
        # a graph captured on this buffer, replayed between eager calls
        hist = torch.empty((F, nb, 3), dtype=torch.float32, device="cuda:0")
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            B.gbdt_hist_build(p.packed, n, F, nb, idx, idx.numel(), p.grad, p.hess, hist_out=hist)
        for trial in range(3):
            hist.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert_hist_close(B.hist_to_numpy(hist), ref_leaf, lg, lh, f"replay {trial}")
            check(f"eager after replay {trial}")
    finally:
        B.gbdt_set_workspace(None)
    check("library scratch at the end")


def test_runs_on_a_side_stream():
    w = synth.config1_tiny_dense()
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    ref = p.oracle()
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        h = p.build()
        sp = B.gbdt_best_split(h, w.lam, w.min_child_hess)
    s.synchronize()
    assert (B.hist_to_numpy(h)["count"] == ref["count"]).all()
    r = orc.best_split(ref, w.lam, w.min_child_hess)
    assert B.split_to_dict(sp)["feature"] == r["feature"]


# ------------------------------------------------------- scaled-down configs 2..5


def test_config2_scaled_tree_leaves():
    w = synth.config2_dense_wide(n_rows=60_000, n_features=520, tree_depth=5, min_fraction=0.02)
    _say(f"config2 scaled: {len(w.leaves)} leaves")
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    for k, leaf in enumerate(w.leaves):
        h, ref = p.build(leaf), p.oracle(leaf)
        assert_hist_close(B.hist_to_numpy(h), ref, *p.leaf_abs_sums(leaf), f"leaf{k}")
        check_split(h, ref, w.lam, w.min_child_hess, f"config2 leaf{k}")


def test_config4_scaled_sparse_leaves():
    w = synth.config4_ranking_sparse(n_rows=150_000)
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    for k, leaf in enumerate(w.leaves):
        h, ref = p.build(leaf), p.oracle(leaf)
        assert_hist_close(B.hist_to_numpy(h), ref, *p.leaf_abs_sums(leaf), f"leaf{k}")
        check_split(h, ref, w.lam, w.min_child_hess, f"config4 leaf{k}")


def _grow_tree(p, w, n_leaves):
    """Leaf-wise growth: split the open leaf of largest gain, build the smaller child,
    obtain the sibling by subtraction.  Row sets follow the ORACLE's split so that a GPU /
    oracle divergence cannot compound.  Every histogram and split is compared."""
    bins_np = p.bins_cpu.numpy()
    root_rows = np.arange(p.n_rows, dtype=np.int32)
    h_gpu = p.build()
    h_ref = p.oracle()
    assert_hist_close(B.hist_to_numpy(h_gpu), h_ref, *p.leaf_abs_sums(), "root")
    _, s_ref = check_split(h_gpu, h_ref, w.lam, w.min_child_hess, "root")
    open_leaves = [dict(rows=root_rows, gpu=h_gpu, ref=h_ref, split=s_ref)]
    n = 1
    while n < n_leaves:
        cand = [l for l in open_leaves if l["split"]["feature"] >= 0]
        if not cand:
            break
        leaf = max(cand, key=lambda l: l["split"]["gain"])
        open_leaves = [l for l in open_leaves if l is not leaf]
        f, t = leaf["split"]["feature"], leaf["split"]["bin"]
        go_left = bins_np[leaf["rows"], f] <= t
        left, right = leaf["rows"][go_left], leaf["rows"][~go_left]
        assert left.size == leaf["split"]["left_count"] and right.size == leaf["split"]["right_count"]
        small, large = (left, right) if left.size <= right.size else (right, left)
        hs_gpu = p.build(small)
        hs_ref = p.oracle(small)
        assert_hist_close(B.hist_to_numpy(hs_gpu), hs_ref, *p.leaf_abs_sums(small), f"small@{n}")
        hl_gpu = B.gbdt_hist_subtract(leaf["gpu"], hs_gpu)
        hl_ref = orc.hist_subtract(leaf["ref"], hs_ref)
        # the sibling's error budget is the parent's
        assert_hist_close(B.hist_to_numpy(hl_gpu), hl_ref, *p.leaf_abs_sums(leaf["rows"]), f"sibling@{n}")
        for rows, hg, hr in ((small, hs_gpu, hs_ref), (large, hl_gpu, hl_ref)):
            _, s = check_split(hg, hr, w.lam, w.min_child_hess, f"node@{n}")
            open_leaves.append(dict(rows=rows, gpu=hg, ref=hr, split=s))
        n += 1
    return n


def test_config3_scaled_tree_with_subtraction():
    w = synth.config3_dense_tall(n_rows=300_000, exact_binning=True)
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    n = _grow_tree(p, w, 63)
    _say(f"config3 scaled: grew {n} leaves")
    assert n == 63


def test_config5_scaled_tree_with_subtraction():
    w = synth.config5_categorical(n_rows=200_000, n_features=700)
    p = GpuProblem(w.bins, w.n_bins, w.grad, w.hess)
    n = _grow_tree(p, w, 31)
    _say(f"config5 scaled: grew {n} leaves")
    assert n == 31

"""GPU parity of gbdt_partition_rows (through the C ABI) against the CPU oracle: integer
work, so every output element must be identical.  Also grows whole trees with the library
alone (build, split search, partition, smaller-child build, subtraction) and checks each
node against the oracle."""
import numpy as np
import pytest
import torch

from oracle import gbdt_oracle as orc
from paper_1706_08359_amd import binding as B
from paper_1706_08359_amd import synth

from gpu_util import GpuProblem, assert_hist_close

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _partition(p, feature, thr, idx=None, n_leaf=None):
    """Run the HIP partition; returns (left, right) numpy arrays and the device count."""
    dev = p.dev
    if idx is None:
        n = p.n_rows if n_leaf is None else n_leaf
        idx_d = None
    else:
        idx_d = torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32)).to(dev)
        n = idx_d.numel() if n_leaf is None else n_leaf
    rec = B.split_record(feature, thr, dev)
    out = torch.full((max(n, 1) + 8,), -7, dtype=torch.int32, device=dev)   # guard words behind
    n_left = torch.full((1,), -1, dtype=torch.int64, device=dev)
    B.gbdt_partition_rows(p.packed, p.n_rows, p.n_features, p.n_bins, idx_d, n, rec, out, n_left)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    nl = int(n_left.item())
    assert (o[n:] == -7).all(), "wrote past children_out[n_leaf_rows]"
    return o[:nl], o[nl:n], nl


def _check(p, feature, thr, idx=None, n_leaf=None, what=""):
    left, right, nl = _partition(p, feature, thr, idx, n_leaf)
    ref_l, ref_r = orc.partition_rows(p.bins_cpu.numpy(), feature, thr, idx, n_leaf)
    assert nl == ref_l.size, (what, nl, ref_l.size)
    assert np.array_equal(left, ref_l), what
    assert np.array_equal(right, ref_r), what


SHAPES = [
    # n_rows, n_features, n_bins: every kernel variant, both tile kinds, 4-bit halves
    (1, 1, 2), (63, 4, 16), (257, 5, 16), (2049, 7, 17), (4099, 33, 63), (5003, 65, 65),
    (3001, 100, 256), (7001, 137, 255), (2500, 129, 16), (2500, 257, 15), (20011, 150, 32),
]


@pytest.mark.parametrize("n_rows,n_features,n_bins", SHAPES)
def test_partition_small_shapes(n_rows, n_features, n_bins):
    _say(f"partition small {n_rows}x{n_features} bins={n_bins}")
    rng = np.random.default_rng(31 * n_rows + n_features)
    bins = rng.integers(0, n_bins, size=(n_rows, n_features), dtype=np.uint8)
    zeros = np.zeros(n_rows, np.float32)
    p = GpuProblem(bins, n_bins, zeros, zeros)
    feats = sorted({0, n_features - 1, n_features // 2, min(n_features - 1, 1), min(n_features - 1, 64),
                    min(n_features - 1, 33), min(n_features - 1, 127)})
    for f in feats:
        thr = int(rng.integers(0, n_bins - 1))
        _check(p, f, thr, None, None, f"root f={f} t={thr}")
        if n_rows > 2:
            sub = np.sort(rng.choice(n_rows, size=n_rows // 2 + 1, replace=False)).astype(np.int32)
            _check(p, f, thr, sub, None, f"sorted f={f} t={thr}")
    f = feats[-1]
    _check(p, f, 0, None, max(1, n_rows // 3), "first rows")
    _check(p, f, n_bins - 1, None, None, "all left")
    _check(p, f, -1, None, None, "all right")
    shuffled = rng.integers(0, n_rows, size=n_rows + 19).astype(np.int32)   # any order, repeats
    _check(p, f, n_bins // 2, shuffled, None, "unsorted with repeats")
    _check(p, f, n_bins // 2, np.array([n_rows - 1], np.int32), None, "single row")


def test_partition_empty_leaf_and_no_split():
    _say("partition empty leaf / feature -1")
    rng = np.random.default_rng(3)
    bins = rng.integers(0, 64, size=(3000, 10), dtype=np.uint8)
    zeros = np.zeros(3000, np.float32)
    p = GpuProblem(bins, 64, zeros, zeros)
    left, right, nl = _partition(p, 2, 10, np.zeros(0, np.int32))
    assert nl == 0 and left.size == 0 and right.size == 0
    # "no admissible split" record: nothing moves, all rows stay (left), order kept
    sub = np.sort(rng.choice(3000, size=1234, replace=False)).astype(np.int32)
    left, right, nl = _partition(p, -1, -1, sub)
    assert nl == sub.size and np.array_equal(left, sub) and right.size == 0


def test_partition_argument_errors():
    dev = torch.device("cuda:0")
    bins = torch.zeros((100, 4), dtype=torch.uint8, device=dev)
    packed = B.gbdt_bins_pack(bins, 16)
    rec = B.split_record(0, 0, dev)
    out = torch.empty(100, dtype=torch.int32, device=dev)
    lib = B.load()
    nl = torch.empty(1, dtype=torch.int64, device=dev)
    args = lambda **k: [k.get("m", packed.data_ptr()), 100, k.get("F", 4), k.get("nb", 16), None,
                        k.get("n", 100), k.get("rec", rec.data_ptr()), k.get("out", out.data_ptr()),
                        nl.data_ptr(), None]
    assert lib.gbdt_partition_rows(*args()) == 0
    assert lib.gbdt_partition_rows(*args(m=None)) == -1
    assert lib.gbdt_partition_rows(*args(rec=None)) == -1
    assert lib.gbdt_partition_rows(*args(out=None)) == -1
    assert lib.gbdt_partition_rows(*args(n=101)) == -1        # NULL index list: n_leaf <= n_rows
    assert lib.gbdt_partition_rows(*args(n=-1)) == -1
    assert lib.gbdt_partition_rows(*args(nb=1)) == -1
    assert lib.gbdt_partition_rows(*args(F=0)) == -1
    torch.cuda.synchronize()


def test_partition_many_chunks_and_caller_workspace():
    """A leaf of several thousand chunks (ragged last one), once with library scratch and once
    with a caller buffer of exactly gbdt_workspace_bytes."""
    n, F, nb = 1_500_037, 40, 200
    _say(f"partition {n}x{F} bins={nb}")
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(11)
    bins = synth.uniform_bins(n, F, nb, gen, torch.device("cuda:0"))
    zeros = torch.zeros(n, dtype=torch.float32)
    p = GpuProblem(bins, nb, zeros, zeros)
    rng = np.random.default_rng(12)
    sub = np.sort(rng.choice(n, size=777_001, replace=False)).astype(np.int32)
    _check(p, 37, 120, None, None, "root")
    _check(p, 3, 10, sub, None, "sorted half")
    ws = torch.empty(B.gbdt_workspace_bytes(n, F, nb), dtype=torch.uint8, device="cuda:0")
    B.gbdt_set_workspace(ws)
    try:
        _check(p, 39, 60, None, None, "root, caller workspace")
    finally:
        B.gbdt_set_workspace(None)


@pytest.mark.parametrize("n", [4_194_304 + 5, 8_388_608 + 4099, 17_000_001])
def test_partition_long_lists_take_longer_chunks(n):
    """Lists of more than 2048 x 2048 positions are cut into chunks of 4096, 8192, ... positions,
    which a workgroup takes 16 steps at a time: the root, a sorted list with a ragged end that
    falls in the first steps of the last chunk, and an unsorted list with repeated rows; one
    split that sends nearly every row left, one that splits evenly."""
    F, nb = 2, 50
    plan = B.gbdt_debug_partition_plan(n)
    _say(f"partition {n}x{F} bins={nb}: {plan}")
    assert plan["rows_per_thread"] >= 16
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(n % 1000)
    bins = synth.uniform_bins(n, F, nb, gen, torch.device("cuda:0"))
    zeros = torch.zeros(n, dtype=torch.float32)
    p = GpuProblem(bins, nb, zeros, zeros)
    _check(p, 1, 24, None, None, "root, even split")
    _check(p, 0, 47, None, None, "root, nearly all left")
    rng = np.random.default_rng(n % 977)
    m = plan["rows_per_thread"] * 256 * (plan["chunks"] - 2) + 300     # ends in the first steps of a chunk
    if B.gbdt_debug_partition_plan(m)["rows_per_thread"] >= 16:
        sub = np.sort(rng.choice(n, size=m, replace=False)).astype(np.int32)
        _check(p, 1, 10, sub, None, "sorted list, ragged end")
    rep = rng.integers(0, n, size=4_194_304 + 77).astype(np.int32)      # unsorted, with repeats
    _check(p, 0, 30, rep, None, "unsorted list with repeats")


# ------------------------------------------------------------------ whole trees on the device

def _grow_tree_on_device(p, n_leaves, lam, mch):
    """Leaf-wise growth with library calls only.  Per split the host reads two 36-byte split
    records (it needs them to choose the next leaf); row lists and histograms stay in HBM.
    Returns one entry per split made.

    Each leaf also carries the sum of |grad| (|hess|) over every leaf whose build kernel
    output entered its histogram: a built child has its own sum, a subtracted sibling its
    parent's budget plus the built child's.  The library's bound of 1e-5 * sum|g| per build
    adds up to 1e-5 * budget for such a histogram."""
    n, F, nb = p.n_rows, p.n_features, p.n_bins
    g64 = np.abs(p.grad_cpu.numpy().astype(np.float64))
    h64 = np.abs(p.hess_cpu.numpy().astype(np.float64))
    root_hist = B.gbdt_hist_build(p.packed, n, F, nb, None, n, p.grad, p.hess)
    root_split = B.gbdt_best_split(root_hist, lam, mch)
    leaves = [dict(rows=None, n=n, hist=root_hist, rec=root_split, s=B.split_to_dict(root_split),
                   budget=(g64.sum(), h64.sum()))]
    made = []
    while len(leaves) < n_leaves:
        cands = [l for l in leaves if l["s"]["feature"] >= 0]
        if not cands:
            break
        best = max(cands, key=lambda l: l["s"]["gain"])
        leaves = [l for l in leaves if l is not best]
        kids, n_left = B.gbdt_partition_rows(p.packed, n, F, nb, best["rows"], best["n"], best["rec"])
        nl, nr = best["s"]["left_count"], best["s"]["right_count"]
        assert nl + nr == best["n"]
        assert int(n_left.item()) == nl           # the histogram's count and the partition agree
        rows_l, rows_r = kids[:nl], kids[nl:nl + nr]
        left_is_small = nl <= nr
        small = rows_l if left_is_small else rows_r
        h_small = B.gbdt_hist_build(p.packed, n, F, nb, small, small.numel(), p.grad, p.hess)
        h_large = B.gbdt_hist_subtract(best["hist"], h_small)
        small_np = small.cpu().numpy()
        b_small = (g64[small_np].sum(), h64[small_np].sum())
        b_large = (best["budget"][0] + b_small[0], best["budget"][1] + b_small[1])
        h_l, h_r = (h_small, h_large) if left_is_small else (h_large, h_small)
        b_l, b_r = (b_small, b_large) if left_is_small else (b_large, b_small)
        rec_l, rec_r = B.gbdt_best_split(h_l, lam, mch), B.gbdt_best_split(h_r, lam, mch)
        parent_rows = np.arange(n, dtype=np.int32) if best["rows"] is None else best["rows"].cpu().numpy()
        made.append(dict(rows=parent_rows, s=best["s"], h_l=h_l, h_r=h_r, rows_l=rows_l, rows_r=rows_r,
                         b_l=b_l, b_r=b_r))
        leaves.append(dict(rows=rows_l, n=nl, hist=h_l, rec=rec_l, s=B.split_to_dict(rec_l), budget=b_l))
        leaves.append(dict(rows=rows_r, n=nr, hist=h_r, rec=rec_r, s=B.split_to_dict(rec_r), budget=b_r))
    return made


@pytest.mark.parametrize("shape", [(60_000, 28, 255, 31), (40_000, 70, 16, 15), (30_000, 100, 64, 15)])
def test_tree_grown_on_device_matches_oracle_node_by_node(shape):
    """Every node the device-grown tree splits is replayed with the oracle on the node's own
    rows: the children must be the oracle's partition of those rows (identical lists), their
    histograms must match the oracle's within the accumulated build tolerance, and the split
    of each node must be the oracle scan's choice on the device's own fp32 histogram."""
    n, F, nb, n_leaves = shape
    _say(f"device tree {n}x{F} bins={nb} leaves={n_leaves}")
    rng = np.random.default_rng(n + F)
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    y = (bins[:, 1] > nb // 2) ^ (bins[:, F // 2] > nb // 3) ^ (rng.random(n) < 0.2)
    score = rng.normal(0, 0.3, size=n)
    prob = 1.0 / (1.0 + np.exp(-score))
    grad = (prob - y).astype(np.float32)
    hess = (prob * (1 - prob)).astype(np.float32)
    p = GpuProblem(bins, nb, grad, hess)
    lam, mch = 1.0, 1e-3
    made = _grow_tree_on_device(p, n_leaves, lam, mch)
    assert len(made) == n_leaves - 1
    for k, m in enumerate(made):
        s = m["s"]
        ref_l, ref_r = orc.partition_rows(bins, s["feature"], s["bin"], m["rows"])
        assert np.array_equal(m["rows_l"].cpu().numpy(), ref_l), f"node {k}: left rows"
        assert np.array_equal(m["rows_r"].cpu().numpy(), ref_r), f"node {k}: right rows"
        for side, h, ref_rows, budget in (("left", m["h_l"], ref_l, m["b_l"]), ("right", m["h_r"], ref_r, m["b_r"])):
            got = B.hist_to_numpy(h)
            assert_hist_close(got, orc.hist_build(bins, nb, grad, hess, ref_rows), budget[0], budget[1],
                              f"node {k} {side}")
            lifted = orc.from_f32_hist(got["grad"], got["hess"], got["count"])
            s_same = orc.best_split(lifted, lam, mch)
            s_dev = B.split_to_dict(B.gbdt_best_split(h, lam, mch))
            assert (s_dev["feature"], s_dev["bin"]) == (s_same["feature"], s_same["bin"]), f"node {k} {side}"
    # the first split is found identically by both sides end to end
    ref_root = orc.best_split(orc.hist_build(bins, nb, grad, hess), lam, mch)
    assert (made[0]["s"]["feature"], made[0]["s"]["bin"]) == (ref_root["feature"], ref_root["bin"])


def test_check_inputs_env_turns_a_bad_row_id_into_an_error():
    """GBDT_HIST_CHECK_INPUTS=1 is read when the library is first used, so this runs in a child
    process: a row list with an id past the matrix must come back as GBDT_EINVAL from the build,
    the batched build and the partition, and a clean list must still work."""
    import os
    import subprocess
    import sys
    code = r'''
import numpy as np, torch
from paper_1706_08359_amd import binding as B
dev = torch.device("cuda:0")
bins = torch.randint(0, 32, (5000, 20), dtype=torch.uint8, device=dev)
packed = B.gbdt_bins_pack(bins, 32)
g = torch.randn(5000, device=dev); h = torch.rand(5000, device=dev)
good = torch.arange(0, 5000, 2, dtype=torch.int32, device=dev)
bad = good.clone(); bad[100] = 5000      # one past the last row: inside every buffer's slack, so harmless even unchecked
rec = B.split_record(3, 10, dev)
B.gbdt_hist_build(packed, 5000, 20, 32, good, good.numel(), g, h)
B.gbdt_hist_build_batch(packed, 5000, 20, 32, good, [0, 1000, 2500], g, h)
B.gbdt_partition_rows(packed, 5000, 20, 32, good, good.numel(), rec)
n_err = 0
for call in (lambda: B.gbdt_hist_build(packed, 5000, 20, 32, bad, bad.numel(), g, h),
             lambda: B.gbdt_hist_build_batch(packed, 5000, 20, 32, bad, [0, 1000, 2500], g, h),
             lambda: B.gbdt_partition_rows(packed, 5000, 20, 32, bad, bad.numel(), rec)):
    try:
        call()
    except B.GbdtError as e:
        assert "(-1)" in str(e), e
        n_err += 1
torch.cuda.synchronize()
assert n_err == 3, n_err
print("checked ok")
'''
    env = dict(os.environ, GBDT_HIST_CHECK_INPUTS="1")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, "-c", code], cwd=root, env=env, capture_output=True, text=True, timeout=180)
    assert res.returncode == 0 and "checked ok" in res.stdout, res.stdout + res.stderr


@pytest.mark.parametrize("shape", [(20_011, 150, 32, 7), (9_001, 28, 255, 300), (2_500, 129, 16, 40),
                                   (400_000, 70, 64, 5)])
def test_partition_batch_equals_oracle_leaf_by_leaf(shape):
    """A level of a tree in one call: every leaf's segment of children_out must be the oracle's
    partition of that leaf by that leaf's own split record (empty leaves, records without a
    split, tiny and multi-chunk leaves, more leaves than one launch holds)."""
    n_rows, n_features, n_bins, n_leaves = shape
    _say(f"partition batch {n_rows}x{n_features} bins={n_bins} leaves={n_leaves}")
    rng = np.random.default_rng(n_rows + n_leaves)
    bins = rng.integers(0, n_bins, size=(n_rows, n_features), dtype=np.uint8)
    zeros = np.zeros(n_rows, np.float32)
    p = GpuProblem(bins, n_bins, zeros, zeros)
    perm = rng.permutation(n_rows).astype(np.int32)
    cuts = np.sort(rng.choice(n_rows, size=n_leaves - 1, replace=False))
    lists = [np.sort(x) for x in np.split(perm, cuts)]
    lists[1] = np.zeros(0, np.int32) if n_leaves > 2 else lists[1]          # an empty leaf
    offs = np.concatenate([[3], 3 + np.cumsum([len(l) for l in lists])]).astype(np.int64)
    cat = np.concatenate([np.full(3, -1, np.int32)] + lists + [np.full(5, -1, np.int32)])
    feats = rng.integers(0, n_features, size=n_leaves)
    thrs = rng.integers(0, n_bins - 1, size=n_leaves)
    feats[0] = -1                                                            # "no split": all rows stay left
    recs = np.zeros(n_leaves, dtype=B.SPLIT_DTYPE)
    recs["feature"], recs["bin"] = feats, thrs
    recs_d = torch.from_numpy(recs.view(np.int32).reshape(n_leaves, 9).copy()).to(p.dev)
    out = torch.full((cat.size,), -7, dtype=torch.int32, device=p.dev)
    n_left = torch.full((n_leaves,), -1, dtype=torch.int64, device=p.dev)
    B.gbdt_partition_rows_batch(p.packed, n_rows, n_features, n_bins, torch.from_numpy(cat).to(p.dev), offs,
                                recs_d, out, n_left)
    torch.cuda.synchronize()
    o, nl = out.cpu().numpy(), n_left.cpu().numpy()
    assert (o[:3] == -7).all() and (o[offs[-1]:] == -7).all()              # nothing outside the lists
    for l, rows in enumerate(lists):
        seg = o[offs[l]:offs[l + 1]]
        if feats[l] < 0:
            assert nl[l] == rows.size and np.array_equal(seg, rows), l
            continue
        ref_l, ref_r = orc.partition_rows(bins, int(feats[l]), int(thrs[l]), rows)
        assert nl[l] == ref_l.size, (l, nl[l], ref_l.size)
        assert np.array_equal(seg[:ref_l.size], ref_l) and np.array_equal(seg[ref_l.size:], ref_r), l


@pytest.mark.parametrize("n_rows,n_features,n_bins", [(1, 1, 2), (63, 5, 16), (1000, 28, 64), (4099, 137, 255),
                                                      (2500, 257, 15), (70_001, 65, 63)])
def test_packed_layout_holds_a_column_major_copy(n_rows, n_features, n_bins):
    """Behind the tiles and their slack gbdt_bins_pack stores every feature once more as a column
    of bytes (padded to a multiple of 256 rows): the bytes there are the matrix, transposed."""
    rng = np.random.default_rng(n_rows + n_features)
    bins = rng.integers(0, n_bins, size=(n_rows, n_features), dtype=np.uint8)
    packed = B.gbdt_bins_pack(torch.from_numpy(bins).to("cuda:0"), n_bins)
    torch.cuda.synchronize()
    g = B.gbdt_debug_geometry(n_features, n_bins, n_rows)
    base = (n_rows * g["row_bytes"] + 512 * 64 + 255) // 256 * 256
    stride = (n_rows + 255) // 256 * 256
    assert packed.numel() == B.gbdt_bins_packed_bytes(n_rows, n_features, n_bins) == base + n_features * stride
    cols = packed.cpu().numpy()[base:base + n_features * stride].reshape(n_features, stride)
    assert np.array_equal(cols[:, :n_rows], bins.T)
    assert not cols[:, n_rows:(n_rows + 63) // 64 * 64].any()      # the written part of the padding is zero

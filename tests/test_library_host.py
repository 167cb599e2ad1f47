"""CPU-only checks of the built C-ABI library: it loads, exports every symbol the
header declares, rejects bad arguments before touching a GPU, and its host-side
launch planning (tiles, slots, chunks, workspace) is self-consistent."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_1706_08359_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    header = open(os.path.join(ROOT, "include", "gbdt_hist.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(gbdt_[a-z_]+)\s*\(", header))
    assert declared, "no declarations found"
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror():
    assert B.gbdt_strerror(0) == "ok"
    assert "invalid" in B.gbdt_strerror(-1)
    assert "unknown" in B.gbdt_strerror(-99)


def test_argument_errors_are_rejected_before_any_gpu_work():
    lib = B.load()
    EINVAL, EUNSUP = -1, -2
    assert lib.gbdt_bins_packed_bytes(10, 0, 64) == 0
    assert lib.gbdt_bins_packed_bytes(10, 5, 1) == 0
    assert lib.gbdt_bins_packed_bytes(10, 5, 257) == 0
    assert lib.gbdt_bins_packed_bytes(-1, 5, 64) == 0
    assert lib.gbdt_workspace_bytes(10, 5, 300) == 0
    one = ctypes.c_void_p(256)    # never dereferenced: all calls below fail validation first
    assert lib.gbdt_bins_pack(None, 10, 5, 64, one, None) == EINVAL
    assert lib.gbdt_bins_pack(one, 10, 5, 64, None, None) == EINVAL
    assert lib.gbdt_bins_pack(one, 10, 5, 64, ctypes.c_void_p(260), None) == EINVAL   # misaligned
    assert lib.gbdt_bins_pack(one, 10, 5, 1, one, None) == EINVAL
    assert lib.gbdt_bins_pack(one, 1 << 31, 5, 64, one, None) == EUNSUP
    assert lib.gbdt_hist_build(one, 10, 5, 64, None, 5, one, one, None, None) == EINVAL
    assert lib.gbdt_hist_build(None, 10, 5, 64, None, 5, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 10, 5, 64, None, 5, None, one, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 10, 5, 64, None, 5, one, None, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 10, 5, 64, None, 11, one, one, one, None) == EINVAL   # root leaf > n_rows
    assert lib.gbdt_hist_build(one, 10, 5, 64, None, -1, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 10, 5, 0, None, 5, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 10, 5, 257, None, 5, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 10, 0, 64, None, 5, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build(one, 1 << 31, 5, 64, None, 5, one, one, one, None) == EUNSUP
    assert lib.gbdt_hist_subtract(None, one, one, 5, 64, None) == EINVAL
    assert lib.gbdt_hist_subtract(one, None, one, 5, 64, None) == EINVAL
    assert lib.gbdt_hist_subtract(one, one, None, 5, 64, None) == EINVAL
    assert lib.gbdt_hist_subtract(one, one, one, 5, 1, None) == EINVAL
    assert lib.gbdt_best_split(None, 1.0, 0.0, one, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split(one, 1.0, 0.0, None, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split(one, -1.0, 0.0, one, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split(one, float("nan"), 0.0, one, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split(one, 1.0, 0.0, one, 0, 64, None) == EINVAL
    # batched build: the offsets are a HOST array, validated before anything else happens
    offs = lambda *v: (ctypes.c_int64 * len(v))(*v)
    B.load()
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, offs(0, 3, 7), -1, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, offs(0, 3, 7), 0, one, one, one, None) == 0
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, None, 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, offs(0, 3, 7), 2, one, one, None, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, offs(0, 7, 3), 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, offs(-1, 3, 7), 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, None, offs(0, 3, 7), 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(None, 10, 5, 64, one, offs(0, 3, 7), 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 64, one, offs(0, 3, 7), 2, None, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 10, 5, 1, one, offs(0, 3, 7), 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 0, 5, 64, one, offs(0, 3, 7), 2, one, one, one, None) == EINVAL
    assert lib.gbdt_hist_build_batch(one, 1 << 31, 5, 64, one, offs(0, 3, 7), 2, one, one, one, None) == EUNSUP
    assert lib.gbdt_hist_build_batch_workspace_bytes(5, 1, 4) == 0
    assert lib.gbdt_hist_build_batch_workspace_bytes(5, 64, -1) == 0
    assert lib.gbdt_best_split_batch(one, -1, 1.0, 0.0, one, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split_batch(one, 0, 1.0, 0.0, one, 5, 64, None) == 0
    assert lib.gbdt_best_split_batch(None, 2, 1.0, 0.0, one, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split_batch(one, 2, 1.0, 0.0, None, 5, 64, None) == EINVAL
    assert lib.gbdt_best_split_batch(one, 2, -1.0, 0.0, one, 5, 64, None) == EINVAL
    assert lib.gbdt_partition_rows(None, 10, 5, 64, None, 5, one, one, one, None) == EINVAL
    assert lib.gbdt_partition_rows(one, 10, 5, 64, None, 5, None, one, one, None) == EINVAL
    assert lib.gbdt_partition_rows(one, 10, 5, 64, None, 5, one, None, one, None) == EINVAL
    assert lib.gbdt_partition_rows(one, 10, 5, 64, None, 11, one, one, one, None) == EINVAL
    assert lib.gbdt_partition_rows(one, 10, 5, 64, None, -1, one, one, one, None) == EINVAL
    assert lib.gbdt_partition_rows(one, 1 << 31, 5, 64, None, 5, one, one, one, None) == EUNSUP
    assert lib.gbdt_set_workspace(one, 0) == EINVAL
    assert lib.gbdt_set_workspace(None, 16) == EINVAL
    assert lib.gbdt_set_workspace(ctypes.c_void_p(100), 1024) == EINVAL               # misaligned
    assert lib.gbdt_set_workspace(None, 0) == 0


SHAPES = [(1, 2), (3, 16), (4, 17), (27, 63), (28, 64), (28, 255), (33, 64), (64, 64), (65, 65),
          (100, 256), (137, 255), (129, 16), (130, 16), (255, 16), (257, 16), (700, 16),
          (2000, 63), (2001, 63), (2047, 64), (968, 255)]


@pytest.mark.parametrize("n_features,n_bins", SHAPES)
def test_tile_plan_is_a_bijection_onto_slots(n_features, n_bins):
    g = B.gbdt_debug_geometry(n_features, n_bins, 1000)
    assert g["cap"] >= n_bins and g["cap"] in (16, 64, 256)
    assert g["nib"] == (1 if n_bins <= 16 else 0)
    assert g["wm"] == (32 if g["cap"] == 256 else 64) and g["wr"] in (0, 16, 32) and g["wr"] < g["wm"]
    assert g["row_bytes"] == g["n_main"] * g["wm"] + g["wr"]
    per_byte = 2 if g["nib"] else 1
    assert g["feat_bytes"] == (n_features + per_byte - 1) // per_byte
    assert g["feat_bytes"] <= g["row_bytes"] < g["feat_bytes"] + g["wm"] // 2 + 16
    # tiles, the slack the build kernels may read past them, then one byte per value column by column
    tiles = (12345 * g["row_bytes"] + 512 * 64 + 255) // 256 * 256
    assert B.gbdt_bins_packed_bytes(12345, n_features, n_bins) == tiles + n_features * ((12345 + 255) // 256 * 256)
    seen = set()
    for f in range(n_features):
        t, s = B.gbdt_debug_locate(n_features, n_bins, f)
        w = g["wm"] if t < g["n_main"] else g["wr"]
        assert 0 <= t < g["n_main"] + (1 if g["wr"] else 0) and w > 0
        assert 0 <= s < w * per_byte
        assert (t, s) not in seen
        seen.add((t, s))
    # the main tile's histogram (8-byte cells, 32 slots per page row) must fit the LDS
    # the kernel declares, and the CU
    pages = (g["wm"] * per_byte + 31) // 32
    assert pages * g["cap"] * 32 * 8 <= g["lds_bytes"] <= 160 * 1024


@pytest.mark.parametrize("n_features,n_bins", [(28, 64), (2000, 63), (28, 255), (137, 255), (700, 16), (5, 2)])
@pytest.mark.parametrize("n_leaf", [1, 63, 64, 65, 511, 512, 513, 4000, 100_003, 266_000, 10_500_000])
def test_workgroups_per_tile(n_features, n_bins, n_leaf):
    g = B.gbdt_debug_geometry(n_features, n_bins, n_leaf)
    per_byte = 2 if g["nib"] else 1
    n_epochs = (n_leaf + 511) // 512
    n_tiles = g["n_main"] + (1 if g["wr"] else 0)
    wgs, k = g["wgs"], g["unit_epochs"]
    # the grid fits the machine once; every workgroup's first unit exists
    assert wgs >= 1 and k >= 1 and wgs * n_tiles <= max(256 * 4, n_tiles)
    n_units = (n_epochs + k - 1) // k
    assert wgs <= max(n_units, 1)
    # units beyond a workgroup's first come from the tile's counter; the two epochs of
    # look-ahead across a unit's end need units of at least 3 epochs then
    assert n_units <= wgs or k >= 3
    words = 0
    for w, tiles in ((g["wm"], g["n_main"]), (g["wr"], 1 if g["wr"] else 0)):
        pages = (w * per_byte + 31) // 32
        words += tiles * wgs * 3 * g["cap"] * 32 * pages
    assert words == g["partial_words"]
    assert B.gbdt_workspace_bytes(n_leaf, n_features, n_bins) >= 4 * (g["partial_words"] + n_tiles)
    assert n_tiles * wgs < 2 ** 31


@pytest.mark.parametrize("n_features,n_bins,wg_per_cu", [(28, 255, 2), (2000, 63, 3), (700, 16, 4), (137, 255, 2), (40, 64, 3)])
def test_batched_launch_plan_covers_every_leaf_exactly(n_features, n_bins, wg_per_cu):
    """Host planning of gbdt_hist_build_batch and the block -> (leaf, tile, workgroup) mapping
    the kernel uses: every (leaf, tile, workgroup) is hit by exactly one block, empty leaves get
    none, and a leaf's workgroups (unit c, c + wgs, ...) cover each of its epochs exactly once."""
    rng = np.random.default_rng(n_features + n_bins)
    geo = B.gbdt_debug_geometry(n_features, n_bins, 1)
    n_tiles = geo["n_main"] + (1 if geo["wr"] else 0)
    for trial in range(12):
        n_leaves = int(rng.integers(1, 129))
        kind = trial % 4
        if kind == 0:
            sizes = rng.integers(0, 3000, size=n_leaves)
        elif kind == 1:
            sizes = rng.integers(0, 2, size=n_leaves) * rng.integers(1, 200_000, size=n_leaves)
        elif kind == 2:
            sizes = np.full(n_leaves, 1)
            sizes[0] = 3_000_000
        else:
            sizes = (2_000_000 * rng.dirichlet(np.ones(n_leaves))).astype(np.int64)
        offs = np.concatenate([[5], 5 + np.cumsum(sizes)])
        wgs, ue, blocks = B.gbdt_debug_batch_plan(n_features, n_bins, offs, 256, wg_per_cu)
        assert blocks.shape[0] == int(wgs.sum()) * n_tiles
        seen = set()
        for leaf, tile, wg in blocks.tolist():
            assert 0 <= leaf < n_leaves and 0 <= tile < n_tiles and 0 <= wg < wgs[leaf], (leaf, tile, wg)
            seen.add((leaf, tile, wg))
        assert len(seen) == blocks.shape[0]                      # no (leaf, tile, wg) twice
        for l in range(n_leaves):
            n_epochs = -(-int(sizes[l]) // 512)
            if n_epochs == 0:
                assert wgs[l] == 0
                continue
            # units of 4 epochs, or an even split with one longer unit per workgroup (at most 3 x 4)
            assert 1 <= wgs[l] <= n_epochs and 1 <= ue[l] <= 12
            n_units = -(-n_epochs // int(ue[l]))
            if ue[l] > 4:
                assert n_units == wgs[l]
            assert wgs[l] <= n_units                             # no workgroup without a unit
            # workgroup c takes units c, c + wgs, ...: together all units, each once
            taken = sorted(u for c in range(wgs[l]) for u in range(c, n_units, int(wgs[l])))
            assert taken == list(range(n_units))
        # the leaves share the machine: about one machine-full of workgroup columns, plus the
        # at-least-one of every leaf
        assert int(wgs.sum()) <= 256 * wg_per_cu // n_tiles + n_leaves


@pytest.mark.parametrize("n_features,n_bins", [(28, 64), (2000, 63), (137, 255), (700, 16)])
def test_wide_accumulation_doubles_the_partial_blocks(n_features, n_bins):
    """The wide mode writes two partial blocks per workgroup; the sizes the library reports for
    caller-owned scratch follow the switch (and go back with it)."""
    n_leaf = 266_000
    narrow = B.gbdt_workspace_bytes(n_leaf, n_features, n_bins)
    narrow_batch = B.gbdt_hist_build_batch_workspace_bytes(n_features, n_bins, 64)
    B.gbdt_set_wide_accumulation(True)
    try:
        wide = B.gbdt_workspace_bytes(n_leaf, n_features, n_bins)
        wide_batch = B.gbdt_hist_build_batch_workspace_bytes(n_features, n_bins, 64)
    finally:
        B.gbdt_set_wide_accumulation(False)
    assert wide >= narrow and wide_batch > narrow_batch
    assert wide_batch <= 2 * narrow_batch
    assert B.gbdt_workspace_bytes(n_leaf, n_features, n_bins) == narrow


def test_fusion_plan_is_a_valid_mixed_radix_packing():
    """Host planner of gbdt_bins_fuse: every feature sits in exactly one column, the levels of a
    column multiply to at most 64, at most 6 features share a column, the weights are the running
    products of the levels in some order of the column's features -- so that a joint value
    decodes back to every feature's bin -- and few-level features really share columns."""
    rng = np.random.default_rng(3)
    for levels in (rng.integers(2, 17, size=700), rng.integers(1, 65, size=333), np.full(40, 2), np.full(9, 64),
                   np.array([1, 1, 1, 64, 33, 2]), rng.integers(1, 5, size=1000)):
        levels = levels.astype(np.uint32)
        col, stride, n_cols = B.gbdt_debug_fusion_plan(levels)
        assert col.min() == 0 and col.max() == n_cols - 1 and len(np.unique(col)) == n_cols
        for c in range(n_cols):
            fs = np.nonzero(col == c)[0]
            assert 1 <= len(fs) <= 6
            assert int(np.prod(levels[fs].astype(np.int64))) <= 64
            order = fs[np.argsort(stride[fs], kind="stable")]
            run = 1
            for f in order:                       # weights: 1, L_a, L_a L_b, ...
                assert stride[f] == run, (c, fs, stride[fs], levels[fs])
                run *= int(levels[f])
            # decode a random joint value
            b = [int(rng.integers(0, levels[f])) for f in fs]
            v = sum(bi * int(stride[f]) for bi, f in zip(b, fs))
            assert v < 64
            assert [(v // int(stride[f])) % int(levels[f]) for f in fs] == b
        # lower bound on columns: the sum of log2(levels) in units of 6 bits
        assert n_cols >= int(np.ceil(np.log2(levels.astype(np.float64)).sum() / 6.0 - 1e-9))
    col, stride, n_cols = B.gbdt_debug_fusion_plan(np.full(40, 2, np.uint32))
    assert n_cols == 7                            # six binary features per column
    col, stride, n_cols = B.gbdt_debug_fusion_plan(np.full(9, 64, np.uint32))
    assert n_cols == 9


@pytest.mark.parametrize("n_bins", [2, 16, 63, 64, 100, 255, 256])
def test_split_search_plan_covers_every_feature_within_the_lds_budget(n_bins):
    """The work split of the split search follows the number of histograms of the launch; whatever
    it picks, the groups of all workgroups cover the features, a group fits the kernel's local
    memory budget, and a launch never has more candidates per histogram than a lone histogram
    (the scratch of gbdt_workspace_bytes is sized by that)."""
    for n_features in (1, 2, 7, 28, 137, 255, 256, 257, 700, 2000, 4000, 20000):
        lone = B.gbdt_debug_split_plan(n_features, n_bins, 1)
        for n_hists in (1, 2, 3, 8, 31, 64, 256, 1024, 32768):
            p = B.gbdt_debug_split_plan(n_features, n_bins, n_hists)
            assert p["group"] >= 1 and p["passes"] >= 1 and p["workgroups"] >= 1
            assert p["lds_bytes"] <= 48 * 1024
            assert p["group"] * p["passes"] * p["workgroups"] >= n_features
            # no workgroup without a feature
            assert p["group"] * p["passes"] * (p["workgroups"] - 1) < n_features
            assert p["workgroups"] <= lone["workgroups"]
            # the prefix sums run on one lane per (feature, statistic) of a 256-thread workgroup
            assert 3 * p["group"] <= 256


def test_partition_plan_chunks_cover_the_list():
    """Chunks of 256 * rows_per_thread positions: 8 steps, or a multiple of 16 (the kernels take
    8 or 16 steps at a time), at most 2048 chunks, every position in exactly one chunk."""
    for n in (1, 255, 256, 2047, 2048, 2049, 8192, 8193, 4_194_304, 4_194_305, 10_500_000, 11_000_000,
              67_108_864, 2**31 - 1, 2**32 - 1):
        p = B.gbdt_debug_partition_plan(n)
        r, c = p["rows_per_thread"], p["chunks"]
        assert r == 8 or r % 16 == 0
        assert r & (r - 1) == 0
        assert 1 <= c <= 2048
        assert (c - 1) * 256 * r < n <= c * 256 * r
        assert p["bytes"] == c * r * 4 * 8 + c * 4
    with pytest.raises(B.GbdtError):
        B.gbdt_debug_partition_plan(0)

"""CPU-only checks of the built C-ABI library: it loads, exports every symbol the
header declares, rejects bad arguments before touching a GPU, and its host-side
launch planning (tiles, slots, chunks, workspace) is self-consistent."""
import ctypes
import os
import re

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
    assert B.gbdt_bins_packed_bytes(12345, n_features, n_bins) == 12345 * g["row_bytes"] + 512 * 64
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

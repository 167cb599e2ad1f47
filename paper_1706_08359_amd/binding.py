"""Thin ctypes binding of libgbdt_hist (include/gbdt_hist.h): argument marshalling only.

Every function has the name and argument order of its C counterpart, takes torch
CUDA tensors (used purely as device memory) and launches on torch's current
stream unless `stream` is given.  There is no CPU fallback: if the library has not
been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
import weakref

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# GBDT_HIST_LIB: path of another build of the library (tuning experiments); default in-tree
LIB_PATH = os.environ.get("GBDT_HIST_LIB") or os.path.join(_HERE, "libgbdt_hist.so")

EXPORTS = [
    "gbdt_bins_packed_bytes", "gbdt_bins_pack", "gbdt_hist_build", "gbdt_hist_subtract",
    "gbdt_best_split", "gbdt_workspace_bytes", "gbdt_set_workspace", "gbdt_strerror",
    "gbdt_last_hip_error", "gbdt_debug_geometry", "gbdt_debug_locate",
    "gbdt_profile_enable", "gbdt_profile_collect", "gbdt_debug_occupancy", "gbdt_debug_split_plan",
    "gbdt_debug_partition_plan",
    "gbdt_calibration_copy", "gbdt_set_deterministic", "gbdt_partition_rows",
    "gbdt_hist_build_batch", "gbdt_hist_build_batch_workspace_bytes", "gbdt_best_split_batch",
    "gbdt_debug_batch_plan", "gbdt_grow_tree", "gbdt_grow_tree_scratch_bytes",
    "gbdt_partition_rows_batch", "gbdt_grow_tree_depthwise", "gbdt_grow_tree_depthwise_scratch_bytes",
    "gbdt_set_wide_accumulation", "gbdt_profile_durations", "gbdt_reset",
    "gbdt_hist_build_noalloc", "gbdt_hist_build_noalloc_max_partial_bytes",
    "gbdt_bins_fused_bytes", "gbdt_bins_fuse", "gbdt_bins_unfuse", "gbdt_debug_fusion_plan",
]

# numpy views of the two C structs
BIN_DTYPE = np.dtype([("grad", "<f4"), ("hess", "<f4"), ("count", "<u4")])
SPLIT_DTYPE = np.dtype([("feature", "<i4"), ("bin", "<i4"), ("gain", "<f4"),
                        ("left_grad", "<f4"), ("left_hess", "<f4"), ("left_count", "<u4"),
                        ("right_grad", "<f4"), ("right_hess", "<f4"), ("right_count", "<u4")])

NODE_DTYPE = np.dtype([("parent", "<i4"), ("left", "<i4"), ("right", "<i4"), ("feature", "<i4"),
                       ("bin", "<i4"), ("gain", "<f4"), ("sum_grad", "<f4"), ("sum_hess", "<f4"),
                       ("count", "<u4"), ("reserved", "<i4"), ("row_begin", "<i8")])

_lib = None


class GbdtError(RuntimeError):
    pass


def load():
    """Load the built library; raises if it is missing (build it with
    `python -m paper_1706_08359_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise GbdtError("libgbdt_hist.so is not built: run `python -m paper_1706_08359_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    lib.gbdt_bins_packed_bytes.restype = c.c_size_t
    lib.gbdt_bins_packed_bytes.argtypes = [c.c_int64, c.c_int32, c.c_int32]
    lib.gbdt_bins_pack.restype = c.c_int
    lib.gbdt_bins_pack.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p]
    lib.gbdt_bins_fused_bytes.restype = c.c_size_t
    lib.gbdt_bins_fused_bytes.argtypes = [c.c_int64, c.c_int32, c.c_int32]
    lib.gbdt_bins_fuse.restype = c.c_int
    lib.gbdt_bins_fuse.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p,
                                   c.c_size_t, c.POINTER(c.c_int32), c.c_void_p]
    lib.gbdt_bins_unfuse.restype = c.c_int
    lib.gbdt_bins_unfuse.argtypes = [c.c_void_p]
    lib.gbdt_hist_build.restype = c.c_int
    lib.gbdt_hist_build.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p,
                                    c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.gbdt_hist_build_noalloc.restype = c.c_int
    lib.gbdt_hist_build_noalloc.argtypes = lib.gbdt_hist_build.argtypes
    lib.gbdt_hist_build_noalloc_max_partial_bytes.restype = c.c_size_t
    lib.gbdt_hist_build_noalloc_max_partial_bytes.argtypes = []
    lib.gbdt_profile_durations.restype = c.c_int
    lib.gbdt_profile_durations.argtypes = [c.POINTER(c.c_double), c.c_int64, c.POINTER(c.c_int64)]
    lib.gbdt_reset.restype = c.c_int
    lib.gbdt_reset.argtypes = []
    lib.gbdt_hist_subtract.restype = c.c_int
    lib.gbdt_hist_subtract.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32,
                                       c.c_void_p]
    lib.gbdt_best_split.restype = c.c_int
    lib.gbdt_best_split.argtypes = [c.c_void_p, c.c_float, c.c_float, c.c_void_p, c.c_int32,
                                    c.c_int32, c.c_void_p]
    lib.gbdt_hist_build_batch.restype = c.c_int
    lib.gbdt_hist_build_batch.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p,
                                          c.POINTER(c.c_int64), c.c_int32, c.c_void_p, c.c_void_p,
                                          c.c_void_p, c.c_void_p]
    lib.gbdt_hist_build_batch_workspace_bytes.restype = c.c_size_t
    lib.gbdt_hist_build_batch_workspace_bytes.argtypes = [c.c_int32, c.c_int32, c.c_int32]
    lib.gbdt_best_split_batch.restype = c.c_int
    lib.gbdt_best_split_batch.argtypes = [c.c_void_p, c.c_int32, c.c_float, c.c_float, c.c_void_p,
                                          c.c_int32, c.c_int32, c.c_void_p]
    lib.gbdt_partition_rows_batch.restype = c.c_int
    lib.gbdt_partition_rows_batch.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p,
                                              c.POINTER(c.c_int64), c.c_int32, c.c_void_p, c.c_void_p,
                                              c.c_void_p, c.c_void_p]
    lib.gbdt_grow_tree.restype = c.c_int
    lib.gbdt_grow_tree.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p, c.c_void_p,
                                   c.c_int32, c.c_float, c.c_float, c.c_float, c.c_void_p, c.c_size_t,
                                   c.c_void_p, c.POINTER(c.c_int32), c.c_void_p, c.c_void_p]
    lib.gbdt_grow_tree_depthwise.restype = c.c_int
    lib.gbdt_grow_tree_depthwise.argtypes = lib.gbdt_grow_tree.argtypes
    lib.gbdt_grow_tree_depthwise_scratch_bytes.restype = c.c_size_t
    lib.gbdt_grow_tree_depthwise_scratch_bytes.argtypes = [c.c_int64, c.c_int32, c.c_int32, c.c_int32]
    lib.gbdt_grow_tree_scratch_bytes.restype = c.c_size_t
    lib.gbdt_grow_tree_scratch_bytes.argtypes = [c.c_int64, c.c_int32, c.c_int32, c.c_int32]
    lib.gbdt_partition_rows.restype = c.c_int
    lib.gbdt_partition_rows.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32, c.c_void_p,
                                        c.c_int64, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
    lib.gbdt_workspace_bytes.restype = c.c_size_t
    lib.gbdt_workspace_bytes.argtypes = [c.c_int64, c.c_int32, c.c_int32]
    lib.gbdt_set_workspace.restype = c.c_int
    lib.gbdt_set_workspace.argtypes = [c.c_void_p, c.c_size_t]
    lib.gbdt_strerror.restype = c.c_char_p
    lib.gbdt_strerror.argtypes = [c.c_int]
    lib.gbdt_last_hip_error.restype = c.c_char_p
    lib.gbdt_last_hip_error.argtypes = []
    lib.gbdt_debug_geometry.restype = c.c_int
    lib.gbdt_debug_geometry.argtypes = [c.c_int32, c.c_int32, c.c_int64, c.c_int32,
                                        c.POINTER(c.c_int64), c.c_int32]
    lib.gbdt_debug_locate.restype = c.c_int
    lib.gbdt_debug_locate.argtypes = [c.c_int32, c.c_int32, c.c_int32, c.POINTER(c.c_int32),
                                      c.POINTER(c.c_int32)]
    lib.gbdt_profile_enable.restype = c.c_int
    lib.gbdt_profile_enable.argtypes = [c.c_int]
    lib.gbdt_profile_collect.restype = c.c_int
    lib.gbdt_profile_collect.argtypes = [c.POINTER(c.c_double), c.POINTER(c.c_int64)]
    lib.gbdt_set_deterministic.restype = c.c_int
    lib.gbdt_set_deterministic.argtypes = [c.c_int]
    lib.gbdt_set_wide_accumulation.restype = c.c_int
    lib.gbdt_set_wide_accumulation.argtypes = [c.c_int]
    lib.gbdt_calibration_copy.restype = c.c_int
    lib.gbdt_calibration_copy.argtypes = [c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        lib = load()
        msg = lib.gbdt_strerror(rc).decode()
        hip = lib.gbdt_last_hip_error().decode()
        raise GbdtError(f"{what}: {msg} ({rc})" + (f" [{hip}]" if hip and rc in (-2, -3, -4) else ""))


def _stream(stream) -> int:
    if stream is None:
        return int(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, torch.cuda.Stream):
        return int(stream.cuda_stream)
    return int(stream)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous CUDA tensor of dtype {dtype}")
    return t.data_ptr()


def gbdt_strerror(code: int) -> str:
    return load().gbdt_strerror(int(code)).decode()


def gbdt_bins_packed_bytes(n_rows: int, n_features: int, n_bins: int) -> int:
    return int(load().gbdt_bins_packed_bytes(n_rows, n_features, n_bins))


def gbdt_workspace_bytes(n_rows: int, n_features: int, n_bins: int) -> int:
    return int(load().gbdt_workspace_bytes(n_rows, n_features, n_bins))


def gbdt_set_workspace(buf) -> None:
    """buf: uint8 CUDA tensor (kept alive by the caller) or None."""
    if buf is None:
        _check(load().gbdt_set_workspace(None, 0), "gbdt_set_workspace")
    else:
        _check(load().gbdt_set_workspace(_dev(buf, torch.uint8, "buf"), buf.numel()),
               "gbdt_set_workspace")


FUSE_MIN_ROWS = 8192   # gbdt_bins_pack tries gbdt_bins_fuse from this many rows on (fuse=None)


def gbdt_bins_fused_bytes(n_rows: int, n_features: int, n_bins: int) -> int:
    return int(load().gbdt_bins_fused_bytes(n_rows, n_features, n_bins))


def gbdt_bins_fuse(bins_rowmajor: torch.Tensor, n_bins: int, packed: torch.Tensor, stream=None):
    """Makes the fused copy of few-level features for `packed` when it pays.  Returns (n_columns,
    fused tensor or None); the tensor is also attached to `packed` (attribute `gbdt_fused`) so
    that it lives as long as the packed buffer does."""
    lib = load()
    n_rows, n_features = bins_rowmajor.shape
    nbytes = int(lib.gbdt_bins_fused_bytes(n_rows, n_features, n_bins))
    packed.gbdt_fused = None
    if nbytes == 0:
        _check(lib.gbdt_bins_unfuse(_dev(packed, torch.uint8, "packed")), "gbdt_bins_unfuse")
        return 0, None
    fused = torch.empty(nbytes, dtype=torch.uint8, device=bins_rowmajor.device)
    n_cols = ctypes.c_int32(0)
    _check(lib.gbdt_bins_fuse(_dev(bins_rowmajor, torch.uint8, "bins_rowmajor"), n_rows, n_features, n_bins,
                              _dev(packed, torch.uint8, "packed"), _dev(fused, torch.uint8, "fused"), nbytes,
                              ctypes.byref(n_cols), _stream(stream)), "gbdt_bins_fuse")
    if n_cols.value == 0:
        return 0, None
    packed.gbdt_fused = fused
    # the library remembers the fused copy by the packed buffer's address: forget it when the
    # buffer goes away, so that the address can be reused for something else
    weakref.finalize(packed, lib.gbdt_bins_unfuse, packed.data_ptr())
    return n_cols.value, fused


def gbdt_bins_unfuse(packed: torch.Tensor) -> None:
    _check(load().gbdt_bins_unfuse(_dev(packed, torch.uint8, "packed")), "gbdt_bins_unfuse")
    packed.gbdt_fused = None


def gbdt_bins_pack(bins_rowmajor: torch.Tensor, n_bins: int, packed_out=None, stream=None, fuse=None):
    """bins_rowmajor: uint8 [n_rows, n_features] on the GPU.  Returns the packed uint8 buffer.
    fuse: True / False: also call gbdt_bins_fuse (which waits for the stream) or not; None: from
    FUSE_MIN_ROWS rows on."""
    src = _dev(bins_rowmajor, torch.uint8, "bins_rowmajor")
    n_rows, n_features = bins_rowmajor.shape
    nbytes = gbdt_bins_packed_bytes(n_rows, n_features, n_bins)
    if nbytes == 0 and n_rows != 0:
        raise GbdtError("gbdt_bins_packed_bytes: invalid argument")
    if packed_out is None:
        packed_out = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=bins_rowmajor.device)
    elif packed_out.numel() < nbytes:
        raise GbdtError("packed_out too small")
    _check(load().gbdt_bins_pack(src, n_rows, n_features, n_bins,
                                 _dev(packed_out, torch.uint8, "packed_out"), _stream(stream)),
           "gbdt_bins_pack")
    if fuse is None:
        fuse = n_rows >= FUSE_MIN_ROWS
    if fuse and n_rows > 0:
        gbdt_bins_fuse(bins_rowmajor, n_bins, packed_out, stream=stream)
    return packed_out


def gbdt_hist_build(bin_matrix, n_rows, n_features, n_bins, leaf_row_idx, n_leaf_rows, grad, hess,
                    hist_out=None, stream=None, _entry="gbdt_hist_build"):
    """Returns hist_out: float32 CUDA tensor [n_features, n_bins, 3] holding gbdt_bin_t records
    (the third word of each record is the uint32 count; see hist_to_numpy)."""
    if hist_out is None:
        hist_out = torch.empty((n_features, n_bins, 3), dtype=torch.float32, device=grad.device)
    idx_p = None if leaf_row_idx is None else _dev(leaf_row_idx, torch.int32, "leaf_row_idx")
    if leaf_row_idx is not None and leaf_row_idx.numel() < n_leaf_rows:
        raise GbdtError("leaf_row_idx shorter than n_leaf_rows")
    if grad.numel() < n_rows or hess.numel() < n_rows:
        raise GbdtError("grad/hess shorter than n_rows")
    if bin_matrix.numel() < gbdt_bins_packed_bytes(n_rows, n_features, n_bins):
        raise GbdtError("bin_matrix smaller than the packed layout of this shape")
    if hist_out.numel() < n_features * n_bins * 3:
        raise GbdtError("hist_out too small")
    _check(getattr(load(), _entry)(_dev(bin_matrix, torch.uint8, "bin_matrix"), n_rows, n_features,
                                   n_bins, idx_p, n_leaf_rows, _dev(grad, torch.float32, "grad"),
                                   _dev(hess, torch.float32, "hess"),
                                   _dev(hist_out, torch.float32, "hist_out"), _stream(stream)),
           _entry)
    return hist_out


def gbdt_hist_build_noalloc(bin_matrix, n_rows, n_features, n_bins, leaf_row_idx, n_leaf_rows, grad, hess,
                            hist_out, stream=None):
    """gbdt_hist_build through the entry point that allocates nothing; hist_out is required."""
    return gbdt_hist_build(bin_matrix, n_rows, n_features, n_bins, leaf_row_idx, n_leaf_rows, grad, hess,
                           hist_out=hist_out, stream=stream, _entry="gbdt_hist_build_noalloc")


def gbdt_hist_build_noalloc_max_partial_bytes() -> int:
    return int(load().gbdt_hist_build_noalloc_max_partial_bytes())


def gbdt_reset() -> None:
    _check(load().gbdt_reset(), "gbdt_reset")


def gbdt_hist_build_batch(bin_matrix, n_rows, n_features, n_bins, row_idx, leaf_offsets, grad, hess,
                          hist_out=None, stream=None):
    """leaf_offsets: host sequence of n_leaves + 1 ints into row_idx (int32 CUDA tensor).
    Returns hist_out: float32 CUDA tensor [n_leaves, n_features, n_bins, 3]."""
    offs = [int(o) for o in leaf_offsets]
    n_leaves = len(offs) - 1
    if n_leaves < 0:
        raise GbdtError("leaf_offsets: need n_leaves + 1 entries")
    if hist_out is None:
        hist_out = torch.empty((n_leaves, n_features, n_bins, 3), dtype=torch.float32, device=grad.device)
    elif hist_out.numel() < n_leaves * n_features * n_bins * 3:
        raise GbdtError("hist_out too small")
    idx_p = None if row_idx is None else _dev(row_idx, torch.int32, "row_idx")
    if row_idx is not None and offs and row_idx.numel() < offs[-1]:
        raise GbdtError("row_idx shorter than leaf_offsets[-1]")
    if grad.numel() < n_rows or hess.numel() < n_rows:
        raise GbdtError("grad/hess shorter than n_rows")
    if bin_matrix.numel() < gbdt_bins_packed_bytes(n_rows, n_features, n_bins):
        raise GbdtError("bin_matrix smaller than the packed layout of this shape")
    arr = (ctypes.c_int64 * (n_leaves + 1))(*offs)
    _check(load().gbdt_hist_build_batch(_dev(bin_matrix, torch.uint8, "bin_matrix"), n_rows, n_features,
                                        n_bins, idx_p, arr, n_leaves, _dev(grad, torch.float32, "grad"),
                                        _dev(hess, torch.float32, "hess"),
                                        _dev(hist_out, torch.float32, "hist_out"), _stream(stream)),
           "gbdt_hist_build_batch")
    return hist_out


def gbdt_hist_build_batch_workspace_bytes(n_features: int, n_bins: int, n_leaves: int) -> int:
    return int(load().gbdt_hist_build_batch_workspace_bytes(n_features, n_bins, n_leaves))


def gbdt_best_split_batch(hists, lam, min_child_hess, splits_out=None, stream=None):
    """hists: float32 CUDA tensor [n_hists, n_features, n_bins, 3].  Returns splits_out: int32
    CUDA tensor [n_hists, 9], one gbdt_split_t per histogram."""
    n_hists, n_features, n_bins = hists.shape[0], hists.shape[1], hists.shape[2]
    if splits_out is None:
        splits_out = torch.empty((n_hists, 9), dtype=torch.int32, device=hists.device)
    elif splits_out.numel() < n_hists * 9:
        raise GbdtError("splits_out too small")
    _check(load().gbdt_best_split_batch(_dev(hists, torch.float32, "hists"), n_hists, float(lam),
                                        float(min_child_hess), _dev(splits_out, torch.int32, "splits_out"),
                                        n_features, n_bins, _stream(stream)), "gbdt_best_split_batch")
    return splits_out


def gbdt_hist_subtract(parent, child, sibling_out=None, stream=None):
    n_features, n_bins = parent.shape[0], parent.shape[1]
    if child.shape != parent.shape:
        raise GbdtError("parent/child shape mismatch")
    if sibling_out is None:
        sibling_out = torch.empty_like(parent)
    _check(load().gbdt_hist_subtract(_dev(parent, torch.float32, "parent"),
                                     _dev(child, torch.float32, "child"),
                                     _dev(sibling_out, torch.float32, "sibling_out"), n_features,
                                     n_bins, _stream(stream)), "gbdt_hist_subtract")
    return sibling_out


def gbdt_best_split(hist, lam, min_child_hess, split_out=None, stream=None):
    """Returns split_out: int32 CUDA tensor [9] holding one gbdt_split_t (see split_to_dict)."""
    n_features, n_bins = hist.shape[0], hist.shape[1]
    if split_out is None:
        split_out = torch.empty(9, dtype=torch.int32, device=hist.device)
    _check(load().gbdt_best_split(_dev(hist, torch.float32, "hist"), float(lam),
                                  float(min_child_hess), _dev(split_out, torch.int32, "split_out"),
                                  n_features, n_bins, _stream(stream)), "gbdt_best_split")
    return split_out


def gbdt_partition_rows(bin_matrix, n_rows, n_features, n_bins, leaf_row_idx, n_leaf_rows, split,
                        children_out=None, n_left_out=None, stream=None):
    """split: int32 CUDA tensor [9] holding one gbdt_split_t (as gbdt_best_split returns it).
    Returns (children_out int32 [n_leaf_rows]: left rows then right rows, n_left_out int64 [1])."""
    idx_p = None if leaf_row_idx is None else _dev(leaf_row_idx, torch.int32, "leaf_row_idx")
    if leaf_row_idx is not None and leaf_row_idx.numel() < n_leaf_rows:
        raise GbdtError("leaf_row_idx shorter than n_leaf_rows")
    if bin_matrix.numel() < gbdt_bins_packed_bytes(n_rows, n_features, n_bins):
        raise GbdtError("bin_matrix smaller than the packed layout of this shape")
    if split.numel() < 9:
        raise GbdtError("split: expected one gbdt_split_t (9 words)")
    if children_out is None:
        children_out = torch.empty(max(n_leaf_rows, 1), dtype=torch.int32, device=bin_matrix.device)
    elif children_out.numel() < n_leaf_rows:
        raise GbdtError("children_out too small")
    if n_left_out is None:
        n_left_out = torch.empty(1, dtype=torch.int64, device=bin_matrix.device)
    _check(load().gbdt_partition_rows(_dev(bin_matrix, torch.uint8, "bin_matrix"), n_rows,
                                      n_features, n_bins, idx_p, n_leaf_rows,
                                      _dev(split, torch.int32, "split"),
                                      _dev(children_out, torch.int32, "children_out"),
                                      _dev(n_left_out, torch.int64, "n_left_out"),
                                      _stream(stream)), "gbdt_partition_rows")
    return children_out, n_left_out


def gbdt_partition_rows_batch(bin_matrix, n_rows, n_features, n_bins, row_idx, leaf_offsets, splits,
                              children_out=None, n_left_out=None, stream=None):
    """splits: int32 CUDA tensor [n_leaves, 9].  Returns (children_out int32 like row_idx,
    n_left_out int64 [n_leaves])."""
    offs = [int(o) for o in leaf_offsets]
    n_leaves = len(offs) - 1
    if splits.numel() < 9 * n_leaves:
        raise GbdtError("splits: expected one gbdt_split_t per leaf")
    if row_idx.numel() < offs[-1]:
        raise GbdtError("row_idx shorter than leaf_offsets[-1]")
    if bin_matrix.numel() < gbdt_bins_packed_bytes(n_rows, n_features, n_bins):
        raise GbdtError("bin_matrix smaller than the packed layout of this shape")
    if children_out is None:
        children_out = torch.empty_like(row_idx)
    elif children_out.numel() < offs[-1]:
        raise GbdtError("children_out too small")
    if n_left_out is None:
        n_left_out = torch.empty(max(n_leaves, 1), dtype=torch.int64, device=row_idx.device)
    arr = (ctypes.c_int64 * (n_leaves + 1))(*offs)
    _check(load().gbdt_partition_rows_batch(_dev(bin_matrix, torch.uint8, "bin_matrix"), n_rows, n_features,
                                            n_bins, _dev(row_idx, torch.int32, "row_idx"), arr, n_leaves,
                                            _dev(splits, torch.int32, "splits"),
                                            _dev(children_out, torch.int32, "children_out"),
                                            _dev(n_left_out, torch.int64, "n_left_out"), _stream(stream)),
           "gbdt_partition_rows_batch")
    return children_out, n_left_out


def gbdt_grow_tree_scratch_bytes(n_rows: int, n_features: int, n_bins: int, max_leaves: int) -> int:
    return int(load().gbdt_grow_tree_scratch_bytes(n_rows, n_features, n_bins, max_leaves))


def gbdt_grow_tree(bin_matrix, n_rows, n_features, n_bins, grad, hess, max_leaves, lam, min_child_hess,
                   min_split_gain=0.0, scratch=None, row_order_out=None, want_rows=True, stream=None):
    """Returns (nodes, row_order_out, scratch): nodes is a numpy structured array (NODE_DTYPE) of
    the nodes written; row_order_out an int32 CUDA tensor [n_rows] (None with want_rows=False);
    scratch the uint8 CUDA tensor used (pass it back in to avoid reallocating).  Waits for the stream."""
    need = gbdt_grow_tree_scratch_bytes(n_rows, n_features, n_bins, max_leaves)
    if need == 0:
        raise GbdtError("gbdt_grow_tree_scratch_bytes: invalid argument")
    if scratch is None or scratch.numel() < need:
        scratch = torch.empty(need, dtype=torch.uint8, device=grad.device)
    if grad.numel() < n_rows or hess.numel() < n_rows:
        raise GbdtError("grad/hess shorter than n_rows")
    if bin_matrix.numel() < gbdt_bins_packed_bytes(n_rows, n_features, n_bins):
        raise GbdtError("bin_matrix smaller than the packed layout of this shape")
    if want_rows and row_order_out is None:
        row_order_out = torch.empty(max(n_rows, 1), dtype=torch.int32, device=grad.device)
    nodes = np.zeros(2 * max_leaves - 1, dtype=NODE_DTYPE)
    n_nodes = ctypes.c_int32(0)
    _check(load().gbdt_grow_tree(_dev(bin_matrix, torch.uint8, "bin_matrix"), n_rows, n_features, n_bins,
                                 _dev(grad, torch.float32, "grad"), _dev(hess, torch.float32, "hess"),
                                 max_leaves, float(lam), float(min_child_hess), float(min_split_gain),
                                 _dev(scratch, torch.uint8, "scratch"), scratch.numel(),
                                 nodes.ctypes.data, ctypes.byref(n_nodes),
                                 None if row_order_out is None else _dev(row_order_out, torch.int32, "row_order_out"),
                                 _stream(stream)), "gbdt_grow_tree")
    return nodes[:n_nodes.value], row_order_out, scratch


def gbdt_grow_tree_depthwise(bin_matrix, n_rows, n_features, n_bins, grad, hess, max_depth, lam,
                             min_child_hess, min_split_gain=0.0, scratch=None, row_order_out=None,
                             want_rows=True, stream=None):
    """Level-wise growth to max_depth.  Returns (nodes, row_order_out, scratch) as gbdt_grow_tree."""
    lib = load()
    need = int(lib.gbdt_grow_tree_depthwise_scratch_bytes(n_rows, n_features, n_bins, max_depth))
    if need == 0:
        raise GbdtError("gbdt_grow_tree_depthwise_scratch_bytes: invalid argument")
    if scratch is None or scratch.numel() < need:
        scratch = torch.empty(need, dtype=torch.uint8, device=grad.device)
    if grad.numel() < n_rows or hess.numel() < n_rows:
        raise GbdtError("grad/hess shorter than n_rows")
    if bin_matrix.numel() < gbdt_bins_packed_bytes(n_rows, n_features, n_bins):
        raise GbdtError("bin_matrix smaller than the packed layout of this shape")
    if want_rows and row_order_out is None:
        row_order_out = torch.empty(max(n_rows, 1), dtype=torch.int32, device=grad.device)
    nodes = np.zeros(2 ** (max_depth + 1) - 1, dtype=NODE_DTYPE)
    n_nodes = ctypes.c_int32(0)
    _check(lib.gbdt_grow_tree_depthwise(_dev(bin_matrix, torch.uint8, "bin_matrix"), n_rows, n_features, n_bins,
                                        _dev(grad, torch.float32, "grad"), _dev(hess, torch.float32, "hess"),
                                        max_depth, float(lam), float(min_child_hess), float(min_split_gain),
                                        _dev(scratch, torch.uint8, "scratch"), scratch.numel(),
                                        nodes.ctypes.data, ctypes.byref(n_nodes),
                                        None if row_order_out is None else _dev(row_order_out, torch.int32, "row_order_out"),
                                        _stream(stream)), "gbdt_grow_tree_depthwise")
    return nodes[:n_nodes.value], row_order_out, scratch


def split_record(feature: int, bin_: int, device) -> torch.Tensor:
    """A gbdt_split_t on the device that carries only a (feature, threshold bin) pair."""
    a = np.zeros(1, dtype=SPLIT_DTYPE)
    a["feature"], a["bin"] = feature, bin_
    return torch.from_numpy(a.view(np.int32).copy()).to(device)


GEOMETRY_FIELDS = ["cap", "nib", "wm", "n_main", "wr", "row_bytes", "feat_bytes", "threads",
                   "lds_bytes", "wgs", "unit_epochs", "partial_words"]


def gbdt_debug_geometry(n_features: int, n_bins: int, n_leaf_rows: int, n_cus: int = 256) -> dict:
    out = (ctypes.c_int64 * 16)()
    _check(load().gbdt_debug_geometry(n_features, n_bins, n_leaf_rows, n_cus, out, 16),
           "gbdt_debug_geometry")
    return {k: int(out[i]) for i, k in enumerate(GEOMETRY_FIELDS)}


def gbdt_debug_batch_plan(n_features, n_bins, leaf_offsets, n_cus=256, wg_per_cu=3):
    """(leaf_wgs, leaf_unit_epochs, blocks [n_blocks, 3] = leaf, tile, workgroup) of the launch."""
    offs = [int(o) for o in leaf_offsets]
    n_leaves = len(offs) - 1
    lib = load()
    lib.gbdt_debug_batch_plan.restype = ctypes.c_int
    lib.gbdt_debug_batch_plan.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64),
                                          ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                          ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32]
    arr = (ctypes.c_int64 * (n_leaves + 1))(*offs)
    wgs = np.zeros(max(n_leaves, 1), np.int32)
    ue = np.zeros(max(n_leaves, 1), np.int32)
    n = lib.gbdt_debug_batch_plan(n_features, n_bins, arr, n_leaves, n_cus, wg_per_cu, wgs.ctypes.data,
                                  ue.ctypes.data, None, 0)
    _check(min(n, 0), "gbdt_debug_batch_plan")
    blocks = np.zeros((max(n, 1), 3), np.int32)
    n2 = lib.gbdt_debug_batch_plan(n_features, n_bins, arr, n_leaves, n_cus, wg_per_cu, wgs.ctypes.data,
                                   ue.ctypes.data, blocks.ctypes.data, n)
    _check(min(n2, 0), "gbdt_debug_batch_plan")
    return wgs[:n_leaves], ue[:n_leaves], blocks[:n]


def gbdt_debug_fusion_plan(levels):
    """(column of every feature, weight of its bin in the column's joint value, number of columns)."""
    lib = load()
    lv = np.ascontiguousarray(levels, dtype=np.uint32)
    F = lv.shape[0]
    col, stride = np.zeros(F, np.int32), np.zeros(F, np.int32)
    n = ctypes.c_int32(0)
    lib.gbdt_debug_fusion_plan.restype = ctypes.c_int
    lib.gbdt_debug_fusion_plan.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
                                           ctypes.POINTER(ctypes.c_int32)]
    _check(lib.gbdt_debug_fusion_plan(lv.ctypes.data, F, col.ctypes.data, stride.ctypes.data, ctypes.byref(n)),
           "gbdt_debug_fusion_plan")
    return col, stride, n.value


def gbdt_debug_occupancy(n_bins: int, indexed: bool) -> int:
    lib = load()
    lib.gbdt_debug_occupancy.restype = ctypes.c_int
    lib.gbdt_debug_occupancy.argtypes = [ctypes.c_int32, ctypes.c_int32]
    return int(lib.gbdt_debug_occupancy(n_bins, 1 if indexed else 0))


def gbdt_debug_split_plan(n_features: int, n_bins: int, n_hists: int) -> dict:
    lib = load()
    out = (ctypes.c_int64 * 4)()
    lib.gbdt_debug_split_plan.restype = ctypes.c_int
    lib.gbdt_debug_split_plan.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                                          ctypes.c_int32]
    _check(lib.gbdt_debug_split_plan(n_features, n_bins, n_hists, out, 4), "gbdt_debug_split_plan")
    return dict(zip(("group", "passes", "workgroups", "lds_bytes"), (int(v) for v in out)))


def gbdt_debug_partition_plan(n_leaf_rows: int) -> dict:
    lib = load()
    out = (ctypes.c_int64 * 3)()
    lib.gbdt_debug_partition_plan.restype = ctypes.c_int
    lib.gbdt_debug_partition_plan.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_int32]
    _check(lib.gbdt_debug_partition_plan(n_leaf_rows, out, 3), "gbdt_debug_partition_plan")
    return dict(zip(("rows_per_thread", "chunks", "bytes"), (int(v) for v in out)))


def gbdt_debug_locate(n_features: int, n_bins: int, feature: int):
    t, s = ctypes.c_int32(), ctypes.c_int32()
    _check(load().gbdt_debug_locate(n_features, n_bins, feature, ctypes.byref(t), ctypes.byref(s)),
           "gbdt_debug_locate")
    return t.value, s.value


def gbdt_set_deterministic(enable: bool) -> None:
    _check(load().gbdt_set_deterministic(1 if enable else 0), "gbdt_set_deterministic")


def gbdt_set_wide_accumulation(enable: bool) -> None:
    _check(load().gbdt_set_wide_accumulation(1 if enable else 0), "gbdt_set_wide_accumulation")


def gbdt_calibration_copy(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    """Plain copy kernel over two uint8 CUDA tensors of equal size (a multiple of 16 bytes)."""
    if src.numel() != dst.numel():
        raise GbdtError("src/dst size mismatch")
    _check(load().gbdt_calibration_copy(_dev(src, torch.uint8, "src"), _dev(dst, torch.uint8, "dst"),
                                        src.numel(), _stream(stream)), "gbdt_calibration_copy")


def gbdt_profile_enable(enable: bool) -> None:
    _check(load().gbdt_profile_enable(1 if enable else 0), "gbdt_profile_enable")


def gbdt_profile_collect():
    """(total build-kernel milliseconds, number of launches) since the last collect."""
    ms, n = ctypes.c_double(), ctypes.c_int64()
    _check(load().gbdt_profile_collect(ctypes.byref(ms), ctypes.byref(n)), "gbdt_profile_collect")
    return ms.value, n.value


def gbdt_profile_durations():
    """Build-kernel milliseconds of every launch recorded since the last collect, in launch order."""
    lib = load()
    cap = 1 << 16
    buf = (ctypes.c_double * cap)()
    n = ctypes.c_int64()
    _check(lib.gbdt_profile_durations(buf, cap, ctypes.byref(n)), "gbdt_profile_durations")
    return [buf[i] for i in range(min(n.value, cap))]


# ---- host-side views of results (copies to the host; synchronises) -----------------


def hist_to_numpy(hist: torch.Tensor) -> np.ndarray:
    """[..., n_features, n_bins] structured array (grad f4, hess f4, count u4)."""
    a = hist.detach().cpu().contiguous().numpy()
    return a.view(BIN_DTYPE).reshape(a.shape[:-1])


def split_to_dict(split: torch.Tensor) -> dict:
    a = split.detach().cpu().contiguous().numpy().view(SPLIT_DTYPE)[0]
    return {k: a[k].item() for k in SPLIT_DTYPE.names}


def splits_to_dicts(splits: torch.Tensor) -> list:
    """One dict per gbdt_split_t of a [n, 9] int32 tensor (one device-to-host copy)."""
    a = splits.detach().cpu().contiguous().numpy().reshape(-1, 9).view(SPLIT_DTYPE).reshape(-1)
    return [{k: r[k].item() for k in SPLIT_DTYPE.names} for r in a]

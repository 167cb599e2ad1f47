"""ctypes front end of the CPU oracle (gbdt_oracle.c) -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It knows nothing about the HIP library or its device layout:
inputs are plain numpy arrays (row-major uint8 bins, float32 grad/hess,
int32 row ids), outputs are numpy structured arrays in fp64 / uint64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gbdt_oracle.c")
_LIB = os.path.join(_HERE, "libgbdt_oracle.so")

BIN_DTYPE = np.dtype([("grad", "<f8"), ("hess", "<f8"), ("count", "<u8")])

_lib = None


class _Split(ctypes.Structure):
    _fields_ = [
        ("feature", ctypes.c_int32),
        ("bin", ctypes.c_int32),
        ("gain", ctypes.c_double),
        ("left_grad", ctypes.c_double),
        ("left_hess", ctypes.c_double),
        ("left_count", ctypes.c_uint64),
        ("right_grad", ctypes.c_double),
        ("right_hess", ctypes.c_double),
        ("right_count", ctypes.c_uint64),
    ]


def build(force: bool = False) -> str:
    """Compile gbdt_oracle.c with gcc into libgbdt_oracle.so next to it."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", tmp, _SRC]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c = ctypes
        lib.oracle_hist_build.restype = c.c_int
        lib.oracle_hist_build.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int32,
                                          c.c_void_p, c.c_int64, c.c_void_p, c.c_void_p,
                                          c.c_void_p]
        lib.oracle_hist_subtract.restype = c.c_int
        lib.oracle_hist_subtract.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p,
                                             c.c_int32, c.c_int32]
        lib.oracle_best_split.restype = c.c_int
        lib.oracle_best_split.argtypes = [c.c_void_p, c.c_int32, c.c_int32, c.c_double,
                                          c.c_double, c.POINTER(_Split), c.c_void_p]
        lib.oracle_partition_rows.restype = c.c_int
        lib.oracle_partition_rows.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_void_p,
                                              c.c_int64, c.c_int32, c.c_int32, c.c_void_p,
                                              c.POINTER(c.c_int64), c.c_void_p,
                                              c.POINTER(c.c_int64)]
        lib.oracle_num_threads.restype = c.c_int
        lib.oracle_set_num_threads.argtypes = [c.c_int]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def hist_build(bins, n_bins, grad, hess, leaf_row_idx=None, n_leaf_rows=None):
    """Alg. 1 for every feature.  bins: uint8 [n_rows, n_features] C-order.

    Returns a [n_features, n_bins] array of BIN_DTYPE.
    """
    bins = np.ascontiguousarray(bins, dtype=np.uint8)
    assert bins.ndim == 2
    n_rows, n_features = bins.shape
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    hess = np.ascontiguousarray(hess, dtype=np.float32)
    assert grad.shape == (n_rows,) and hess.shape == (n_rows,)
    if leaf_row_idx is None:
        idx_p = None
        n_leaf = n_rows if n_leaf_rows is None else int(n_leaf_rows)
    else:
        leaf_row_idx = np.ascontiguousarray(leaf_row_idx, dtype=np.int32)
        idx_p = leaf_row_idx.ctypes.data
        n_leaf = leaf_row_idx.shape[0] if n_leaf_rows is None else int(n_leaf_rows)
    out = np.empty((n_features, n_bins), dtype=BIN_DTYPE)
    rc = _load().oracle_hist_build(bins.ctypes.data, n_rows, n_features, int(n_bins), idx_p,
                                   n_leaf, grad.ctypes.data, hess.ctypes.data,
                                   out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_hist_build: bad argument, row id or bin value")
    return out


def hist_subtract(parent, child):
    parent = np.ascontiguousarray(parent, dtype=BIN_DTYPE)
    child = np.ascontiguousarray(child, dtype=BIN_DTYPE)
    assert parent.shape == child.shape and parent.ndim == 2
    out = np.empty_like(parent)
    rc = _load().oracle_hist_subtract(parent.ctypes.data, child.ctypes.data, out.ctypes.data,
                                      parent.shape[0], parent.shape[1])
    if rc != 0:
        raise ValueError("oracle_hist_subtract: child count exceeds parent count")
    return out


def best_split(hist, lam, min_child_hess, return_gains=False):
    """Gain scan over bin boundaries.  Returns a dict (and the gain table)."""
    hist = np.ascontiguousarray(hist, dtype=BIN_DTYPE)
    n_features, n_bins = hist.shape
    s = _Split()
    gains = np.empty((n_features, n_bins), dtype=np.float64) if return_gains else None
    rc = _load().oracle_best_split(hist.ctypes.data, n_features, n_bins, float(lam),
                                   float(min_child_hess), ctypes.byref(s),
                                   gains.ctypes.data if return_gains else None)
    if rc != 0:
        raise ValueError("oracle_best_split: bad argument")
    d = {name: getattr(s, name) for name, _ in _Split._fields_}
    return (d, gains) if return_gains else d


def partition_rows(bins, feature, threshold_bin, leaf_row_idx=None, n_leaf_rows=None):
    """Split() of App. C.1: (left, right) int32 row-id arrays, parent order kept.

    left = rows whose bin of `feature` is <= threshold_bin.
    """
    bins = np.ascontiguousarray(bins, dtype=np.uint8)
    assert bins.ndim == 2
    n_rows, n_features = bins.shape
    if leaf_row_idx is None:
        idx_p = None
        n_leaf = n_rows if n_leaf_rows is None else int(n_leaf_rows)
    else:
        leaf_row_idx = np.ascontiguousarray(leaf_row_idx, dtype=np.int32)
        idx_p = leaf_row_idx.ctypes.data
        n_leaf = leaf_row_idx.shape[0] if n_leaf_rows is None else int(n_leaf_rows)
    left = np.empty(max(n_leaf, 1), dtype=np.int32)
    right = np.empty(max(n_leaf, 1), dtype=np.int32)
    nl, nr = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = _load().oracle_partition_rows(bins.ctypes.data, n_rows, n_features, idx_p, n_leaf,
                                       int(feature), int(threshold_bin), left.ctypes.data,
                                       ctypes.byref(nl), right.ctypes.data, ctypes.byref(nr))
    if rc != 0:
        raise ValueError("oracle_partition_rows: bad argument or row id")
    return left[:nl.value].copy(), right[:nr.value].copy()


def from_f32_hist(grad, hess, count):
    """Lift a float32/uint32 histogram (any producer) into BIN_DTYPE exactly."""
    out = np.empty(np.shape(grad), dtype=BIN_DTYPE)
    out["grad"] = np.asarray(grad, dtype=np.float64)
    out["hess"] = np.asarray(hess, dtype=np.float64)
    out["count"] = np.asarray(count, dtype=np.uint64)
    return out

"""Driver for profiler runs (rocprofv3 --kernel-trace / --pmc): packs one of the
benchmark workloads, launches its root-leaf histogram build (or, with --leaf-fraction, the
build of an index-list leaf) a few times through the C ABI and, with --copy-bytes, one plain copy kernel of that many bytes whose memory
counters calibrate the build kernel's.

    python prof_driver.py dense_wide --launches 3 --copy-bytes 800000000
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload", nargs="?", default="dense_wide")
    ap.add_argument("--launches", type=int, default=3)
    ap.add_argument("--copy-bytes", type=int, default=0)
    ap.add_argument("--leaf-fraction", type=float, default=1.0,
                    help="below 1: build an index-list leaf of this fraction of the rows (random "
                         "permutation, truncated, sorted: the leaf recipe of App. C.2) instead of the root")
    args = ap.parse_args()

    import torch
    import bench
    from paper_1706_08359_amd import binding as B

    dev = torch.device("cuda:0")
    w = bench.make_workload(args.workload, dev)
    packed = B.gbdt_bins_pack(w.bins, w.n_bins)
    hist = None
    leaf, n_leaf = None, w.n_rows
    if args.leaf_fraction < 1.0:
        from paper_1706_08359_amd import synth
        gen = torch.Generator(device=dev)
        gen.manual_seed(17)
        leaf = synth.leaf_by_truncated_permutation(w.n_rows, args.leaf_fraction, gen, dev)
        n_leaf = leaf.numel()
        print("leaf rows:", n_leaf, flush=True)
    for _ in range(args.launches):
        hist = B.gbdt_hist_build(packed, w.n_rows, w.n_features, w.n_bins, leaf, n_leaf,
                                 w.grad, w.hess, hist_out=hist)
    if args.copy_bytes:
        n = args.copy_bytes // 16 * 16
        src = torch.zeros(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        B.gbdt_calibration_copy(src, dst)
    torch.cuda.synchronize()
    print("prof_driver done:", args.workload, args.launches, "launches", flush=True)


if __name__ == "__main__":
    main()

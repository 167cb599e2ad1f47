#!/usr/bin/env python3
"""Benchmark of the histogram hot path on one MI355X.

One step = one pass of the whole path over one leaf of the workload:
  gbdt_hist_build (gather + LDS accumulate + merge)  ->  gbdt_hist_subtract
  (sibling from a resident parent)  ->  gbdt_best_split (gain scan + arg-max).
Default workload: "dense_wide" = 400,000 rows x 2,000 features, 63 bins (uint8),
root leaf (all rows), logistic grad/hess -- the configuration the headline metric
is quoted on.  Inputs are synthetic, seeded, generated on the GPU and resident in
HBM (packed once, outside the timed region) before timing starts.

Prints ONE JSON line.  `value` is feature values processed per second by whole
steps; `roofline` prices the dominant kernel (the histogram build kernel, timed
with HIP events on its own stream inside the library) against HBM peak using
ALGORITHMIC bytes; `cpu_baseline` times the CPU oracle on the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def make_workload(name: str, device):
    from paper_1706_08359_amd import synth
    if name == "dense_wide":
        return synth.config2_dense_wide(device=device, with_leaves=False)
    if name == "tiny_dense":
        return synth.config1_tiny_dense(device=device)
    if name == "dense_tall":
        return synth.config3_dense_tall(device=device)
    if name == "ranking_sparse":
        return synth.config4_ranking_sparse(device=device, fractions=(1.0,))
    if name == "categorical":
        return synth.config5_categorical(device=device)
    if name in ("paper_synthetic_k64", "paper_synthetic_k256"):
        # the matrix of the paper's kernel benchmark (App. C.2): 8,000,000 x 500 uniform random bins
        import torch
        nb = 64 if name.endswith("k64") else 256
        gen = torch.Generator(device=device)
        gen.manual_seed(100 + nb)
        bins = synth.uniform_bins(8_000_000, 500, nb, gen, device)
        grad, hess = synth.logistic_grad_hess(8_000_000, gen, device)
        return synth.Workload(name, bins, nb, grad, hess)
    raise SystemExit(f"unknown workload {name}")


def algorithmic_bytes(n_leaf, n_features, n_bins, indexed):
    """Bytes the method itself must move for one leaf build: one binned value per
    (row, feature) at 1 byte (0.5 with 4-bit bins), the row's gradient and hessian
    (+ its 4-byte row id when the leaf is an index list), and the histogram written."""
    bpv = 0.5 if n_bins <= 16 else 1.0
    return n_leaf * n_features * bpv + n_leaf * (12 if indexed else 8) + n_features * n_bins * 12


def measured_traffic(workload: str):
    """HBM bytes per build-kernel launch from the committed counter summary of this
    workload (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc runs, scaled by a copy kernel of
    known size), or None when no summary is committed."""
    import re
    path = os.path.join(ROOT, "profiles", f"hist_build_{workload}_hbm_traffic.md")
    try:
        m = re.search(r"TRAFFIC_BYTES_PER_LAUNCH\s*=\s*([0-9.eE+]+)", open(path).read())
    except OSError:
        return None
    return float(m.group(1)) if m else None


def cpu_baseline(w, budget_values=1.2e9):
    """Time the CPU oracle (as it stands) on the same leaf: build + subtract + best split."""
    import numpy as np
    from oracle import gbdt_oracle as orc
    n = w.n_rows
    per_row = w.n_features
    rows = int(min(n, max(1, budget_values // per_row)))
    bins = w.bins[:rows].cpu().numpy()
    grad = w.grad[:rows].cpu().numpy()
    hess = w.hess[:rows].cpu().numpy()
    orc.hist_build(bins[: min(rows, 2000)], w.n_bins, grad[: min(rows, 2000)], hess[: min(rows, 2000)])
    passes = []
    for _ in range(5):      # about 0.4 s of wall time each on 16 threads: ~30 s of CPU work in all
        t0 = time.perf_counter()
        h = orc.hist_build(bins, w.n_bins, grad, hess)
        sib = orc.hist_subtract(h, h)
        orc.best_split(h, w.lam, w.min_child_hess)
        passes.append(time.perf_counter() - t0)
        del sib
    dt = sorted(passes)[len(passes) // 2]
    return {
        "value": rows * per_row / dt / 1e9,
        "unit": "G feature-values/s",
        "cores": orc.num_threads(),
        "kind": "oracle",
        "sample": f"first {rows} of {n} rows x {per_row} features, root leaf, median of {len(passes)} passes "
                  f"({dt:.2f} s wall each; fp64 loops, OpenMP over features)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="dense_wide")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                         "use --gpus 1")

    import torch
    from paper_1706_08359_amd import binding as B

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    B.load()
    dev = torch.device("cuda:0")
    w = make_workload(args.workload, dev)
    n, F, nb = w.n_rows, w.n_features, w.n_bins
    packed = B.gbdt_bins_pack(w.bins, nb)
    leaf = w.leaves[0] if w.leaves else None
    n_leaf = n if leaf is None else leaf.numel()
    parent = B.gbdt_hist_build(packed, n, F, nb, None, n, w.grad, w.hess)   # resident parent
    hist = torch.empty_like(parent)
    sib = torch.empty_like(parent)
    split = torch.empty(9, dtype=torch.int32, device=dev)

    def step():
        B.gbdt_hist_build(packed, n, F, nb, leaf, n_leaf, w.grad, w.hess, hist_out=hist)
        B.gbdt_hist_subtract(parent, hist, sibling_out=sib)
        B.gbdt_best_split(hist, w.lam, w.min_child_hess, split_out=split)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.gbdt_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    B.gbdt_profile_enable(False)
    k_ms, k_n = B.gbdt_profile_collect()
    ms_per_step = dt * 1e3 / args.steps
    values = float(n_leaf) * F

    kernel_ms = k_ms / max(1, k_n)
    alg = algorithmic_bytes(n_leaf, F, nb, leaf is not None)
    achieved = alg / (kernel_ms * 1e-3) / 1e9
    out = {
        "metric": "histogram build G feature-values/s (whole step: build + subtract + best split)",
        "value": values / (ms_per_step * 1e-3) / 1e9,
        "unit": "G feature-values/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {n} rows x {F} features, {nb} bins, "
                               f"leaf of {n_leaf} rows ({'root' if leaf is None else 'indexed'})"},
        "roofline": {
            "bound": "hbm",
            "kernel": "hist_build_kernel",
            "achieved": achieved,
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS,
            "traffic": measured_traffic(w.name),
            "kernel_ms": kernel_ms,
            "algorithmic_bytes": alg,
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

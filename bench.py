#!/usr/bin/env python3
"""Benchmark of the histogram hot path on one MI355X.

One step = one pass of the whole path over one leaf of the workload:
  gbdt_hist_build (gather + LDS accumulate + merge)  ->  gbdt_hist_subtract
  (sibling from a resident parent)  ->  gbdt_best_split (gain scan + arg-max).
Default workload: "dense_wide" = 400,000 rows x 2,000 features, 63 bins (uint8),
root leaf (all rows), logistic grad/hess -- the configuration the headline metric
is quoted on.  Inputs are synthetic, seeded, generated on the GPU and resident in
HBM (packed once, outside the timed region) before timing starts.

Protocol: untimed steps for --prewarm-s seconds of wall time (the clocks the GPU
settles at under this load), --warmup untimed steps, then exactly --steps steps between
two synchronisations (`ms_per_step`, `value`); then the same number of steps with the
library's HIP events around every build kernel (recorded on the call's stream), and once
more with events around the whole gbdt_hist_build call.

Prints ONE JSON line.  `value` is feature values processed per second by whole
steps; `roofline` prices the dominant kernel (the histogram build kernel) against HBM
peak using ALGORITHMIC bytes and the MEAN of the per-launch durations (median and minimum
beside it; `build_plus_merge` prices the whole call the same way); `cpu_baseline` times
the CPU oracle on the same workload.
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


def cpu_baseline_build_rate(w, leaf, budget_values=6e8):
    """G feature values / s of the CPU oracle on a bounded sample of the leaf: median of 3 passes
    with all host threads, then of 3 passes with one thread on a tenth of the sample."""
    import statistics
    from oracle import gbdt_oracle as orc
    n_leaf = w.n_rows if leaf is None else leaf.numel()

    def timed(rows):
        if leaf is None:
            bins = w.bins[:rows].cpu().numpy()
            grad, hess, idx = w.grad[:rows].cpu().numpy(), w.hess[:rows].cpu().numpy(), None
        else:
            idx = leaf[:rows].cpu().numpy()
            hi = int(idx.max()) + 1
            bins = w.bins[:hi].cpu().numpy()
            grad, hess = w.grad[:hi].cpu().numpy(), w.hess[:hi].cpu().numpy()
        dts = []
        for _ in range(3):
            t0 = time.perf_counter()
            orc.hist_build(bins, w.n_bins, grad, hess, idx)
            dts.append(time.perf_counter() - t0)
        return rows * w.n_features / statistics.median(dts) / 1e9

    rows = int(min(n_leaf, max(1, budget_values // w.n_features)))
    threads = orc.num_threads()
    rate = timed(rows)
    rows1 = max(1, rows // 10)
    orc.set_num_threads(1)
    try:
        rate1 = timed(rows1)
    finally:
        orc.set_num_threads(threads)
    return rate, rows, threads, rate1, rows1


def _stats(ms):
    import statistics
    return {"mean": sum(ms) / len(ms), "median": statistics.median(ms), "min": min(ms), "n": len(ms)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="dense_wide")
    ap.add_argument("--prewarm-s", type=float, default=1.0,
                    help="seconds of untimed steps before the --warmup steps (clocks ramp up under load; "
                         "a handful of warm-up launches is a millisecond of GPU work)")
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

    def build():
        B.gbdt_hist_build(packed, n, F, nb, leaf, n_leaf, w.grad, w.hess, hist_out=hist)

    def step():
        build()
        B.gbdt_hist_subtract(parent, hist, sibling_out=sib)
        B.gbdt_best_split(hist, w.lam, w.min_child_hess, split_out=split)

    # untimed: the same steps for a fixed wall time, so that the timed region sees the clocks the
    # GPU settles at under this load, whatever --warmup says
    t_pre = time.perf_counter()
    while time.perf_counter() - t_pre < args.prewarm_s:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    prewarm_s = time.perf_counter() - t_pre
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: K whole steps, nothing else on the stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    values = float(n_leaf) * F

    # ---- the same K steps again with the library's events around every build kernel
    # (hipEventRecord on the call's stream right before and after the kernel): per-launch durations
    B.gbdt_profile_enable(True)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    B.gbdt_profile_enable(False)
    k = _stats(B.gbdt_profile_durations())

    # ---- and the whole gbdt_hist_build call (build kernel + reduction pass), events on the same stream
    call_ms = []
    for _ in range(args.steps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        build()
        e1.record()
        B.gbdt_hist_subtract(parent, hist, sibling_out=sib)
        B.gbdt_best_split(hist, w.lam, w.min_child_hess, split_out=split)
        call_ms.append((e0, e1))
    torch.cuda.synchronize()
    c = _stats([a.elapsed_time(b) for a, b in call_ms])

    alg = algorithmic_bytes(n_leaf, F, nb, leaf is not None)
    gbs = lambda ms: alg / (ms * 1e-3) / 1e9
    achieved = gbs(k["mean"])
    traffic = measured_traffic(w.name)
    out = {
        "metric": "histogram build G feature-values/s (whole step: build + subtract + best split)",
        "value": values / (ms_per_step * 1e-3) / 1e9,
        "unit": "G feature-values/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "prewarm_s": round(prewarm_s, 3),
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 in/out; 27-bit fixed-point accumulation in 64-bit LDS cells per 512-row epoch, "
                 "fp32 per-workgroup sums, fp64 merge",
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
            "traffic": traffic,
            "traffic_source": None if traffic is None else
                f"profiles/hist_build_{w.name}_hbm_traffic.md (committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE "
                "measurement, not re-measured by this run)",
            "kernel_ms": k["mean"],
            "kernel_ms_median": k["median"],
            "kernel_ms_min": k["min"],
            "kernel_launches": k["n"],
            "frac_at_median": gbs(k["median"]) / HBM_PEAK_GBS,
            "algorithmic_bytes": alg,
            "build_plus_merge": {
                "what": "whole gbdt_hist_build call: build kernel + reduction pass, same algorithmic bytes",
                "call_ms": c["mean"], "call_ms_median": c["median"], "call_ms_min": c["min"],
                "achieved": gbs(c["mean"]), "frac": gbs(c["mean"]) / HBM_PEAK_GBS,
            },
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

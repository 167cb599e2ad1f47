"""Measurement sweep over the five workloads and the paper's synthetic benchmark.

For every (workload, leaf) it times gbdt_hist_build on one GPU -- the build kernel alone
(HIP events recorded by the library around that kernel) and the whole call (counter
fill + build + merge, torch events) -- and prints a markdown table with feature values
per second, algorithmic GB/s and the fraction of the 8 TB/s HBM peak.  With --oracle the
CPU oracle is timed beside it on a bounded sample of the same leaf.

    python -m paper_1706_08359_amd.measure_all                # the five workloads
    python -m paper_1706_08359_amd.measure_all --depth-sweep  # App. C.2: 8,000,000 x 500, leaf = N / 2^D
    python -m paper_1706_08359_amd.measure_all --skew         # App. A.3: constant-bin features
"""
from __future__ import annotations

import argparse
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(n_leaf, n_features, n_bins, indexed):
    bpv = 0.5 if n_bins <= 16 else 1.0
    return n_leaf * n_features * bpv + n_leaf * (12 if indexed else 8) + n_features * n_bins * 12


def time_leaf(B, torch, packed, w, leaf, reps=20, warmup=3):
    """Median kernel-only and whole-call milliseconds of gbdt_hist_build for one leaf."""
    n, F, nb = w.n_rows, w.n_features, w.n_bins
    n_leaf = n if leaf is None else leaf.numel()
    hist = None
    for _ in range(warmup):
        hist = B.gbdt_hist_build(packed, n, F, nb, leaf, n_leaf, w.grad, w.hess, hist_out=hist)
    torch.cuda.synchronize()
    kernel_ms, call_ms = [], []
    for _ in range(reps):
        B.gbdt_profile_enable(True)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.gbdt_hist_build(packed, n, F, nb, leaf, n_leaf, w.grad, w.hess, hist_out=hist)
        e1.record()
        torch.cuda.synchronize()
        B.gbdt_profile_enable(False)
        ms, k = B.gbdt_profile_collect()
        kernel_ms.append(ms / max(1, k))
        call_ms.append(e0.elapsed_time(e1))
    return statistics.median(kernel_ms), min(kernel_ms), statistics.median(call_ms), hist


def oracle_rate(w, leaf, budget_values=6e8):
    """G feature values / s of the CPU oracle on a bounded sample of the leaf."""
    from oracle import gbdt_oracle as orc
    n_leaf = w.n_rows if leaf is None else leaf.numel()
    rows = int(min(n_leaf, max(1, budget_values // w.n_features)))
    if leaf is None:
        bins = w.bins[:rows].cpu().numpy()
        grad, hess, idx = w.grad[:rows].cpu().numpy(), w.hess[:rows].cpu().numpy(), None
    else:
        idx = leaf[:rows].cpu().numpy()
        hi = int(idx.max()) + 1
        bins = w.bins[:hi].cpu().numpy()
        grad, hess = w.grad[:hi].cpu().numpy(), w.hess[:hi].cpu().numpy()
    t0 = time.perf_counter()
    orc.hist_build(bins, w.n_bins, grad, hess, idx)
    dt = time.perf_counter() - t0
    return rows * w.n_features / dt / 1e9, rows, orc.num_threads()


def row(name, leaf_name, w, leaf, k_med, k_min, call_med, oracle=None):
    n_leaf = w.n_rows if leaf is None else leaf.numel()
    vals = float(n_leaf) * w.n_features
    alg = algorithmic_bytes(n_leaf, w.n_features, w.n_bins, leaf is not None)
    gbs = alg / (k_med * 1e-3) / 1e9
    cells = [name, leaf_name, f"{n_leaf:,}", f"{k_med:.4f}", f"{k_min:.4f}", f"{call_med:.4f}",
             f"{vals / (k_med * 1e-3) / 1e9:,.0f}", f"{gbs:,.0f}", f"{100 * gbs / HBM_PEAK_GBS:.1f}"]
    if oracle is not None:
        cells.append(f"{oracle[0]:.2f} ({oracle[2]} threads, {oracle[1]:,} rows)")
    print("| " + " | ".join(cells) + " |", flush=True)


def header(with_oracle):
    cols = ["workload", "leaf", "leaf rows", "kernel ms (median)", "kernel ms (min)", "call ms (median)",
            "G feature-values/s", "algorithmic GB/s", "% of 8 TB/s"]
    if with_oracle:
        cols.append("oracle G feature-values/s")
    print("| " + " | ".join(cols) + " |")
    print("|" + "---|" * len(cols), flush=True)


def five_workloads(args, torch, B, synth, dev):
    header(args.oracle)
    makers = [
        ("tiny_dense", lambda: synth.config1_tiny_dense(device=dev)),
        ("dense_wide", lambda: synth.config2_dense_wide(device=dev, with_leaves=True)),
        ("dense_tall", lambda: synth.config3_dense_tall(device=dev)),
        ("ranking_sparse", lambda: synth.config4_ranking_sparse(device=dev)),
        ("categorical", lambda: synth.config5_categorical(device=dev)),
    ]
    for name, make in makers:
        if args.only and name not in args.only:
            continue
        w = make()
        packed = B.gbdt_bins_pack(w.bins, w.n_bins)
        leaves = [("root", None)]
        extra = [l for l in w.leaves if l is not None]
        if name == "dense_wide":            # one node per depth of the random-split tree
            by_size = sorted(extra, key=lambda t: -t.numel())
            picks, last = [], w.n_rows
            for t in by_size:
                if t.numel() <= 0.62 * last:
                    picks.append(t)
                    last = t.numel()
            extra = picks[:6]
        if name in ("dense_tall", "categorical"):   # a smaller child, as in the 255-leaf tree
            extra = [torch.nonzero(w.bins[:, 3] <= w.n_bins // 3).flatten().to(torch.int32),
                     torch.nonzero(w.bins[:, 5] == 0).flatten().to(torch.int32)]
        for l in extra:
            leaves.append((f"{100.0 * l.numel() / w.n_rows:.1f} % (index list)", l))
        for leaf_name, leaf in leaves:
            k_med, k_min, call_med, _ = time_leaf(B, torch, packed, w, leaf)
            orc = oracle_rate(w, leaf) if args.oracle and leaf_name == "root" else None
            row(name, leaf_name, w, leaf, k_med, k_min, call_med, orc)
        del w, packed
        torch.cuda.empty_cache()


def depth_sweep(args, torch, B, synth, dev):
    """The paper's kernel benchmark (App. C.2): 8,000,000 x 500 uniform random bins, a leaf of
    N / 2^D rows chosen by random permutation, truncation and sorting."""
    header(False)
    for nb in (64, 256):
        gen = torch.Generator(device=dev)
        gen.manual_seed(100 + nb)
        n, F = 8_000_000, 500
        bins = synth.uniform_bins(n, F, nb, gen, dev)
        grad, hess = synth.logistic_grad_hess(n, gen, dev)
        w = synth.Workload(f"paper_synthetic_k{nb}", bins, nb, grad, hess)
        packed = B.gbdt_bins_pack(w.bins, nb)
        for depth in range(0, 11):
            leaf = None if depth == 0 else synth.leaf_by_truncated_permutation(n, 0.5 ** depth, gen, dev)
            k_med, k_min, call_med, _ = time_leaf(B, torch, packed, w, leaf)
            row(w.name, f"D = {depth}", w, leaf, k_med, k_min, call_med)
        del w, packed, bins
        torch.cuda.empty_cache()


def skew(args, torch, B, synth, dev):
    """App. A.3: every feature holds a single bin value (the paper's worst case, ~4x slower
    there) against uniform bins, same shape."""
    header(False)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    n, F = 2_000_000, 512
    for nb in (64, 256):
        grad, hess = synth.logistic_grad_hess(n, gen, dev)
        for kind in ("uniform", "constant", "60 % in bin 0"):
            if kind == "uniform":
                bins = synth.uniform_bins(n, F, nb, gen, dev)
            elif kind == "constant":
                bins = torch.full((n, F), nb // 2, dtype=torch.uint8, device=dev)
            else:
                bins = synth.uniform_bins(n, F, nb, gen, dev)
                bins[torch.rand((n, F), generator=gen, device=dev) < 0.6] = 0
            w = synth.Workload(f"skew_k{nb}", bins, nb, grad, hess)
            packed = B.gbdt_bins_pack(bins, nb)
            k_med, k_min, call_med, _ = time_leaf(B, torch, packed, w, None)
            row(w.name, kind, w, None, k_med, k_min, call_med)
            del w, packed, bins
            torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--depth-sweep", action="store_true")
    ap.add_argument("--skew", action="store_true")
    ap.add_argument("--oracle", action="store_true", help="time the CPU oracle on the root leaves")
    ap.add_argument("--only", nargs="*", default=None)
    args = ap.parse_args()

    import torch
    from paper_1706_08359_amd import binding as B
    from paper_1706_08359_amd import synth

    if not torch.cuda.is_available():
        raise SystemExit("measure_all needs a GPU")
    B.load()
    dev = torch.device("cuda:0")
    if args.depth_sweep:
        depth_sweep(args, torch, B, synth, dev)
    elif args.skew:
        skew(args, torch, B, synth, dev)
    else:
        five_workloads(args, torch, B, synth, dev)


if __name__ == "__main__":
    main()

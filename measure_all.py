"""Measurement sweep over the five workloads and the paper's synthetic benchmark.

For every (workload, leaf) it times gbdt_hist_build on one GPU -- the build kernel alone
(HIP events recorded by the library around that kernel) and the whole call (counter
fill + build + merge, torch events) -- and prints a markdown table with feature values
per second, algorithmic GB/s and the fraction of the 8 TB/s HBM peak.  With --oracle the
CPU oracle is timed beside it on a bounded sample of the same leaf.

    python measure_all.py                # the five workloads
    python measure_all.py --depth-sweep  # App. C.2: 8,000,000 x 500, leaf = N / 2^D
    python measure_all.py --skew         # App. A.3: constant-bin features
    python measure_all.py --partition    # row partition after a split (App. C.1)
    python measure_all.py --tree         # 255-leaf trees grown by gbdt_grow_tree
    python measure_all.py --batch-sweep  # a whole tree level per launch vs. leaf by leaf
"""
from __future__ import annotations

import argparse
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
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
    """The CPU oracle's build rate on a bounded sample of the leaf (bench.py's cpu_baseline leg)."""
    import bench
    return bench.cpu_baseline_build_rate(w, leaf, budget_values)


def row(name, leaf_name, w, leaf, k_med, k_min, call_med, oracle=None):
    n_leaf = w.n_rows if leaf is None else leaf.numel()
    vals = float(n_leaf) * w.n_features
    alg = algorithmic_bytes(n_leaf, w.n_features, w.n_bins, leaf is not None)
    gbs = alg / (k_med * 1e-3) / 1e9
    cells = [name, leaf_name, f"{n_leaf:,}", f"{k_med:.4f}", f"{k_min:.4f}", f"{call_med:.4f}",
             f"{vals / (k_med * 1e-3) / 1e9:,.0f}", f"{gbs:,.0f}", f"{100 * gbs / HBM_PEAK_GBS:.1f}"]
    if oracle is not None:
        cells.append(f"{oracle[0]:.2f} ({oracle[2]} threads, {oracle[1]:,} rows); "
                     f"{oracle[3]:.3f} (1 thread, {oracle[4]:,} rows)")
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


def paired_leaves(args, torch, B, synth, dev):
    """What the 128-byte cache line costs index-list leaves: the depth benchmark's matrix (8,000,000 x
    500, 64 bins: 64-byte tile rows, two per line), leaves of N / 2^D rows drawn as single random rows
    (the paper's recipe), as random ALIGNED PAIRS of rows (2i, 2i + 1: every fetched line is used in
    full) and as aligned groups of four.  Same kernel, same number of rows; build kernel time."""
    print("| D | leaf rows | random rows: kernel ms | aligned pairs: kernel ms | speed-up | aligned fours: kernel ms | "
          "speed-up |")
    print("|" + "---|" * 7, flush=True)
    n, F, nb = 8_000_000, 500, 64
    gen = torch.Generator(device=dev)
    gen.manual_seed(164)
    bins = synth.uniform_bins(n, F, nb, gen, dev)
    grad, hess = synth.logistic_grad_hess(n, gen, dev)
    w = synth.Workload("paper_synthetic_k64", bins, nb, grad, hess)
    packed = B.gbdt_bins_pack(w.bins, nb)
    for depth in range(1, 8):
        m = n >> depth
        single = synth.leaf_by_truncated_permutation(n, 0.5 ** depth, gen, dev)
        base2 = torch.sort(torch.randperm(n // 2, generator=gen, device=dev)[:m // 2]).values
        pairs = torch.stack([2 * base2, 2 * base2 + 1], 1).flatten().to(torch.int32)
        base4 = torch.sort(torch.randperm(n // 4, generator=gen, device=dev)[:m // 4]).values
        fours = (4 * base4[:, None] + torch.arange(4, device=dev)[None, :]).flatten().to(torch.int32)
        a = time_leaf(B, torch, packed, w, single)[0]
        b = time_leaf(B, torch, packed, w, pairs)[0]
        c = time_leaf(B, torch, packed, w, fours)[0]
        print(f"| {depth} | {single.numel():,} | {a:.4f} | {b:.4f} | {a / b:.2f}x | {c:.4f} | {a / c:.2f}x |", flush=True)


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
            packed = B.gbdt_bins_pack(bins, nb, fuse=False)   # the atomics' behaviour on the plain tiles
            k_med, k_min, call_med, _ = time_leaf(B, torch, packed, w, None)
            row(w.name, kind, w, None, k_med, k_min, call_med)
            del w, packed, bins
            torch.cuda.empty_cache()


WORKLOADS = {
    "tiny_dense": lambda synth, dev: synth.config1_tiny_dense(device=dev),
    "dense_wide": lambda synth, dev: synth.config2_dense_wide(device=dev, with_leaves=False),
    "dense_tall": lambda synth, dev: synth.config3_dense_tall(device=dev),
    "ranking_sparse": lambda synth, dev: synth.config4_ranking_sparse(device=dev, fractions=(1.0,)),
    "categorical": lambda synth, dev: synth.config5_categorical(device=dev),
}


def _events(torch):
    return torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)


def partition(args, torch, B, synth, dev):
    """gbdt_partition_rows (flag pass + scatter pass) on the root and on an index-list leaf of
    every workload, split on a middle feature at the middle bin.  Bytes: what the step must
    move -- row id in (if listed), one bin value from the column-major copy, row id out."""
    print("| workload | leaf | leaf rows | call ms (median) | call ms (min) | G rows/s | "
          "algorithmic MB | algorithmic GB/s |")
    print("|" + "---|" * 8, flush=True)
    for name, make in WORKLOADS.items():
        if args.only and name not in args.only:
            continue
        w = make(synth, dev)
        n, F, nb = w.n_rows, w.n_features, w.n_bins
        packed = B.gbdt_bins_pack(w.bins, nb)
        f = F // 2
        rec = B.split_record(f, nb // 2 - 1, dev)
        half = torch.nonzero(w.bins[:, 0] <= (nb - 1) // 2).flatten().to(torch.int32)
        out = torch.empty(n, dtype=torch.int32, device=dev)
        n_left = torch.empty(1, dtype=torch.int64, device=dev)
        for leaf_name, leaf in (("root", None), (f"{100.0 * half.numel() / n:.1f} % (index list)", half)):
            n_leaf = n if leaf is None else leaf.numel()
            times = []
            for rep in range(23):
                e0, e1 = _events(torch)
                e0.record()
                B.gbdt_partition_rows(packed, n, F, nb, leaf, n_leaf, rec, out, n_left)
                e1.record()
                torch.cuda.synchronize()
                if rep >= 3:
                    times.append(e0.elapsed_time(e1))
            med, mn = statistics.median(times), min(times)
            alg = n_leaf * ((4 if leaf is not None else 0) + 1 + 4)
            print(f"| {name} | {leaf_name} | {n_leaf:,} | {med:.4f} | {mn:.4f} | {n_leaf / (med * 1e-3) / 1e9:.1f} | "
                  f"{alg / 1e6:.1f} | {alg / (med * 1e-3) / 1e9:,.0f} |", flush=True)
        del w, packed, half, out
        torch.cuda.empty_cache()


def tree(args, torch, B, synth, dev):
    """Whole trees on every workload: 255 leaves grown leaf-wise by gbdt_grow_tree (the tree size of
    Sec. 5) and depth 8 grown level-wise by gbdt_grow_tree_depthwise (the depth Sec. 5 gives the
    comparison trainers).  Host wall time per tree, stream synchronised at both ends (median of 5
    after a warm-up)."""
    print("| workload | rows x features, bins | growth | leaves reached | deepest leaf | wall ms / tree (median) | "
          "wall ms / tree (min) | splits / s |")
    print("|" + "---|" * 8, flush=True)
    runs = [(name, make, False) for name, make in WORKLOADS.items()]
    # the three large shapes once more with labels that depend on the features (balanced trees)
    runs += [(name + "+signal", WORKLOADS[name], True) for name in ("dense_wide", "dense_tall", "categorical")]
    for name, make, signal in runs:
        if args.only and name not in args.only:
            continue
        w = make(synth, dev)
        n, F, nb = w.n_rows, w.n_features, w.n_bins
        if signal:
            gen = torch.Generator(device=dev)
            gen.manual_seed(31)
            w.grad, w.hess = synth.labels_with_signal(w.bins, nb, gen)
        packed = B.gbdt_bins_pack(w.bins, nb)
        del w.bins
        order = torch.empty(n, dtype=torch.int32, device=dev)
        for growth in ("leaf-wise, 255 leaves", "level-wise, depth 8"):
            scratch, walls = None, []
            for rep in range(6):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                if growth.startswith("leaf"):
                    nodes, _, scratch = B.gbdt_grow_tree(packed, n, F, nb, w.grad, w.hess, 255, w.lam,
                                                         w.min_child_hess, scratch=scratch, row_order_out=order)
                else:
                    nodes, _, scratch = B.gbdt_grow_tree_depthwise(packed, n, F, nb, w.grad, w.hess, 8, w.lam,
                                                                   w.min_child_hess, scratch=scratch,
                                                                   row_order_out=order)
                torch.cuda.synchronize()
                if rep:
                    walls.append((time.perf_counter() - t0) * 1e3)
            leaves = int((nodes["left"] < 0).sum())
            depth = [0] * len(nodes)
            for k in range(1, len(nodes)):
                depth[k] = depth[int(nodes[k]["parent"])] + 1
            med = statistics.median(walls)
            print(f"| {name} | {n:,} x {F}, {nb} | {growth} | {leaves} | {max(depth)} | {med:.2f} | {min(walls):.2f} | "
                  f"{(leaves - 1) / (med * 1e-3):,.0f} |", flush=True)
            del scratch
        del w, packed, order
        torch.cuda.empty_cache()


def split_sweep(args, torch, B, synth, dev):
    """gbdt_best_split_batch over 1 .. 64 histograms in one launch, at the shapes of the five
    workloads (random histograms: the time does not depend on the values).  A round of leaf-wise
    growth searches up to 64 children at once, a level of level-wise growth up to 256."""
    print("| features x bins | histograms | call ms (median) | call ms (min) | us per histogram | "
          "histogram GB/s |")
    print("|" + "---|" * 6, flush=True)
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    for F, nb in ((28, 64), (2000, 63), (28, 255), (137, 255), (700, 16)):
        for nh in (1, 2, 4, 8, 16, 32, 64, 256):
            h = torch.rand((nh, F, nb, 3), device=dev, generator=gen)
            h.view(torch.int32)[..., 2] = torch.randint(1, 100, (nh, F, nb), device=dev, dtype=torch.int32,
                                                        generator=gen)
            out = torch.empty((nh, 9), dtype=torch.int32, device=dev)
            times = []
            for rep in range(25):
                e0, e1 = _events(torch)
                e0.record()
                B.gbdt_best_split_batch(h, 1.0, 1e-3, out)
                e1.record()
                torch.cuda.synchronize()
                if rep >= 5:
                    times.append(e0.elapsed_time(e1))
            med, mn = statistics.median(times), min(times)
            print(f"| {F} x {nb} | {nh} | {med:.4f} | {mn:.4f} | {med * 1e3 / nh:.2f} | "
                  f"{nh * F * nb * 12 / (med * 1e-3) / 1e9:,.0f} |", flush=True)
            del h, out


def copy_sweep(args, torch, B, synth, dev):
    """Plain copies and fills of the sizes the row partition moves (42 MB = the row ids of a
    10.5 M-row list), as a yardstick for its two passes: the library's calibration copy kernel and
    torch's copy_ / fill_, calls back to back, median of 50."""
    print("| bytes | library copy kernel us | torch copy_ us | torch fill_ us | copy GB/s (read + write) |")
    print("|" + "---|" * 5, flush=True)

    def timed(fn, n=50):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(n):
            e0, e1 = _events(torch)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3)
        return statistics.median(ts)

    for mb in (2, 10, 42, 168, 672):
        nbytes = mb * 1_000_000 // 16 * 16
        src = torch.ones(nbytes, dtype=torch.uint8, device=dev)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        lib_us = timed(lambda: B.gbdt_calibration_copy(src, dst))
        t_copy = timed(lambda: dst.copy_(src))
        t_fill = timed(lambda: dst.fill_(3))
        best = min(lib_us, t_copy)
        print(f"| {nbytes:,} | {lib_us:.1f} | {t_copy:.1f} | {t_fill:.1f} | {2 * nbytes / (best * 1e-6) / 1e9:,.0f} |",
              flush=True)
        del src, dst


def batch_sweep(args, torch, B, synth, dev):
    """The depth benchmark of App. C.2 (8,000,000 x 500, leaves of N / 2^D rows), taken over a
    whole tree level: the 2^D leaves of depth D (a random partition of the rows into equal
    sorted lists) built one call per leaf, and all of them in one gbdt_hist_build_batch call."""
    print("| bins | D | leaves | rows per leaf | leaf by leaf: ms per level (calls) | batched: ms per level | "
          "batched build kernels ms | speed-up | batched G feature-values/s | batched algorithmic GB/s | % of 8 TB/s |")
    print("|" + "---|" * 11, flush=True)
    n, F = 8_000_000, 500
    for nb in (64, 256):
        gen = torch.Generator(device=dev)
        gen.manual_seed(100 + nb)
        bins = synth.uniform_bins(n, F, nb, gen, dev)
        grad, hess = synth.logistic_grad_hess(n, gen, dev)
        packed = B.gbdt_bins_pack(bins, nb)
        del bins
        perm = torch.randperm(n, generator=gen, device=dev).to(torch.int32)
        for depth in range(1, 11):
            n_leaves = 2 ** depth
            per = n // n_leaves
            offs = [i * per for i in range(n_leaves)] + [n]
            rows = torch.cat([torch.sort(perm[offs[i]:offs[i + 1]]).values for i in range(n_leaves)]).contiguous()
            hist = torch.empty((n_leaves, F, nb, 3), dtype=torch.float32, device=dev)

            def one_by_one():
                for i in range(n_leaves):
                    B.gbdt_hist_build(packed, n, F, nb, rows[offs[i]:offs[i + 1]], offs[i + 1] - offs[i],
                                      grad, hess, hist_out=hist[i])

            def batched():
                B.gbdt_hist_build_batch(packed, n, F, nb, rows, offs, grad, hess, hist_out=hist)

            res = {}
            for name, fn, reps in (("single", one_by_one, 3 if depth >= 7 else 5), ("batch", batched, 10)):
                fn()
                torch.cuda.synchronize()
                ts, ks = [], []
                for _ in range(reps):
                    B.gbdt_profile_enable(True)
                    e0, e1 = _events(torch)
                    e0.record()
                    fn()
                    e1.record()
                    torch.cuda.synchronize()
                    B.gbdt_profile_enable(False)
                    ms, _k = B.gbdt_profile_collect()
                    ts.append(e0.elapsed_time(e1))
                    ks.append(ms)
                res[name] = (statistics.median(ts), statistics.median(ks))
            t_single, t_batch, k_batch = res["single"][0], res["batch"][0], res["batch"][1]
            alg = algorithmic_bytes(n, F, nb, True) + (n_leaves - 1) * F * nb * 12
            print(f"| {nb} | {depth} | {n_leaves} | {per:,} | {t_single:.3f} ({n_leaves}) | {t_batch:.3f} | {k_batch:.3f} | "
                  f"{t_single / t_batch:.2f}x | {n * F / (t_batch * 1e-3) / 1e9:,.0f} | {alg / (t_batch * 1e-3) / 1e9:,.0f} | "
                  f"{100 * alg / (t_batch * 1e-3) / 1e9 / HBM_PEAK_GBS:.1f} |", flush=True)
            del rows, hist
        del packed, perm
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--depth-sweep", action="store_true")
    ap.add_argument("--skew", action="store_true")
    ap.add_argument("--paired-leaves", action="store_true",
                    help="index-list leaves of single rows against leaves of aligned row pairs")
    ap.add_argument("--partition", action="store_true")
    ap.add_argument("--tree", action="store_true")
    ap.add_argument("--batch-sweep", action="store_true")
    ap.add_argument("--split", action="store_true", help="split search over 1 .. 256 histograms per launch")
    ap.add_argument("--copy", action="store_true", help="plain copies and fills, the yardstick of the row partition")
    ap.add_argument("--oracle", action="store_true", help="time the CPU oracle on the root leaves")
    ap.add_argument("--only", nargs="*", default=None)
    ap.add_argument("--wide", action="store_true", help="measure in the wide-accumulation mode")
    ap.add_argument("--deterministic", action="store_true", help="measure with the fixed split of units")
    args = ap.parse_args()

    import torch
    from paper_1706_08359_amd import binding as B
    from paper_1706_08359_amd import synth

    if not torch.cuda.is_available():
        raise SystemExit("measure_all needs a GPU")
    B.load()
    B.gbdt_set_wide_accumulation(args.wide)
    B.gbdt_set_deterministic(args.deterministic)
    dev = torch.device("cuda:0")
    if args.depth_sweep:
        depth_sweep(args, torch, B, synth, dev)
    elif args.skew:
        skew(args, torch, B, synth, dev)
    elif args.paired_leaves:
        paired_leaves(args, torch, B, synth, dev)
    elif args.partition:
        partition(args, torch, B, synth, dev)
    elif args.tree:
        tree(args, torch, B, synth, dev)
    elif args.batch_sweep:
        batch_sweep(args, torch, B, synth, dev)
    elif args.split:
        split_sweep(args, torch, B, synth, dev)
    elif args.copy:
        copy_sweep(args, torch, B, synth, dev)
    else:
        five_workloads(args, torch, B, synth, dev)


if __name__ == "__main__":
    main()

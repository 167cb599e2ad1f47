"""Leaf-wise growth of one regression tree on the CPU -- TEST INFRASTRUCTURE.

Sec. 3.1 grows a tree from the root by splitting existing leaves until a stopping
condition holds; Sec. 5 stops at a fixed number of leaves (255) with at least one sample
per leaf.  The paper does not say which leaf is split next; the reading taken here is the
trainer's it builds on: always the open leaf whose best split has the largest gain
(best-first), ties to the leaf created first.  Every step is one of the pinned oracle
functions, called on the node's own rows, with nothing reused between nodes (no
histogram subtraction, no incremental bookkeeping):

    histogram of the node's rows   (Alg. 1)             gbdt_oracle.hist_build
    best split of that histogram   (Sec. 3.3)           gbdt_oracle.best_split
    rows of the two children       (App. C.1, Split())  gbdt_oracle.partition_rows

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
"""
from __future__ import annotations

import numpy as np

from . import gbdt_oracle as orc


def grow_tree(bins, n_bins, grad, hess, max_leaves, lam, min_child_hess, min_split_gain=0.0):
    """Returns a list of node dicts in creation order (node 0 = root; the children of a
    split get the next two ids, left first).  Keys: parent, left, right (-1 for none), rows
    (int32 row ids, ascending), split (the node's best split as best_split returns it;
    feature -1 when no threshold is admissible), count, sum_grad, sum_hess."""
    bins = np.ascontiguousarray(bins, dtype=np.uint8)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    hess = np.ascontiguousarray(hess, dtype=np.float32)
    n_rows = bins.shape[0]

    def make_node(parent, rows):
        hist = orc.hist_build(bins, n_bins, grad, hess, rows)
        return dict(parent=parent, left=-1, right=-1, rows=rows,
                    split=orc.best_split(hist, lam, min_child_hess),
                    count=int(rows.size),
                    sum_grad=float(grad[rows].astype(np.float64).sum()),
                    sum_hess=float(hess[rows].astype(np.float64).sum()))

    nodes = [make_node(-1, np.arange(n_rows, dtype=np.int32))]
    n_leaves = 1
    while n_leaves < max_leaves:
        best = -1
        for k, nd in enumerate(nodes):            # ascending id: ties go to the older leaf
            if nd["left"] >= 0 or nd["split"]["feature"] < 0:
                continue
            if not nd["split"]["gain"] > min_split_gain:
                continue
            if best < 0 or nd["split"]["gain"] > nodes[best]["split"]["gain"]:
                best = k
        if best < 0:
            break
        nd = nodes[best]
        left, right = orc.partition_rows(bins, nd["split"]["feature"], nd["split"]["bin"], nd["rows"])
        nd["left"], nd["right"] = len(nodes), len(nodes) + 1
        nodes.append(make_node(best, left))
        nodes.append(make_node(best, right))
        n_leaves += 1
    return nodes


def grow_tree_depthwise(bins, n_bins, grad, hess, max_depth, lam, min_child_hess, min_split_gain=0.0):
    """Level-wise growth (the other common stopping rule: Sec. 5 runs the comparison trainers
    with a maximum tree depth of 8): every node of the current level whose best split is
    admissible and gains more than min_split_gain is split, level after level, until max_depth.
    Nodes are numbered level by level, the children of a level in the order of their parents,
    left first.  Same node dicts as grow_tree, plus "depth"."""
    bins = np.ascontiguousarray(bins, dtype=np.uint8)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    hess = np.ascontiguousarray(hess, dtype=np.float32)

    def make_node(parent, rows, depth):
        hist = orc.hist_build(bins, n_bins, grad, hess, rows)
        return dict(parent=parent, left=-1, right=-1, rows=rows, depth=depth,
                    split=orc.best_split(hist, lam, min_child_hess),
                    count=int(rows.size),
                    sum_grad=float(grad[rows].astype(np.float64).sum()),
                    sum_hess=float(hess[rows].astype(np.float64).sum()))

    nodes = [make_node(-1, np.arange(bins.shape[0], dtype=np.int32), 0)]
    level = [0]
    for depth in range(max_depth):
        nxt = []
        for k in level:
            nd = nodes[k]
            if nd["split"]["feature"] < 0 or not nd["split"]["gain"] > min_split_gain:
                continue
            left, right = orc.partition_rows(bins, nd["split"]["feature"], nd["split"]["bin"], nd["rows"])
            nd["left"], nd["right"] = len(nodes), len(nodes) + 1
            nodes.append(make_node(k, left, depth + 1))
            nodes.append(make_node(k, right, depth + 1))
            nxt += [nd["left"], nd["right"]]
        if not nxt:
            break
        level = nxt
    return nodes


def route_rows(bins, nodes):
    """Leaf reached by every row when it is sent down the tree by the stored splits alone
    (left when bin <= threshold).  Independent of the row lists kept while growing."""
    bins = np.asarray(bins)
    at = np.zeros(bins.shape[0], dtype=np.int64)
    for k, nd in enumerate(nodes):                # parents precede children
        if nd["left"] < 0:
            continue
        here = np.nonzero(at == k)[0]
        goes_left = bins[here, nd["split"]["feature"]] <= nd["split"]["bin"]
        at[here[goes_left]] = nd["left"]
        at[here[~goes_left]] = nd["right"]
    return at

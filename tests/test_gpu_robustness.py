"""Process-wide state of the library (scratch workspace, unit counters, split tickets) after
things went wrong, and the calls a stream capture may and may not contain.

No test here makes the GPU fault: a scratch buffer the caller scribbled over only changes
which units of rows the build's workgroups take (every take is bounds-checked against the
leaf), so the wrong histogram it produces is a harmless wrong histogram.
"""
import numpy as np
import pytest
import torch

from oracle import gbdt_oracle as orc
from paper_1706_08359_amd import binding as B

from gpu_util import GpuProblem, REL_TOL, assert_hist_close

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _problem(n, F, nb, seed):
    rng = np.random.default_rng(seed)
    bins = rng.integers(0, nb, size=(n, F), dtype=np.uint8)
    grad = rng.normal(size=n).astype(np.float32)
    hess = rng.uniform(0.01, 1.0, size=n).astype(np.float32)
    return GpuProblem(bins, nb, grad, hess)


def _check(p, hist, what):
    ref = p.oracle(None)
    sg, sh = p.leaf_abs_sums(None)
    assert_hist_close(B.hist_to_numpy(hist), ref, sg, sh, what)


def test_reset_recovers_from_a_scribbled_caller_workspace():
    """The unit counters at the head of a scratch buffer are zero between calls and the library
    remembers that.  A caller that reuses its registered buffer for something else breaks the
    assumption; gbdt_reset makes the next call clear them again."""
    p = _problem(5_000_000, 64, 64, 11)        # long enough for the run-time hand-out of units
    need = B.gbdt_workspace_bytes(p.n_rows, p.n_features, p.n_bins)
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda:0")
    try:
        B.gbdt_set_workspace(ws)
        _check(p, p.build(), "caller workspace, first call")
        ws.fill_(0x11)                         # the caller scribbles over its buffer
        torch.cuda.synchronize()
        bad = B.hist_to_numpy(p.build())
        torch.cuda.synchronize()
        lost = p.n_rows - int(bad["count"][0].sum())
        _say(f"  scribbled counters: {lost} of {p.n_rows} rows missing from feature 0's counts")
        assert lost != 0, "the scribble went unnoticed: the scenario no longer tests anything"
        ws.fill_(0x11)                         # (the reduction pass of that call had set them back to zero)
        torch.cuda.synchronize()
        B.gbdt_reset()
        _check(p, p.build(), "caller workspace after gbdt_reset")
        _check(p, p.build(), "caller workspace, call after that")
    finally:
        B.gbdt_set_workspace(None)
        B.gbdt_reset()
    _check(p, p.build(), "library workspace after gbdt_reset")


def test_too_small_caller_workspace_fails_cleanly_and_later_calls_are_right():
    p = _problem(300_000, 70, 255, 12)
    small = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda:0")
    try:
        B.gbdt_set_workspace(small)
        with pytest.raises(B.GbdtError) as e:
            p.build()
        assert "(-4)" in str(e.value)
        # the split search fits (a few KB of candidates) and must still be right on the same buffer
        B.gbdt_set_workspace(None)
        hist = p.build()
        B.gbdt_set_workspace(small)
        s_small = B.split_to_dict(B.gbdt_best_split(hist, 1.0, 1e-3))
    finally:
        B.gbdt_set_workspace(None)
    _check(p, hist, "library workspace after ENOMEM")
    s_lib = B.split_to_dict(B.gbdt_best_split(hist, 1.0, 1e-3))
    assert s_small == s_lib


def test_growth_of_the_library_scratch_is_refused_under_capture_and_noalloc_is_capturable():
    """After gbdt_reset the library owns no scratch; a build inside a stream capture would have
    to allocate and is refused with GBDT_ENOMEM before anything is enqueued.  The entry point that
    allocates nothing can be captured cold; every replay must equal the eager result."""
    p = _problem(200_000, 40, 64, 13)
    out = torch.empty((p.n_features, p.n_bins, 3), dtype=torch.float32, device="cuda:0")
    ref = p.oracle(None)
    sg, sh = p.leaf_abs_sums(None)
    B.gbdt_debug_occupancy(p.n_bins, False)    # (cached by the library; queried outside the capture)
    B.gbdt_reset()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        graph = torch.cuda.CUDAGraph()
        refused = None
        with torch.cuda.graph(graph):
            try:
                B.gbdt_hist_build(p.packed, p.n_rows, p.n_features, p.n_bins, None, p.n_rows, p.grad, p.hess,
                                  hist_out=out)
            except B.GbdtError as e:
                refused = str(e)
            B.gbdt_hist_build_noalloc(p.packed, p.n_rows, p.n_features, p.n_bins, None, p.n_rows, p.grad, p.hess,
                                      out)
        assert refused is not None and "(-4)" in refused, refused
        for rep in range(3):
            out.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert_hist_close(B.hist_to_numpy(out), ref, sg, sh, f"replay {rep}")
            # eager work of the program between the replays
            _check(p, p.build(), f"eager build between replays {rep}")
    torch.cuda.current_stream().wait_stream(s)


def test_split_search_over_many_workgroups_is_stable():
    """The arg-max over the workgroups' candidates runs in the workgroup that draws the last
    ticket; candidates cross between workgroups (and XCDs) through device-scope atomics.  4,000
    features = 256 workgroups per histogram, 64 histograms per launch, the winner planted in a
    different feature of every histogram; repeated launches must all find it."""
    F, nb, H = 4000, 16, 64
    rng = np.random.default_rng(14)
    hists = np.zeros((H, F, nb, 3), np.float32)
    hists[..., 1] = 1.0                               # hessian 1 per bin
    cnt = np.full((H, F, nb), 10, np.uint32)          # the third word of a bin is a uint32
    hists[..., 2] = cnt.view(np.float32)
    grad = rng.normal(0, 0.01, size=(H, F, nb)).astype(np.float32)
    want = []
    for h in range(H):
        f = int(rng.integers(0, F))
        t = int(rng.integers(0, nb - 1))
        grad[h, f, : t + 1] = 50.0
        grad[h, f, t + 1:] = -50.0
        want.append((f, t))
    hists[..., 0] = grad
    d = torch.from_numpy(hists).cuda()
    for rep in range(20):
        recs = B.splits_to_dicts(B.gbdt_best_split_batch(d, 1.0, 1e-3))
        got = [(r["feature"], r["bin"]) for r in recs]
        assert got == want, (rep, [i for i in range(H) if got[i] != want[i]][:5])
    # and against the oracle's scan of the same numbers, one histogram
    o = orc.best_split(orc.from_f32_hist(grad[3], hists[3, ..., 1], cnt[3]), 1.0, 1e-3)
    assert (o["feature"], o["bin"]) == want[3]

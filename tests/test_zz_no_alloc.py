"""gbdt_hist_build_noalloc (the entry point for callers that cannot allocate) against
gbdt_hist_build, through the C ABI: same inputs, same outputs to the bar of the other parity
tests -- counts bit-exact, gradient / hessian sums within 1e-5 of the leaf's sum of magnitudes
(bit-equal in the deterministic mode whenever both entry points plan the same grid), and
both against the CPU oracle.  Two calls in a row share the fixed scratch, the second with a
smaller input; a shape whose partial histograms exceed the fixed scratch is refused."""
import ctypes

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


def _both(p, idx, what):
    """Builds one leaf through both entry points and compares them with each other and the oracle."""
    n_leaf = p.n_rows if idx is None else int(idx.numel())
    _say(f"{what}: {n_leaf} leaf rows x {p.n_features} features, {p.n_bins} bins")
    ref_call = B.gbdt_hist_build(p.packed, p.n_rows, p.n_features, p.n_bins, idx, n_leaf, p.grad, p.hess)
    out = torch.full_like(ref_call, float("nan"))
    B.gbdt_hist_build_noalloc(p.packed, p.n_rows, p.n_features, p.n_bins, idx, n_leaf, p.grad, p.hess, out)
    torch.cuda.synchronize()
    a, b = B.hist_to_numpy(ref_call), B.hist_to_numpy(out)
    sg, sh = p.leaf_abs_sums(idx)
    assert (a["count"] == b["count"]).all(), f"{what}: counts differ between the entry points"
    assert np.abs(a["grad"].astype(np.float64) - b["grad"]).max() <= REL_TOL * sg
    assert np.abs(a["hess"].astype(np.float64) - b["hess"]).max() <= REL_TOL * sh
    ref = p.oracle(idx)
    assert_hist_close(b, ref, sg, sh, what)
    return a, b


def test_noalloc_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    # first call: a root leaf long enough for the run-time hand-out of units (unit counters in use)
    big = _problem(5_000_000, 64, 64, 1)
    _both(big, None, "first call (root)")
    # second call right behind it, smaller, on the same fixed scratch: an index list with repeats
    small = _problem(9_000, 33, 255, 2)
    idx = torch.from_numpy(np.random.default_rng(3).integers(0, 9_000, size=5_000).astype(np.int32)).cuda()
    _both(small, idx, "second call (index list)")
    # and a third, smaller still, that one workgroup per tile writes directly
    tiny = _problem(700, 9, 16, 4)
    _both(tiny, None, "third call (tiny)")
    # the first shape again: what the earlier calls left in the scratch does not matter
    _both(big, torch.arange(0, 5_000_000, 3, dtype=torch.int32, device="cuda:0"), "fourth call (strided list)")


def test_noalloc_is_bit_equal_in_the_deterministic_mode():
    p = _problem(300_000, 40, 64, 5)
    B.gbdt_set_deterministic(True)
    try:
        a, b = _both(p, None, "deterministic root")
        assert np.array_equal(a["grad"].view(np.uint32), b["grad"].view(np.uint32))
        assert np.array_equal(a["hess"].view(np.uint32), b["hess"].view(np.uint32))
    finally:
        B.gbdt_set_deterministic(False)


def test_noalloc_shrinks_the_grid_to_fit_the_fixed_scratch():
    """Wide accumulation writes two partial blocks per workgroup: at 256 bins the usual grid of a
    long leaf (two workgroups per compute unit) would need about 100 MB, so the entry point plans
    fewer workgroups; the histogram is the same up to the summation order (here: the stored value
    is the exact sum rounded to fp32 in both)."""
    p = _problem(1_200_000, 28, 255, 7)
    B.gbdt_set_wide_accumulation(True)
    try:
        a, b = _both(p, None, "wide root, shrunk grid")
        ref = p.oracle(None)
        sg, sh = p.leaf_abs_sums(None)
        for got in (a, b):
            assert np.abs(got["grad"].astype(np.float64) - ref["grad"]).max() <= 1e-9 * sg + 2.0 ** -23 * np.abs(ref["grad"]).max()
    finally:
        B.gbdt_set_wide_accumulation(False)


def test_noalloc_empty_leaf_and_argument_errors():
    p = _problem(2_000, 5, 64, 6)
    out = torch.full((5, 64, 3), 7.0, dtype=torch.float32, device="cuda:0")
    B.gbdt_hist_build_noalloc(p.packed, p.n_rows, 5, 64, None, 0, p.grad, p.hess, out)
    torch.cuda.synchronize()
    assert (out == 0).all()
    lib = B.load()
    args = [p.packed.data_ptr(), p.n_rows, 5, 64, None, p.n_rows, p.grad.data_ptr(), p.hess.data_ptr()]
    assert lib.gbdt_hist_build_noalloc(*args, None, None) == -1                 # no output buffer
    assert lib.gbdt_hist_build_noalloc(*args[:3], 300, *args[4:], out.data_ptr(), None) == -1


def test_noalloc_refuses_what_the_fixed_scratch_cannot_hold():
    """One workgroup per tile of a 30,000-feature, 256-bin matrix writes 92 MB of partial
    histograms: more than the 64 MiB of the fixed scratch.  The call must say so before it
    enqueues anything (it never looks at the buffers)."""
    lib = B.load()
    cap = B.gbdt_hist_build_noalloc_max_partial_bytes()
    assert cap == 64 << 20
    n, F, nb = 100_000, 30_000, 256
    dummy = torch.zeros(1024, dtype=torch.float32, device="cuda:0")
    rc = lib.gbdt_hist_build_noalloc(dummy.data_ptr(), n, F, nb, None, n, dummy.data_ptr(), dummy.data_ptr(),
                                     dummy.data_ptr(), None)
    assert rc == -2, rc
    assert b"fixed scratch" in lib.gbdt_last_hip_error()
    torch.cuda.synchronize()

"""GPU parity of gbdt_best_split on hand-made histograms (through the C ABI), against the oracle's
scan of the SAME fp32 numbers: the chosen (feature, bin) must be identical, with no tolerance.

The kernel sums a feature's bins strictly left to right in fp64, as the oracle does.  These
histograms put exact ties and near-ties on the thresholds, where a prefix sum that differed in
its last bit would change the choice, spread bin sums over 60 binary orders of magnitude, and
fill launches with many histograms, where a workgroup takes several groups of features in turn
and ties between them must still fall to the smaller feature."""
import numpy as np
import pytest
import torch

from oracle import gbdt_oracle as orc
from paper_1706_08359_amd import binding as B

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)


def _check(grad, hess, count, lam=1.0, mch=1e-3, what=""):
    F, nb = grad.shape
    h = np.zeros((F, nb), dtype=B.BIN_DTYPE)
    h["grad"], h["hess"], h["count"] = grad, hess, count
    t = torch.from_numpy(h.view(np.float32).reshape(F, nb, 3).copy()).to("cuda:0")
    got = B.split_to_dict(B.gbdt_best_split(t, lam, mch))
    ref, gains = orc.best_split(orc.from_f32_hist(h["grad"], h["hess"], h["count"]), lam, mch, return_gains=True)
    assert (got["feature"], got["bin"]) == (ref["feature"], ref["bin"]), (what, got, ref)
    if ref["feature"] >= 0:
        assert got["left_count"] == ref["left_count"] and got["right_count"] == ref["right_count"]
        # the prefix sums behind the record, rounded to fp32 once: identical
        assert np.float32(ref["left_grad"]) == np.float32(got["left_grad"]), what
        assert np.float32(ref["left_hess"]) == np.float32(got["left_hess"]), what
        with np.errstate(over="ignore"):
            ref_gain = float(np.float32(ref["gain"]))            # the record stores fp32 (may overflow to inf)
        assert got["gain"] == ref_gain or abs(got["gain"] - ref_gain) <= 1e-6 * max(1.0, abs(ref_gain)), what
    return got


@pytest.mark.parametrize("F,nb", [(1, 2), (3, 16), (28, 64), (70, 63), (28, 255), (137, 256), (300, 17), (2000, 63)])
def test_split_of_ordinary_histograms(F, nb):
    """Magnitudes within a few decades."""
    _say(f"split {F}x{nb} ordinary")
    rng = np.random.default_rng(F * 1000 + nb)
    count = rng.integers(0, 500, size=(F, nb)).astype(np.uint32)
    grad = (rng.normal(size=(F, nb)) * np.sqrt(count + 1.0)).astype(np.float32) * (count > 0)
    hess = (rng.uniform(0.05, 0.25, size=(F, nb)) * count).astype(np.float32)
    _check(grad, hess, count, what="ordinary")


@pytest.mark.parametrize("F,nb", [(3, 16), (28, 64), (28, 255), (137, 256), (500, 63)])
def test_split_of_wide_range_histograms(F, nb):
    """Bin sums spread over 60 binary orders of magnitude: partial sums round, so the order of the
    additions shows in the result; such rows are mixed with ordinary rows in the same workgroup."""
    _say(f"split {F}x{nb} wide range")
    rng = np.random.default_rng(F * 77 + nb)
    count = rng.integers(1, 500, size=(F, nb)).astype(np.uint32)
    scale = 2.0 ** rng.integers(-30, 30, size=(F, nb))
    wide = rng.random(F) < 0.5                                   # about half of the features
    scale[~wide] = 1.0
    grad = (rng.normal(size=(F, nb)) * scale).astype(np.float32)
    hess = (rng.uniform(0.05, 0.25, size=(F, nb)) * count * np.where(wide[:, None], scale, 1.0)).astype(np.float32)
    _check(grad, hess, count, what="wide")


def test_split_exact_ties_and_empty_bins():
    """Empty bins make neighbouring thresholds the same partition, copies of a feature make
    different features tie: the smaller feature, then the smaller bin, must win -- which they
    only do when equal prefixes come out bit-identical."""
    rng = np.random.default_rng(5)
    for nb in (16, 64, 255):
        F = 12
        count = rng.integers(0, 3, size=(F, nb)).astype(np.uint32) * rng.integers(0, 2, size=(F, nb)).astype(np.uint32)
        grad = (rng.normal(size=(F, nb)) * (count > 0)).astype(np.float32)
        hess = (0.25 * count).astype(np.float32)
        for f in range(1, F, 2):                                 # odd features copy the one before
            count[f], grad[f], hess[f] = count[f - 1], grad[f - 1], hess[f - 1]
        _say(f"split ties {F}x{nb}")
        got = _check(grad, hess, count, lam=0.0, mch=0.25, what="ties")
        assert got["feature"] % 2 == 0


def test_split_denormals_zeros_and_huge_counts():
    nb, F = 64, 6
    count = np.full((F, nb), 2**31 // nb, dtype=np.uint32)        # sums reach 2^31
    grad = np.zeros((F, nb), dtype=np.float32)
    hess = np.ones((F, nb), dtype=np.float32)
    grad[0] = np.float32(1e-42)                                  # denormal bins only
    grad[1, ::3] = np.float32(-1e-40)
    grad[2] = np.linspace(-1, 1, nb, dtype=np.float32)
    grad[3, 5] = np.float32(3e38)                                # one huge bin among tiny ones
    grad[3, 6:] = np.float32(1e-30)
    grad[4] = -grad[2]
    _check(grad, hess, count, what="denormals")


@pytest.mark.parametrize("F,nb,H", [(2000, 63, 24), (137, 255, 64), (700, 16, 40), (28, 255, 64), (45, 64, 3)])
def test_split_batch_of_many_histograms(F, nb, H):
    """One launch over H histograms: the work split depends on H (larger feature groups, several
    groups per workgroup, a ragged last group), the records must not.  Every histogram against the
    oracle; two of them are copies of one another up to a shift of the features by one group, so
    that the same gain turns up in different workgroups and passes."""
    _say(f"split batch {H} x {F}x{nb}")
    rng = np.random.default_rng(F * 31 + nb * 7 + H)
    count = rng.integers(0, 400, size=(H, F, nb)).astype(np.uint32)
    grad = (rng.normal(size=(H, F, nb)) * np.sqrt(count + 1.0)).astype(np.float32) * (count > 0)
    hess = (rng.uniform(0.05, 0.25, size=(H, F, nb)) * count).astype(np.float32)
    if H >= 2 and F > 20:
        count[1], grad[1], hess[1] = np.roll(count[0], 17, axis=0), np.roll(grad[0], 17, axis=0), np.roll(hess[0], 17, axis=0)
    # the same feature twice, far apart: an exact tie that the smaller feature must win
    if F > 20:
        for h in range(2, H, 5):
            a, b = int(rng.integers(0, F // 2)), int(rng.integers(F // 2, F))
            grad[h, a] *= 3.0                                     # make it the likely winner
            count[h, b], grad[h, b], hess[h, b] = count[h, a], grad[h, a], hess[h, a]
    hist = np.zeros((H, F, nb), dtype=B.BIN_DTYPE)
    hist["grad"], hist["hess"], hist["count"] = grad, hess, count
    t = torch.from_numpy(hist.view(np.float32).reshape(H, F, nb, 3).copy()).to("cuda:0")
    got = B.splits_to_dicts(B.gbdt_best_split_batch(t, 1.0, 1e-3))
    for h in range(H):
        ref = orc.best_split(orc.from_f32_hist(grad[h], hess[h], count[h]), 1.0, 1e-3)
        assert (got[h]["feature"], got[h]["bin"]) == (ref["feature"], ref["bin"]), (h, got[h], ref)
        if ref["feature"] >= 0:
            assert got[h]["left_count"] == ref["left_count"] and got[h]["right_count"] == ref["right_count"], h
            assert np.float32(ref["left_grad"]) == np.float32(got[h]["left_grad"]), h
            assert np.float32(ref["right_hess"]) == np.float32(got[h]["right_hess"]), h
    # and one histogram at a time gives the same records
    for h in (0, H - 1):
        one = B.split_to_dict(B.gbdt_best_split(t[h], 1.0, 1e-3))
        assert one == got[h], h

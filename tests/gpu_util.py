"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI and
compare with the CPU oracle under the stated tolerances."""
import numpy as np
import torch

from oracle import gbdt_oracle as orc
from paper_1706_08359_amd import binding as B

REL_TOL = 1e-5   # |gpu - oracle| <= REL_TOL * sum_leaf |g|  (and sum |h| for hessians)


class GpuProblem:
    """A workload resident on the GPU in the library's layout."""

    def __init__(self, bins, n_bins, grad, hess, device="cuda:0"):
        self.dev = torch.device(device)
        self.bins_cpu = bins.cpu().contiguous() if isinstance(bins, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(bins))
        self.n_rows, self.n_features = self.bins_cpu.shape
        self.n_bins = int(n_bins)
        as_t = lambda a: a if isinstance(a, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(a))
        self.grad_cpu, self.hess_cpu = as_t(grad).cpu().contiguous(), as_t(hess).cpu().contiguous()
        bins_d = bins.to(self.dev) if isinstance(bins, torch.Tensor) else self.bins_cpu.to(self.dev)
        self.packed = B.gbdt_bins_pack(bins_d.contiguous(), self.n_bins)
        del bins_d
        self.grad = self.grad_cpu.to(self.dev)
        self.hess = self.hess_cpu.to(self.dev)

    def build(self, idx=None, n_leaf=None):
        """idx: None (root / first n_leaf rows), or int32 row ids (tensor or numpy)."""
        if idx is None:
            n = self.n_rows if n_leaf is None else n_leaf
            idx_d = None
        else:
            idx_t = idx if isinstance(idx, torch.Tensor) else torch.from_numpy(np.ascontiguousarray(idx, dtype=np.int32))
            idx_d = idx_t.to(self.dev).contiguous()
            n = idx_d.numel() if n_leaf is None else n_leaf
        return B.gbdt_hist_build(self.packed, self.n_rows, self.n_features, self.n_bins, idx_d, n,
                                 self.grad, self.hess)

    def oracle(self, idx=None, n_leaf=None, features=None):
        bins = self.bins_cpu.numpy()
        if features is not None:
            bins = np.ascontiguousarray(bins[:, features])
        idx_np = None
        if idx is not None:
            idx_np = idx.cpu().numpy() if isinstance(idx, torch.Tensor) else np.asarray(idx, dtype=np.int32)
        return orc.hist_build(bins, self.n_bins, self.grad_cpu.numpy(), self.hess_cpu.numpy(), idx_np, n_leaf)

    def leaf_abs_sums(self, idx=None, n_leaf=None):
        g, h = self.grad_cpu.numpy().astype(np.float64), self.hess_cpu.numpy().astype(np.float64)
        if idx is None:
            n = self.n_rows if n_leaf is None else n_leaf
            return np.abs(g[:n]).sum(), np.abs(h[:n]).sum()
        i = idx.cpu().numpy() if isinstance(idx, torch.Tensor) else np.asarray(idx)
        if n_leaf is not None:
            i = i[:n_leaf]
        return np.abs(g[i]).sum(), np.abs(h[i]).sum()


def assert_hist_close(got, ref, sum_abs_g, sum_abs_h, what=""):
    """got: gpu structured array (f4,f4,u4); ref: oracle structured array (f8,f8,u8)."""
    assert got.shape == ref.shape, (got.shape, ref.shape)
    bad = np.argwhere(got["count"].astype(np.uint64) != ref["count"])
    assert bad.size == 0, f"{what}: {len(bad)} count mismatches, first at {bad[:3].tolist()}"
    dg = np.abs(got["grad"].astype(np.float64) - ref["grad"]).max() if got.size else 0.0
    dh = np.abs(got["hess"].astype(np.float64) - ref["hess"]).max() if got.size else 0.0
    assert dg <= REL_TOL * sum_abs_g + 1e-30, f"{what}: grad err {dg} > {REL_TOL * sum_abs_g}"
    assert dh <= REL_TOL * sum_abs_h + 1e-30, f"{what}: hess err {dh} > {REL_TOL * sum_abs_h}"
    return dg, dh


def check_split(hist_gpu_t, ref_hist, lam, mch, what=""):
    """Two checks of gbdt_best_split on a GPU-built histogram:
    (1) kernel level: the oracle scan of the SAME fp32 histogram must choose the identical
        (feature, bin), with no tolerance band;
    (2) end to end: against the oracle scan of the oracle's fp64 histogram the choice must be
        identical unless the oracle's own margin between distinct partitions is inside the
        fp32 noise band, in which case any candidate inside the band is accepted.
    """
    got_hist = B.hist_to_numpy(hist_gpu_t)
    s_gpu = B.split_to_dict(B.gbdt_best_split(hist_gpu_t, lam, mch))
    lifted = orc.from_f32_hist(got_hist["grad"], got_hist["hess"], got_hist["count"])
    s_same = orc.best_split(lifted, lam, mch)
    assert (s_gpu["feature"], s_gpu["bin"]) == (s_same["feature"], s_same["bin"]), (what, s_gpu, s_same)
    if s_same["feature"] >= 0:
        assert abs(s_gpu["gain"] - s_same["gain"]) <= 1e-6 * max(1.0, abs(s_same["gain"]))
        assert s_gpu["left_count"] == s_same["left_count"] and s_gpu["right_count"] == s_same["right_count"]
        assert abs(s_gpu["left_grad"] - s_same["left_grad"]) <= 1e-6 * max(1.0, abs(s_same["left_grad"]))
        assert abs(s_gpu["right_hess"] - s_same["right_hess"]) <= 1e-6 * max(1.0, abs(s_same["right_hess"]))
    else:
        assert s_gpu["gain"] == 0.0 and s_gpu["bin"] == -1
    s_ref, gains = orc.best_split(ref_hist, lam, mch, return_gains=True)
    if (s_gpu["feature"], s_gpu["bin"]) != (s_ref["feature"], s_ref["bin"]):
        assert s_ref["feature"] >= 0 and s_gpu["feature"] >= 0, (what, s_gpu, s_ref)
        band = 1e-4 * max(1.0, abs(s_ref["gain"]))
        g_at = gains[s_gpu["feature"], s_gpu["bin"]]
        assert np.isfinite(g_at) and s_ref["gain"] - g_at <= band, (what, s_gpu, s_ref, g_at)
        print(f"[near-tie] {what}: gpu {s_gpu['feature'], s_gpu['bin']} vs oracle "
              f"{s_ref['feature'], s_ref['bin']}, gain gap {s_ref['gain'] - g_at:.3e}")
    return s_gpu, s_ref

"""Helpers of the GPU parity tests: host<->device conversion and the parity bar.

The bar (stated with the workloads): indices and hit flags must agree exactly wherever
the oracle's top-2 similarity gap exceeds 1e-3 (hit flags additionally only where the
oracle's similarity is further than the tolerance from the threshold, since a flag can
flip on rounding alone); similarities must agree within 2e-3 for bf16 inputs and 1e-5
for fp32 inputs."""

import numpy as np
import torch

GAP = 1e-3
SIM_TOL = {"bf16": 2e-3, "f32": 1e-5}
DEV = "cuda:0"


def to_dev(arr: np.ndarray, dtype: str) -> torch.Tensor:
    from paper_2508_18736_amd import siso
    return siso.to_dev(arr, dtype, DEV)


def to_host(t: torch.Tensor, dtype: str) -> np.ndarray:
    from paper_2508_18736_amd import siso
    return siso.to_host(t, dtype)


def siso_dtype(dtype: str) -> int:
    from paper_2508_18736_amd import siso
    return siso.BF16 if dtype == "bf16" else siso.F32


def check_lookup(gpu, ora, threshold: float, dtype: str, label: str = "", gap_bar: float = GAP):
    """gpu = (idx, sim, hit) tensors; ora = (idx, sim, hit, second) numpy from the oracle.
    Returns a dict of statistics; raises AssertionError on a parity violation."""
    gi = gpu[0].cpu().numpy()
    gs = gpu[1].cpu().numpy().astype(np.float64)
    gh = gpu[2].cpu().numpy()
    oi, os_, oh, osec = ora
    tol = SIM_TOL[dtype]
    finite = np.isfinite(os_)
    # special values must agree exactly
    assert np.array_equal(np.isnan(gs), np.isnan(os_)), f"{label}: NaN pattern differs"
    assert np.array_equal(np.isneginf(gs), np.isneginf(os_)), f"{label}: -inf pattern differs"
    assert np.array_equal(gi[~finite], oi[~finite]), f"{label}: idx of special queries differs"
    assert np.all(gh[~finite] == 0)
    err = np.abs(gs[finite] - os_[finite])
    assert err.size == 0 or err.max() <= tol, f"{label}: similarity error {err.max():.3e} above {tol}"
    gap = np.where(np.isfinite(osec), os_ - osec, np.inf)
    clear = finite & (gap > gap_bar)
    bad = clear & (gi != oi)
    assert not bad.any(), f"{label}: {bad.sum()} indices differ with a clear top-2 gap, first at {np.nonzero(bad)[0][:5]}"
    th = np.float64(np.float32(threshold))
    decided = clear & (np.abs(os_ - th) > tol)
    badh = decided & (gh != oh)
    assert not badh.any(), f"{label}: {badh.sum()} hit flags differ"
    # the flag must be consistent with the similarity the GPU itself reports
    assert np.array_equal(gh[finite], (gs[finite].astype(np.float32) > np.float32(threshold)).astype(np.uint8))
    return {"n": len(oi), "clear": int(clear.sum()), "max_err": float(err.max()) if err.size else 0.0,
            "idx_equal": int((gi == oi).sum()), "near_threshold": int((clear & ~decided).sum())}

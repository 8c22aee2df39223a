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


# The k closest: the similarity at every rank agrees with the oracle's within the lookup's tolerance; the index at a
# rank is compared exactly where the oracle's similarity at that rank is further than the gap bar from both
# neighbouring ranks, or ties exactly with a neighbour (equal rows: lower index first).
# The oracle may be asked for one rank more than the library (`ora` with k + 1 columns): the index at the last rank is
# then compared as well, where the extra rank shows its gap to be clear; without it the last rank's index is not
# compared (what comes behind it is unknown, and may be arbitrarily close).
def check_topk(gpu, ora, dtype, label):
    gi, gs = gpu[0].cpu().numpy(), gpu[1].cpu().numpy().astype(np.float64)
    oi, os_ = ora
    beyond = None
    if oi.shape[1] == gi.shape[1] + 1:
        beyond = os_[:, -1]
        oi, os_ = oi[:, :-1], os_[:, :-1]
    n, k = oi.shape
    tol = SIM_TOL[dtype]
    assert np.array_equal(np.isnan(gs), np.isnan(os_)), f"{label}: NaN pattern"
    assert np.array_equal(np.isneginf(gs), np.isneginf(os_)), f"{label}: empty entries"
    fin = np.isfinite(os_)
    assert np.array_equal(gi[~fin], oi[~fin]), label
    err = np.abs(gs[fin] - os_[fin])
    assert err.size == 0 or err.max() <= tol, f"{label}: similarity error {err.max():.3e}"
    both = fin[:, 1:] & fin[:, :-1]
    assert np.all(np.diff(np.where(fin, gs, 0.0), axis=1)[both] <= 0), f"{label}: not sorted"
    pad = np.full((n, 1), np.inf)
    after = -pad if beyond is None else np.where(np.isfinite(beyond), beyond, -np.inf).reshape(n, 1)
    left = np.abs(np.diff(np.concatenate([pad, os_], axis=1), axis=1))     # gap to the rank before
    right = np.abs(np.diff(np.concatenate([os_, after], axis=1), axis=1))  # gap to the rank after
    left, right = np.nan_to_num(left, nan=np.inf), np.nan_to_num(right, nan=np.inf)
    clear = fin & (left > GAP) & (right > GAP)
    if beyond is None:
        clear[:, -1] = False
    bad = clear & (gi != oi)
    assert not bad.any(), f"{label}: {bad.sum()} indices differ at ranks with clear gaps, first {np.argwhere(bad)[:4].tolist()}"
    # runs of exactly equal similarities (equal rows) come in index order on both sides - checked where the run's two
    # outer neighbours are further away than single precision can blur (a third row within 1e-5 of the run may
    # land before, inside or behind it in fp32)
    tie = fin & ((left == 0) | (right == 0))
    edge_ok = np.ones_like(tie)
    for q in range(n):
        r = 0
        while r < k:
            e = r
            while e + 1 < k and tie[q, e] and right[q, e] == 0:
                e += 1
            if e > r and not (left[q, r] > 1e-5 and right[q, e] > 1e-5):
                edge_ok[q, r:e + 1] = False
            r = e + 1
    tie &= edge_ok
    assert np.array_equal(gi[tie], oi[tie]), f"{label}: exact ties"
    # each row names k different centroids, and the set agrees except for members near the k-th similarity
    for q in range(n):
        row = gi[q][gi[q] >= 0]
        assert len(set(row.tolist())) == len(row), f"{label}: a centroid twice in query {q}"
    return {"clear": int(clear.sum()), "ties": int(tie.sum()), "max_err": float(err.max()) if err.size else 0.0,
            "same": float((gi == oi).mean())}

"""The library's host-side bookkeeping of a cache refresh (Algorithm 1: the chain of merge decisions, the
eviction, the decay) against the oracle.  The similarities that the kernels would supply come from numpy
here, so no GPU work is involved: these run wherever the library loads."""

import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2508_18736_amd", "libsiso.so")
INF = 0xFFFFFFFF


@pytest.fixture(scope="module")
def siso():
    if not os.path.exists(LIB):
        from paper_2508_18736_amd import build
        build.build(verbose=False)
    from paper_2508_18736_amd import siso as binding
    return binding


def unit(x, dtype):
    u = W.storage_to_f32(x, dtype).astype(np.float64)
    return u / np.linalg.norm(u, axis=1, keepdims=True)


@pytest.mark.parametrize("n_cur,M,seed", [(300, 10_000, 1), (300, 350, 2), (0, 10_000, 3), (500, 200, 4)])
def test_refresh_plan_matches_oracle(siso, oracle, n_cur, M, seed):
    dtype, dim, theta = "bf16", 64, 0.9
    rng = np.random.default_rng(seed)
    wl = W.c5_merge(n_groups=120, copies=5, dim=dim, sigma=0.05, dtype=dtype, seed=40 + seed)
    cur, repo = wl.centroids[:n_cur], wl.centroids[n_cur:]
    counts = rng.integers(1, 50, size=max(n_cur, 1)).astype(np.int32)[:n_cur]
    sizes = rng.integers(1, 30, size=len(repo)).astype(np.float32)
    cap = len(wl.centroids) + 8
    M = min(M, cap)
    ora = oracle.OracleCache(dim, cap, dtype)
    ora.load(cur, counts if n_cur else None)
    if n_cur:
        ora.lookup(cur[rng.integers(0, n_cur, size=200)], 0.9)      # some references first
    loc, acc = ora.export_meta()
    # what the kernels would supply, through numpy
    uc, ur = unit(cur, dtype), unit(repo, dtype)
    if n_cur:
        s = ur @ uc.T
        best_idx, best_sim = s.argmax(axis=1), s.max(axis=1)
    else:
        best_idx, best_sim = np.full(len(repo), -1), np.full(len(repo), -np.inf)
    rr = ur @ ur.T
    a, b = np.nonzero(np.triu(rr > theta, 1))
    order = rng.permutation(len(a))
    pairs, cosines = np.stack([a, b], 1)[order], rr[a, b][order]
    src, out_size, stats = siso.refresh_plan(loc, acc, sizes, best_idx, best_sim, pairs, cosines, theta, M)
    want = ora.refresh(repo, sizes, theta, M)
    assert want[3] > 0.01                                       # no decision was a close call
    assert stats == want[:3]
    rows = np.concatenate([cur, repo])[src]
    assert np.array_equal(rows, ora.export()[0])                # the same survivors in the same order
    assert np.array_equal(out_size, ora.export_meta()[0])       # single precision on both sides


def test_refresh_plan_rejects_bad_input(siso):
    ok = dict(cluster_size=[1.0], access_count=[0], repo_size=[2.0, 3.0], best_idx=[0, 0], best_sim=[0.1, 0.2],
              pairs=[(0, 1)], pair_cosine=[0.95], theta_c=0.9, max_centroids=3)
    src, size, stats = siso.refresh_plan(**ok)
    assert src.tolist() == [0, 1] and stats == (1, 1, 0)        # row 0 joins, row 1 merges into it
    assert size.tolist() == [np.float32(1.0) / np.float32(1.1), np.float32(5.0) / np.float32(1.1)]
    for key, bad in (("pairs", [(1, 0)]), ("pairs", [(0, 2)]), ("best_idx", [1, 0]), ("repo_size", [0.0, 1.0]),
                     ("max_centroids", 0)):
        with pytest.raises(siso.SisoError):
            siso.refresh_plan(**{**ok, key: bad})

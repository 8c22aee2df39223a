"""GPU parity of the lookup variants against the CPU oracle, through the C ABI: one lookup judged against
several thresholds, and the k closest centroids.

Bar for the k closest: the similarity at every rank agrees with the oracle's within the lookup's tolerance;
the index at a rank is compared exactly where the oracle's similarity at that rank is further than the gap bar
from both neighbouring ranks, or ties exactly with a neighbour (equal rows: lower index first)."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import DEV, GAP, SIM_TOL, check_lookup, check_topk, siso_dtype, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


# -------------------------------------------------------------------- several thresholds
@pytest.mark.parametrize("dtype,dim,K,n", [("bf16", 768, 5000, 700), ("bf16", 256, 3000, 64), ("f32", 384, 1024, 256)])
def test_lookup_multi_vs_oracle(siso, oracle, dtype, dim, K, n):
    print(f"case: lookup_multi {dtype} dim={dim} K={K} n={n}", flush=True)
    wl = W.c2_mid(n_clusters=128, per_cluster=(K + 127) // 128, n_queries=n, dim=dim, dtype=dtype, sigma=0.45, seed=301)
    wl.centroids = wl.centroids[:K].copy()
    wl.queries = W.spread_sample(wl.centroids, dtype, n, seed=302)   # similarities spread over the sweep
    th = np.array([0.92, 0.75, 0.85, 0.6, 0.98], np.float32)
    cache = siso.SisoCache(dim, K, siso_dtype(dtype))
    cache.load(to_dev(wl.centroids, dtype))
    q = to_dev(wl.queries, dtype)
    idx, sim, hit = cache.lookup_multi(q, th, count_index=2)
    oc = oracle.OracleCache(dim, K, dtype)
    oc.load(wl.centroids)
    oi, os_, oh, osec = oc.lookup_multi(wl.queries, th, 2)
    for j, t in enumerate(th):
        check_lookup((idx, sim, hit[:, j].contiguous()), (oi, os_, oh[:, j], osec), float(t), dtype, f"multi theta {t}")
    assert 0 < oh[:, 4].sum() < oh[:, 3].sum()          # the sweep discriminates
    # the same bits as one lookup per threshold
    for j, t in enumerate(th):
        one = cache.lookup(q, float(t))
        assert torch.equal(one[0], idx) and torch.equal(one[1], sim) and torch.equal(one[2], hit[:, j])
    # references were counted for thetas[2] only (then once more by each of the five single lookups)
    acc = cache.export_meta()[1].cpu().numpy()
    want = np.bincount(oi[oh[:, 2] == 1], minlength=K)
    for j in range(len(th)):
        want = want + np.bincount(oi[oh[:, j] == 1], minlength=K)
    near = np.abs(os_[:, None] - th.astype(np.float64)[None, :]).min(axis=1) < SIM_TOL[dtype]
    if not near.any():
        assert np.array_equal(acc, want)
    assert np.array_equal(oc.export_meta()[1], np.bincount(oi[oh[:, 2] == 1], minlength=K))
    with pytest.raises(siso.SisoError):
        cache.lookup_multi(q, np.zeros(33, np.float32))
    with pytest.raises(siso.SisoError):
        cache.lookup_multi(q, th, count_index=5)


# -------------------------------------------------------------------- the k closest
@pytest.mark.parametrize("dtype,dim,K,n,k", [
    ("bf16", 768, 40000, 300, 8),     # two passes of the 256 x 256 kernel
    ("bf16", 256, 70000, 64, 16),     # two passes, small batch
    ("bf16", 512, 33000, 100, 32),    # two passes, mid batch, largest k
    ("bf16", 128, 9000, 130, 1),      # k = 1
    ("bf16", 768, 2100, 65, 5),       # too few centroids for the two passes: row by row
    ("f32", 384, 1024, 256, 10),      # fp32 cache: row by row
    ("bf16", 72, 700, 33, 7),         # a dimension the MFMA kernels do not take
])
def test_lookup_topk_vs_oracle(siso, oracle, dtype, dim, K, n, k):
    print(f"case: lookup_topk {dtype} dim={dim} K={K} n={n} k={k}", flush=True)
    wl = W.c2_mid(n_clusters=256, per_cluster=(K + 255) // 256, n_queries=n, dim=dim, dtype=dtype, sigma=0.3, seed=311)
    wl.centroids = wl.centroids[:K].copy()
    r = np.random.default_rng(7)
    for a in r.choice(K, size=20, replace=False):          # exact duplicates at distant rows
        for b in r.choice(K, size=2, replace=False):
            wl.centroids[b] = wl.centroids[a]
    cache = siso.SisoCache(dim, K + 9, siso_dtype(dtype))
    cache.load(to_dev(wl.centroids, dtype))
    out = cache.lookup_topk(to_dev(wl.queries, dtype), k)
    torch.cuda.synchronize()
    oc = oracle.OracleCache(dim, K, dtype)
    oc.load(wl.centroids)
    ora = oc.lookup_topk(wl.queries, k + 1)     # one rank more: what lies behind the last rank decides whether it is clear
    st = check_topk(out, ora, dtype, "topk")
    print(f"  {st}", flush=True)
    assert st["clear"] >= min(n, n * k // 8) and st["max_err"] < (1e-4 if dtype == "bf16" else 2e-6) and st["same"] > 0.97
    # rank 1 is the lookup
    one = cache.lookup(to_dev(wl.queries, dtype), 0.5)
    assert torch.equal(one[0], out[0][:, 0].contiguous())
    # a second call is bit-identical, and nothing was counted as a reference by the top-k calls
    again = cache.lookup_topk(to_dev(wl.queries, dtype), k)
    torch.cuda.synchronize()
    assert torch.equal(again[0], out[0]) and torch.equal(again[1], out[1])


def test_lookup_topk_degenerate_cases(siso, oracle):
    print("case: lookup_topk degenerate", flush=True)
    dim, K, k = 256, 20000, 6
    wl = W.c2_mid(n_clusters=64, per_cluster=(K + 63) // 64, n_queries=40, dim=dim, sigma=0.3, seed=312)
    wl.centroids = wl.centroids[:K].copy()
    wl.centroids[100:400] = wl.centroids[50]               # 301 equal rows: more than the list of the second pass holds
    c = wl.centroids_f32().copy()
    c[10] = 0.0                                            # a centroid without length: similarity 0
    c[11, 3] = np.nan                                      # never chosen
    c[12] *= 7.0
    keep = wl.centroids.copy()
    wl.centroids = W.f32_to_bf16_bits(c)
    wl.centroids[100:400] = keep[100:400]
    wl.centroids[50] = keep[50]
    q = wl.queries_f32().copy()
    q[0] = 0.0                                             # similarity 0 to everything: rows 0 .. k-1
    q[1, 5] = np.nan
    q[2, 7] = np.inf
    q[3] *= 250.0
    q[4] = W.bf16_bits_to_f32(wl.centroids[50])            # the equal rows tie for the first 301 ranks
    wl.queries = W.f32_to_bf16_bits(q)
    cache = siso.SisoCache(dim, K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    oc = oracle.OracleCache(dim, K, "bf16")
    oc.load(wl.centroids)
    out = cache.lookup_topk(to_dev(wl.queries, "bf16"), k)
    ora = oc.lookup_topk(wl.queries, k)
    check_topk(out, ora, "bf16", "degenerate")
    gi = out[0].cpu().numpy()
    assert gi[0].tolist() == [0, 1, 2, 3, 4, 5] and (gi[1] == -1).all() and (gi[2] == -1).all()
    assert gi[4].tolist() == [50, 100, 101, 102, 103, 104]
    # more than the cache holds; an empty cache; bad k
    small = siso.SisoCache(dim, 8, siso.BF16)
    small.load(to_dev(wl.centroids[:3], "bf16"))
    si, ss = small.lookup_topk(to_dev(wl.queries[5:9], "bf16"), 5)
    so = oracle.OracleCache(dim, 8, "bf16")
    so.load(wl.centroids[:3])
    check_topk((si, ss), so.lookup_topk(wl.queries[5:9], 5), "bf16", "k beyond the cache")
    assert (si[:, 3:] == -1).all() and torch.isneginf(ss[:, 3:]).all()
    empty = siso.SisoCache(dim, 8, siso.BF16)
    ei, es = empty.lookup_topk(to_dev(wl.queries[5:9], "bf16"), 2)
    assert (ei == -1).all() and torch.isneginf(es).all()
    for bad in (0, 33):
        with pytest.raises(siso.SisoError):
            cache.lookup_topk(to_dev(wl.queries, "bf16"), bad)
    cache.lookup_topk(to_dev(wl.queries[:0], "bf16"), 3)


def test_lookup_topk_mid_size(siso, oracle):
    """65,536 centroids x 768, 4,096 queries (the mid-size workload), k = 8: the whole batch on the GPU, 128
    sampled queries through the oracle."""
    print("case: lookup_topk c2_mid", flush=True)
    wl = W.c2_mid()
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    out = cache.lookup_topk(to_dev(wl.queries, "bf16"), 8)
    torch.cuda.synchronize()
    rows = np.arange(0, wl.n, 32)
    oc = oracle.OracleCache(wl.dim, wl.K, "bf16")
    oc.load(wl.centroids)
    st = check_topk((out[0][rows], out[1][rows]), oc.lookup_topk(wl.queries[rows], 9), "bf16", "c2 top-8")
    print(f"  {st}", flush=True)
    assert st["clear"] >= 80 and st["same"] > 0.98 and st["max_err"] < 1e-4
    gi = out[0].cpu().numpy()
    near = wl.planted >= 0
    # queries next to a centroid: their own cluster's 16 members fill the ranks
    assert (wl.cluster_of[gi[near]] == wl.cluster_of[wl.planted[near]][:, None]).mean() > 0.995
    one = cache.lookup(to_dev(wl.queries, "bf16"), 0.85)
    assert torch.equal(one[0], out[0][:, 0].contiguous())

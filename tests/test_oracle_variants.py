"""Pins for the oracle's lookup variants: the k closest centroids, and one lookup judged against several
thresholds.  CPU only.  Closed-form cosines of plane vectors, an independent float64 route through numpy
(matmul + stable argsort), planted exact duplicates, the degenerate cases."""

import math
import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "topk_hand_computed.txt")


def bf(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def plane(angle_deg, length):
    d = f32([math.cos(math.radians(angle_deg)), math.sin(math.radians(angle_deg))])
    return d * np.float32(length)


def read_golden():
    cents, queries = [], []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.startswith("cent"):
            _, i, a, l = line.split()
            cents.append(plane(float(a), float(l)))
        else:
            head, order, sims = line.split("|")
            _, a, l = head.split()
            queries.append((plane(float(a), float(l)), [int(t) for t in order.split()], [float(t) for t in sims.split()]))
    return f32(cents), queries


def numpy_topk(cents64, qs64, k):
    """Independent route: normalise, one float64 matmul, stable argsort of the negated similarities (equal
    values keep their index order)."""
    S = (qs64 / np.linalg.norm(qs64, axis=1, keepdims=True)) @ (cents64 / np.linalg.norm(cents64, axis=1, keepdims=True)).T
    order = np.argsort(-S, axis=1, kind="stable")[:, :k]
    return order, np.take_along_axis(S, order, axis=1)


def test_topk_closed_form_plane_vectors(oracle):
    cents, queries = read_golden()
    assert len(cents) == 6 and len(queries) == 3
    oc = oracle.OracleCache(2, 8, "f32")
    oc.load(cents)
    for q, order, sims in queries:
        for k in (1, 2, 3, 6):
            idx, sim = oc.lookup_topk(f32([q]), k)
            assert idx[0].tolist() == order[:k]
            assert np.allclose(sim[0], sims[:k], rtol=0, atol=1e-7)   # coordinates are rounded to float32
        idx, sim = oc.lookup_topk(f32([q]), 3)
        if 2 in idx[0] and 4 in idx[0]:
            a, b = list(idx[0]).index(2), list(idx[0]).index(4)
            assert sim[0][a] == sim[0][b] and a + 1 == b              # the exact tie: lower index first


def test_topk_more_than_the_cache_holds_and_degenerate_queries(oracle):
    cents, queries = read_golden()
    oc = oracle.OracleCache(2, 8, "f32")
    oc.load(cents)
    idx, sim = oc.lookup_topk(f32([queries[0][0], [0.0, 0.0], [np.nan, 1.0], [np.inf, 1.0]]), 9)
    assert idx[0].tolist() == queries[0][1] + [-1, -1, -1] and np.all(np.isneginf(sim[0][6:]))
    # a query without length has similarity 0 to everything: all tie, index order
    assert idx[1].tolist() == [0, 1, 2, 3, 4, 5, -1, -1, -1] and np.all(sim[1][:6] == 0.0)
    for r in (2, 3):
        assert np.all(idx[r] == -1) and np.all(np.isnan(sim[r]))
    # a centroid holding a NaN is never chosen; one without length has similarity 0
    c2 = cents.copy()
    c2[0] = [np.nan, 1.0]
    c2[3] = [0.0, 0.0]
    oc.load(c2)
    idx, sim = oc.lookup_topk(f32([queries[1][0]]), 6)      # query at 180 degrees
    assert idx[0].tolist() == [1, 3, 2, 4, 5, -1]           # 6e-17 (90 degrees) > 0 (no length) > -0.5, -0.5, -0.64
    empty = oracle.OracleCache(2, 4, "f32")
    idx, sim = empty.lookup_topk(f32([[1.0, 0.0]]), 2)
    assert idx.tolist() == [[-1, -1]] and np.all(np.isneginf(sim))


@pytest.mark.parametrize("dtype,dim,K,n,k", [("bf16", 64, 500, 40, 5), ("f32", 48, 300, 25, 16), ("bf16", 128, 90, 10, 32)])
def test_topk_against_numpy_route(oracle, dtype, dim, K, n, k):
    wl = W.c2_mid(n_clusters=16, per_cluster=(K + 15) // 16, n_queries=n, dim=dim, dtype=dtype, sigma=0.4, seed=201)
    wl.centroids = wl.centroids[:K].copy()
    wl.centroids[7] = wl.centroids[3]          # exact duplicates: ties by index
    wl.centroids[K - 1] = wl.centroids[3]
    oc = oracle.OracleCache(dim, K, dtype)
    oc.load(wl.centroids)
    idx, sim = oc.lookup_topk(wl.queries, k)
    want_i, want_s = numpy_topk(wl.centroids_f32().astype(np.float64), wl.queries_f32().astype(np.float64), k)
    assert np.abs(sim - want_s).max() < 1e-12
    # same order wherever neighbouring similarities are not within rounding of each other (or exactly tied)
    for q in range(n):
        for r in range(k):
            if idx[q, r] != want_i[q, r]:
                assert abs(want_s[q, r] - sim[q, r]) < 1e-12
    assert (idx == want_i).mean() > 0.99
    # every row: non-increasing, no index twice, rank 1 is the plain lookup
    assert np.all(np.diff(sim, axis=1) <= 0)
    assert all(len(set(r)) == k for r in idx.tolist())
    one = oracle.lookup_rows(wl.centroids, wl.queries, 0.5, dtype)
    assert np.array_equal(idx[:, 0], one[0]) and np.array_equal(sim[:, 0], one[1])
    assert np.array_equal(sim[:, 1], one[3])   # rank 2 is what the lookup reports as the runner-up
    # the duplicates of centroid 3 appear together, in index order
    for q in range(n):
        row = idx[q].tolist()
        if 3 in row and row.index(3) + 2 < k:
            p = row.index(3)
            assert row[p:p + 3] == [3, 7, K - 1]


def test_topk_is_invariant_under_query_scaling_and_equivariant_under_permutation(oracle):
    wl = W.c2_mid(n_clusters=8, per_cluster=10, n_queries=12, dim=32, dtype="f32", sigma=0.5, seed=202)
    oc = oracle.OracleCache(32, wl.K, "f32")
    oc.load(wl.centroids)
    idx, sim = oc.lookup_topk(wl.queries, 4)
    idx2, sim2 = oc.lookup_topk(f32(wl.queries * np.float32(8.0)), 4)   # power of two: exact
    assert np.array_equal(idx, idx2) and np.array_equal(sim, sim2)
    perm = np.random.default_rng(5).permutation(wl.K)
    oc.load(wl.centroids[perm])
    idx3, sim3 = oc.lookup_topk(wl.queries, 4)
    assert np.array_equal(perm[idx3], idx) and np.array_equal(sim3, sim)


# ------------------------------------------------------------ several thresholds at once
def test_multi_threshold_flags_closed_form_and_strictness(oracle):
    # unit basis vectors: the query (3, 4) has cosines 0.6 and 0.8 exactly to the two axes... as rounded doubles:
    # 4/5 = 0.8 and the threshold float32(0.8) = 0.800000011920929 > 0.8, so that threshold is a miss
    oc = oracle.OracleCache(2, 4, "f32")
    oc.load(f32([[1.0, 0.0], [0.0, 1.0]]))
    th = f32([0.5, 0.75, 0.8, 0.875, -1.0, 1.0])
    idx, sim, hit, second = oc.lookup_multi(f32([[3.0, 4.0], [0.0, 2.0], [1.0, 0.0]]), th)
    assert idx.tolist() == [1, 1, 0] and sim[0] == 0.8 and second[0] == 0.6 and sim[1] == 1.0
    assert hit[0].tolist() == [1, 1, 0, 0, 1, 0]
    assert hit[1].tolist() == [1, 1, 1, 1, 1, 0]          # sim = 1 is not above the threshold 1: strict
    assert hit[2].tolist() == [1, 1, 1, 1, 1, 0]
    # exactly representable: (1,1,1,1) against the first axis has cosine 1/2; the threshold 0.5 itself is a miss,
    # the float just below it a hit
    oc4 = oracle.OracleCache(4, 2, "f32")
    oc4.load(f32([[1.0, 0.0, 0.0, 0.0]]))
    below = np.nextafter(np.float32(0.5), np.float32(0.0))
    idx, sim, hit, _ = oc4.lookup_multi(f32([[1.0, 1.0, 1.0, 1.0]]), f32([0.5, below]))
    assert sim[0] == 0.5 and hit[0].tolist() == [0, 1]


def test_multi_threshold_against_numpy_route_and_monotone(oracle):
    wl = W.c2_mid(n_clusters=32, per_cluster=8, n_queries=300, dim=64, dtype="bf16", sigma=0.5, seed=203)
    oc = oracle.OracleCache(64, wl.K, "bf16")
    oc.load(wl.centroids)
    th = f32([0.92, 0.75, 0.85, 0.6, 0.98])
    idx, sim, hit, second = oc.lookup_multi(wl.queries, th)
    c64, q64 = wl.centroids_f32().astype(np.float64), wl.queries_f32().astype(np.float64)
    S = (q64 / np.linalg.norm(q64, axis=1, keepdims=True)) @ (c64 / np.linalg.norm(c64, axis=1, keepdims=True)).T
    top = S.max(axis=1)
    assert np.abs(top - sim).max() < 1e-12
    want = (top[:, None] > th.astype(np.float64)[None, :]).astype(np.uint8)
    near = np.abs(top[:, None] - th.astype(np.float64)[None, :]) < 1e-12
    assert np.array_equal(hit[~near], want[~near])
    # the hit set shrinks as the threshold grows (hit ratio against threshold, section 3.3)
    order = np.argsort(th)
    assert np.all(np.diff(hit[:, order].astype(int), axis=1) <= 0)
    assert 0 < hit[:, 0].sum() < hit[:, 3].sum()


def test_multi_threshold_counts_references_for_one_threshold_only(oracle):
    wl = W.c2_mid(n_clusters=16, per_cluster=4, n_queries=100, dim=32, dtype="f32", sigma=0.4, seed=204)
    th = f32([0.6, 0.9])
    for count_index in (-1, 0, 1):
        oc = oracle.OracleCache(32, wl.K, "f32")
        oc.load(wl.centroids)
        idx, sim, hit, _ = oc.lookup_multi(wl.queries, th, count_index)
        acc = oc.export_meta()[1]
        if count_index < 0:
            assert acc.sum() == 0
        else:
            assert np.array_equal(acc, np.bincount(idx[hit[:, count_index] == 1], minlength=wl.K))
    assert hit[:, 0].sum() > hit[:, 1].sum() > 0

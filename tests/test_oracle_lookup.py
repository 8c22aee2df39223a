"""Pins for the oracle's lookup (cosine, top-1, hit test).  CPU only.

Each test fixes the oracle against something other than itself: hand-computed
cosines, geometric invariants, an independent float64 route through numpy's
matmul, planted structure in the data."""

import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "cosine_hand_computed.txt")


def bf(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def numpy_route(cents64, qs64):
    """Independent route: normalise first, one float64 matmul, library argmax."""
    cn = np.linalg.norm(cents64, axis=1, keepdims=True)
    qn = np.linalg.norm(qs64, axis=1, keepdims=True)
    S = (qs64 / qn) @ (cents64 / cn).T
    return S


# ----------------------------------------------------------------- cosine
def test_golden_hand_computed_cosines(oracle):
    rows = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                rows.append([float(t) for t in line.split()])
    assert len(rows) >= 10
    for ax, ay, bx, by, want, tol in rows:
        idx, sim, hit, _ = oracle.lookup_rows(f32([[bx, by]]), f32([[ax, ay]]), 0.0, "f32")
        assert idx[0] == 0
        assert abs(sim[0] - want) <= tol, (ax, ay, bx, by, sim[0], want)
        assert hit[0] == (1 if want > 0.0 else 0)


def test_basis_vectors_give_identity(oracle):
    d = 24
    eye = np.eye(d, dtype=np.float32) * np.arange(1, d + 1, dtype=np.float32)[:, None]  # any lengths
    for dtype, conv in (("f32", f32), ("bf16", bf)):
        idx, sim, hit, second = oracle.lookup_rows(conv(eye), conv(eye[::-1].copy()), 0.5, dtype)
        assert np.array_equal(idx, np.arange(d)[::-1])
        assert np.all(sim == 1.0)
        assert np.all(second == 0.0)
        assert np.all(hit == 1)


def test_scale_invariance_and_bound(oracle):
    r = np.random.default_rng(1)
    cents = f32(r.standard_normal((50, 16)))
    qs = f32(r.standard_normal((20, 16)))
    i0, s0, _, _ = oracle.lookup_rows(cents, qs, 0.0, "f32")
    i1, s1, _, _ = oracle.lookup_rows(f32(cents * 4.0), f32(qs * 0.125), 0.0, "f32")  # exact scalings
    assert np.array_equal(i0, i1)
    assert np.allclose(s0, s1, rtol=0, atol=1e-15)
    assert np.all(np.abs(s0) <= 1.0 + 1e-15)


def test_bf16_inputs_are_widened_exactly(oracle):
    """A bf16 input must behave exactly like the float32 vector with the same value."""
    r = np.random.default_rng(2)
    cents = W.bf16_bits_to_f32(bf(r.standard_normal((64, 32))))
    qs = W.bf16_bits_to_f32(bf(r.standard_normal((16, 32))))
    a = oracle.lookup_rows(bf(cents), bf(qs), 0.3, "bf16")
    b = oracle.lookup_rows(f32(cents), f32(qs), 0.3, "f32")
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ------------------------------------------------------------------ top-1
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_top1_matches_independent_float64_route(oracle, dtype):
    wl = W.c2_mid(n_clusters=32, per_cluster=8, n_queries=96, dim=64, dtype=dtype, seed=11)
    idx, sim, hit, second = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, dtype)
    S = numpy_route(wl.centroids_f32().astype(np.float64), wl.queries_f32().astype(np.float64))
    assert np.array_equal(idx, np.argmax(S, axis=1))
    assert np.allclose(sim, S.max(axis=1), rtol=0, atol=1e-14)
    part = np.sort(S, axis=1)
    assert np.allclose(second, part[:, -2], rtol=0, atol=1e-14)
    # invariant: the returned similarity is the maximum over all centroids
    assert np.all(sim[:, None] >= S - 1e-14)
    assert np.array_equal(hit, (S.max(axis=1) > np.float64(np.float32(0.85))).astype(np.uint8))


def test_planted_neighbours_are_found(oracle):
    wl = W.c2_mid(n_clusters=64, per_cluster=16, n_queries=128, dim=128, seed=12)
    idx, sim, hit, second = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    near = wl.planted >= 0
    assert near.sum() > 60 and (~near).sum() > 20
    assert np.array_equal(idx[near], wl.planted[near])
    assert np.all(hit[near] == 1) and np.all(hit[~near] == 0)
    assert np.all(sim[near] > 0.99) and np.all(sim[~near] < 0.6)


def test_lowest_index_wins_ties(oracle):
    r = np.random.default_rng(3)
    cents = f32(r.standard_normal((40, 12)))
    cents[31] = cents[7]
    cents[19] = cents[7]
    qs = f32(np.stack([cents[7], cents[7] + 1e-3 * r.standard_normal(12).astype(np.float32)]))
    idx, sim, _, second = oracle.lookup_rows(cents, qs, 0.0, "f32")
    assert idx[0] == 7 and idx[1] == 7
    assert second[0] == sim[0]  # the duplicates tie exactly, and the runner-up reports it


def test_permutation_equivariance_and_self_query(oracle):
    wl = W.c1_tiny(n_clusters=8, per_cluster=8, n_queries=32, dim=48, seed=13)
    perm = np.random.default_rng(4).permutation(wl.K)
    i0, s0, _, _ = oracle.lookup_rows(wl.centroids, wl.queries, 0.8, "f32")
    i1, s1, _, _ = oracle.lookup_rows(wl.centroids[perm].copy(), wl.queries, 0.8, "f32")
    assert np.array_equal(perm[i1], i0)
    assert np.array_equal(s0, s1)
    i2, s2, _, _ = oracle.lookup_rows(wl.centroids, wl.centroids, 0.8, "f32")
    assert np.array_equal(i2, np.arange(wl.K))
    assert np.allclose(s2, 1.0, rtol=0, atol=1e-15)


# -------------------------------------------------------------------- hit
def test_hit_is_strict_and_monotone_in_threshold(oracle):
    e = f32([[1.0, 0.0, 0.0]])
    for th, want in ((1.0, 0), (np.nextafter(np.float32(1.0), np.float32(0.0)), 1), (-2.0, 1), (1.5, 0)):
        _, sim, hit, _ = oracle.lookup_rows(e, e, float(th), "f32")
        assert sim[0] == 1.0 and hit[0] == want
    # similarity exactly equal to a representable threshold is a miss (strict ">")
    _, sim, hit, _ = oracle.lookup_rows(f32([[3.0, 4.0]]), f32([[5.0, 0.0]]), 0.6, "f32")
    assert sim[0] == 0.6  # 15/25 in double is the double nearest 0.6
    assert hit[0] == 0    # (double)(float)0.6 is above the double 0.6
    _, sim, hit, _ = oracle.lookup_rows(f32([[1.0, 1.0, 1.0, 1.0]]), f32([[1.0, 0.0, 0.0, 0.0]]), 0.5, "f32")
    assert sim[0] == 0.5 and hit[0] == 0
    _, _, hit, _ = oracle.lookup_rows(f32([[1.0, 1.0, 1.0, 1.0]]), f32([[1.0, 0.0, 0.0, 0.0]]), 0.4999999, "f32")
    assert hit[0] == 1

    wl = W.c2_mid(n_clusters=32, per_cluster=8, n_queries=200, dim=64, sigma=0.5, seed=14)
    prev = None
    ratios = []
    for th in (0.60, 0.70, 0.80, 0.86, 0.92, 0.98):  # the sweep range of the threshold-to-hit-ratio table
        i, s, hit, _ = oracle.lookup_rows(wl.centroids, wl.queries, th, "bf16")
        if prev is not None:
            assert np.all(hit <= prev)  # the hit set shrinks as the threshold grows (section 3.3)
        prev = hit
        ratios.append(hit.mean())
    assert ratios[0] > ratios[-1]


# ------------------------------------------------------------ special cases
def test_zero_nan_and_empty(oracle):
    cents = f32([[1.0, 0.0], [0.0, 0.0], [np.nan, 1.0], [-1.0, 0.0]])
    qs = f32([[0.0, 0.0], [np.nan, 1.0], [np.inf, 0.0], [-2.0, 0.0], [0.0, 1.0]])
    idx, sim, hit, second = oracle.lookup_rows(cents, qs, -0.5, "f32")
    # zero query: every similarity is 0, lowest non-NaN index wins
    assert idx[0] == 0 and sim[0] == 0.0 and hit[0] == 1
    # non-finite queries
    for i in (1, 2):
        assert idx[i] == -1 and np.isnan(sim[i]) and hit[i] == 0
    # the NaN centroid never wins; the zero centroid scores 0
    assert idx[3] == 3 and sim[3] == 1.0
    assert idx[4] == 0 and sim[4] == 0.0 and second[4] == 0.0
    # empty cache
    idx, sim, hit, second = oracle.lookup_rows(np.zeros((0, 2), np.float32), qs[3:], 0.1, "f32")
    assert np.all(idx == -1) and np.all(np.isneginf(sim)) and np.all(hit == 0)
    # no queries
    idx, sim, hit, _ = oracle.lookup_rows(cents, np.zeros((0, 2), np.float32), 0.1, "f32")
    assert idx.shape == (0,)


def test_cache_object_lookup_equals_stateless(oracle):
    wl = W.c2_mid(n_clusters=16, per_cluster=8, n_queries=40, dim=32, seed=15)
    oc = oracle.OracleCache(wl.dim, wl.K + 5, "bf16")
    oc.load(wl.centroids)
    assert oc.count == wl.K
    a = oc.lookup(wl.queries, 0.85)
    b = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    cents, means, sizes = oc.export()
    assert np.array_equal(cents, wl.centroids)  # stored verbatim
    assert np.all(sizes == 1)
    assert np.allclose(np.linalg.norm(means, axis=1), 1.0, atol=1e-15)

"""Pins for the oracle's cache replacement (Algorithm 1, section 4.2: MergeCentroids,
FilteringCentroids, UpdateCentroids) and for the access counts kept by lookups.  CPU only."""

import math
import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

INF = 0xFFFFFFFF
F = np.float32


def plane(angles_deg, dim=8):
    """unit vectors of the plane spanned by the first two axes"""
    a = np.deg2rad(np.asarray(angles_deg, dtype=np.float64))
    out = np.zeros((len(angles_deg), dim), np.float32)
    out[:, 0], out[:, 1] = np.cos(a), np.sin(a)
    return out


def golden_case():
    cur, repo = [], []
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "refresh_hand_worked.txt")):
        t = line.split("#")[0].split()
        if len(t) == 3:
            (cur if t[0] == "cur" else repo).append((float(t[1]), float(t[2])))
    return cur, repo


def make_cache(oracle, cur, capacity=16):
    cache = oracle.OracleCache(8, capacity, "f32")
    cache.load(plane([a for a, _ in cur]), np.array([int(s) for _, s in cur], np.int32))
    return cache


@pytest.mark.parametrize("M,want_angles,want_sizes,want_stats", [
    (3, [0, 90, 200], [7, 9, 5], (3, 1, 0)),
    (2, [0, 90], [7, 9], (3, 1, 1)),
    (1, [90], [9], (3, 1, 2)),
])
def test_refresh_hand_worked_example(oracle, M, want_angles, want_sizes, want_stats):
    cur, repo = golden_case()
    assert len(cur) == 2 and len(repo) == 4
    cache = make_cache(oracle, cur)
    merged, added, evicted, margin = cache.refresh(plane([a for a, _ in repo]), [s for _, s in repo], 0.9, M)
    assert (merged, added, evicted) == want_stats
    cents, _, _ = cache.export()
    assert np.allclose(cents, plane(want_angles), atol=1e-7)
    loc, acc = cache.export_meta()
    assert loc.tolist() == [F(s) / F(1.1) for s in want_sizes]  # one single-precision division by 1.1
    assert acc.tolist() == [0] * len(want_angles)
    assert margin == pytest.approx(math.cos(math.radians(10)) - 0.9, abs=1e-6)  # the closest call: 10 degrees


def test_refresh_is_sequential_and_takes_the_closest(oracle):
    # two repository rows 4 degrees apart, both far from the cache: the first joins, the second merges into it;
    # in the other order the other one survives
    cache = make_cache(oracle, [(0, 1)])
    cache.refresh(plane([120, 124]), [2, 3], 0.9, 8)
    cents, _, _ = cache.export()
    assert np.allclose(cents, plane([0, 120]), atol=1e-7)
    assert cache.export_meta()[0].tolist() == [F(1) / F(1.1), F(5) / F(1.1)]
    cache = make_cache(oracle, [(0, 1)])
    cache.refresh(plane([124, 120]), [3, 2], 0.9, 8)
    assert np.allclose(cache.export()[0], plane([0, 124]), atol=1e-7)
    # a row above the threshold for two centroids goes to the closest, not to the first:
    # cache at 0 and 30 degrees, repository row at 20 degrees (cos 20 = 0.94, cos 10 = 0.985)
    cache = make_cache(oracle, [(0, 1), (30, 1)])
    cache.refresh(plane([20]), [4], 0.9, 8)
    assert cache.export_meta()[0].tolist() == [F(1) / F(1.1), F(5) / F(1.1)]
    # equal cosines: the lowest index of C_new takes it (row at 15 degrees between 0 and 30)
    cache = make_cache(oracle, [(0, 1), (30, 1)])
    cache.refresh(plane([15]), [4], 0.9, 8)
    loc = cache.export_meta()[0].tolist()
    c15 = math.cos(math.radians(15))
    assert sorted(loc) == sorted([F(1) / F(1.1), F(5) / F(1.1)])  # one of the two took it ...
    a, b = float(plane([15])[0] @ plane([0])[0]), float(plane([15])[0] @ plane([30])[0])
    assert (loc[0] > loc[1]) == (a >= b)  # ... the closer one in the arithmetic of the stored values, index 0 on a tie


def test_refresh_reports_the_lead_of_the_closest_centroid(oracle):
    # cache at 0 and 30 degrees; rows at 20 degrees (closest 30 at cos 10, second 0 at cos 20) and at 2 degrees
    # (closest 0 at cos 2, second 30 at cos 28); a row at 100 degrees joins and does not count; margin: cos 10 - 0.9
    cache = make_cache(oracle, [(0, 1), (30, 1)])
    merged, added, evicted, margin, lead = cache.refresh(plane([20, 100, 2]), [1, 1, 1], 0.9, 8, want_gap=True)
    cosd = lambda a: math.cos(math.radians(a))
    assert (merged, added, evicted) == (2, 1, 0)
    assert abs(lead - (cosd(10) - cosd(20))) < 1e-7 and cosd(10) - cosd(20) < cosd(2) - cosd(28)
    assert abs(margin - (cosd(10) - 0.9)) < 1e-6
    # equal rows tie exactly and do not count: the lead is then the one over the next different cosine
    cache = make_cache(oracle, [(0, 1), (0, 1), (30, 1)])
    lead = cache.refresh(plane([5]), [1], 0.9, 8, want_gap=True)[4]
    assert abs(lead - (cosd(5) - cosd(25))) < 1e-7
    # without a merged row there is no lead
    cache = make_cache(oracle, [(0, 1)])
    assert cache.refresh(plane([90]), [1], 0.9, 8, want_gap=True)[4] == math.inf


def test_refresh_threshold_extremes_and_conservation(oracle):
    wl = W.c5_merge(n_groups=40, copies=4, dim=64, seed=5)
    cents = W.storage_to_f32(wl.centroids, "bf16")
    cur, repo = cents[:100], cents[100:]
    sizes = np.arange(1, repo.shape[0] + 1).astype(np.float32)
    # nothing exceeds a threshold above 1: every repository row joins
    c = oracle.OracleCache(64, 400, "f32")
    c.load(cur)
    assert c.refresh(repo, sizes, 1.5, 400)[:3] == (0, 60, 0)
    assert c.count == 160 and (c.export()[0][100:] == repo).all()  # joined rows are stored verbatim, in order
    loc, acc = c.export_meta()
    assert np.array_equal(loc[100:], sizes / F(1.1)) and (acc == 0).all()
    # the cache itself as repository: everything merges, nothing is added, cluster sizes add up
    c = oracle.OracleCache(64, 400, "f32")
    c.load(cur, np.full(100, 3, np.int32))
    assert c.refresh(cur, np.full(100, 2.0, np.float32), 0.999, 400)[:3] == (100, 0, 0)
    # (near-duplicates: a row's closest centroid is itself; its copies sit at cosine 0.999 or so)
    assert c.count == 100 and c.export_meta()[0].sum() == pytest.approx(500 / 1.1, rel=1e-6)
    # total cluster size is conserved by the merge step (before the decay) when nothing is evicted
    c = oracle.OracleCache(64, 400, "f32")
    c.load(cur)
    merged, added, evicted, _ = c.refresh(repo, sizes, 0.9, 400)
    assert merged + added == 60 and evicted == 0 and added == c.count - 100
    assert c.export_meta()[0].astype(np.float64).sum() * 1.1 == pytest.approx(100 + sizes.sum(), rel=1e-6)


def test_filtering_order_cluster_size_then_access_count_then_position(oracle):
    # five cached centroids 60 degrees apart... on different axes instead: orthogonal rows
    eye = np.eye(8, dtype=np.float32)
    c = oracle.OracleCache(8, 8, "f32")
    c.load(eye[:5], np.array([4, 2, 2, 2, 9], np.int32))
    # references: centroid 1 twice, centroid 3 once (queries = the rows themselves, threshold 0.5)
    c.lookup(eye[[1, 1, 3]], 0.5)
    assert c.export_meta()[1].tolist() == [0, 2, 0, 1, 0]
    # one new row (cluster size 2, access infinity); C_new has 6 rows; keep 2:
    # cluster size 2 goes first: access 0 (row 2), then 1 (row 3), then 2 (row 1), and the new row (infinity) last
    order = []
    for M in (5, 4, 3, 2):
        cc = oracle.OracleCache(8, 8, "f32")
        cc.load(eye[:5], np.array([4, 2, 2, 2, 9], np.int32))
        cc.lookup(eye[[1, 1, 3]], 0.5)
        cc.refresh(eye[5:6], [2.0], 0.9, M)
        order.append([int(np.argmax(row)) for row in cc.export()[0]])
    assert order == [[0, 1, 3, 4, 5], [0, 1, 4, 5], [0, 4, 5], [0, 4]]
    # equal cluster size and access count: the first in the order of C_new goes
    cc = oracle.OracleCache(8, 8, "f32")
    cc.load(eye[:4])
    cc.refresh(eye[:0], np.zeros(0, np.float32), 0.9, 2)
    assert [int(np.argmax(row)) for row in cc.export()[0]] == [2, 3]


def test_access_counts_follow_hits_and_saturate(oracle):
    eye = np.eye(8, dtype=np.float32)
    c = oracle.OracleCache(8, 8, "f32")
    c.load(eye[:3])
    q = eye[[0, 0, 2, 5]]  # two hits on 0, one on 2, one miss (cosine 0 with everything)
    c.lookup(q, 0.5)
    c.lookup(q[:1], 0.5)
    assert c.export_meta()[1].tolist() == [3, 0, 1]
    c.lookup(q, 1.0)  # strict: cosine 1 is no hit at threshold 1
    assert c.export_meta()[1].tolist() == [3, 0, 1]
    # a centroid that just joined has access_count infinity until the next refresh resets it
    c.refresh(eye[4:5], [1.0], 0.9, 8)
    assert c.export_meta()[1].tolist() == [0, 0, 0, 0]
    # test lookups of the T2H table are no references
    c.t2h(q, np.array([0.5], np.float32))
    assert c.export_meta()[1].tolist() == [0, 0, 0, 0]


def test_refresh_rejects_bad_input(oracle):
    eye = np.eye(8, dtype=np.float32)
    c = oracle.OracleCache(8, 4, "f32")
    c.load(eye[:2])
    bad = eye[2:3].copy()
    bad[0, 0] = np.nan
    with pytest.raises(RuntimeError):
        c.refresh(bad, [1.0], 0.9, 4)
    with pytest.raises(RuntimeError):
        c.refresh(eye[2:3], [0.0], 0.9, 4)  # a cluster has at least one member
    with pytest.raises(RuntimeError):
        c.refresh(eye[2:3], [1.0], 0.9, 5)  # more survivors than the cache holds
    assert c.count == 2  # nothing changed

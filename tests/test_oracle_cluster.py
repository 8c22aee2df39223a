"""Pins for the oracle's clustering (section 4.1: community detection at the clustering threshold,
centroid = average of the cluster, cluster_size = number of members).  CPU only."""

import math
import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W


def plane(angles_deg, dim=8):
    a = np.deg2rad(np.asarray(angles_deg, dtype=np.float64))
    out = np.zeros((len(angles_deg), dim), np.float32)
    out[:, 0], out[:, 1] = np.cos(a), np.sin(a)
    return out


def golden():
    angles, cases = [], {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "cluster_hand_worked.txt")):
        t = line.split("#")[0].split()
        if not t:
            continue
        if t[0] == "v":
            assert int(t[1]) == len(angles)
            angles.append(float(t[2]))
        elif t[0] == "rep_case":
            cases["rep"] = {"angles": [float(v) for v in t[2:t.index("rep")]], "rep": int(t[t.index("rep") + 1]),
                            "gap": float(t[t.index("gap") + 1])}
        elif t[0] == "min_size":
            case = cases.setdefault(int(t[1]), {})
            rest, key = t[2:], None
            for w in rest:
                if w in ("labels", "seeds", "centroid_angles", "mean_lengths"):
                    key = w
                    case[key] = []
                else:
                    case[key].append(float(w))
    return angles, cases


@pytest.mark.parametrize("min_size", [2, 1])
def test_cluster_hand_worked_example(oracle, min_size):
    angles, cases = golden()
    want = cases[min_size]
    cache = oracle.OracleCache(8, 16, "f32")
    labels, seeds, margin = cache.cluster(plane(angles), 0.94, min_size)
    assert labels.tolist() == [int(v) for v in want["labels"]]
    assert seeds.tolist() == [int(v) for v in want["seeds"]]
    cents, means, sizes = cache.export()
    assert np.allclose(cents, plane(want["centroid_angles"]), atol=1e-6)
    assert sizes.tolist() == [labels.tolist().count(k) for k in range(len(seeds))]
    loc, acc = cache.export_meta()
    assert loc.tolist() == [float(s) for s in sizes] and acc.tolist() == [0] * len(seeds)
    if "mean_lengths" in want:
        assert np.allclose(np.linalg.norm(means, axis=1), want["mean_lengths"], atol=1e-6)
    # the closest call of the example: 20 degrees between 110 and 130 (and 15 degrees on the other side)
    assert margin == pytest.approx(min(0.94 - math.cos(math.radians(20)), math.cos(math.radians(15)) - 0.94), abs=1e-6)


def test_threshold_test_is_strict(oracle):
    # <(1,1,1,1), (1,1,1,-1)> = 2 and both lengths are 2: the cosine is exactly 0.5
    x = np.array([[1, 1, 1, 1], [1, 1, 1, -1]], np.float32)
    cache = oracle.OracleCache(4, 4, "f32")
    labels, _, margin = cache.cluster(x, 0.5, 1)
    assert labels.tolist() == [0, 1] and margin == 0.0
    labels, _, _ = cache.cluster(x, np.nextafter(np.float32(0.5), np.float32(0)), 1)
    assert labels.tolist() == [0, 0]


def brute_force(x64, theta, min_size):
    """the same scheme through sets and a sort, for small inputs"""
    n = len(x64)
    u = x64 / np.linalg.norm(x64, axis=1, keepdims=True)
    s = u @ u.T
    near = [set(np.flatnonzero(s[i] > theta).tolist()) | {i} for i in range(n)]
    taken, clusters, seeds = set(), [], []
    for i in sorted(range(n), key=lambda i: (-len(near[i]), i)):
        if len(near[i]) < min_size:
            continue
        rest = near[i] - taken
        if len(rest) >= min_size:
            clusters.append(sorted(rest))
            seeds.append(i)
            taken |= rest
    labels = np.full(n, -1)
    for k, members in enumerate(clusters):
        labels[members] = k
    return labels, seeds, clusters, u


@pytest.mark.parametrize("dtype,min_size,seed", [("f32", 1, 3), ("bf16", 2, 4), ("bf16", 3, 5), ("f32", 4, 6)])
def test_cluster_against_brute_force_and_invariants(oracle, dtype, min_size, seed):
    x, topic = W.query_log_chains(n_chains=6, chain_len=5, n_noise=20, dim=64, dtype=dtype, seed=seed, sigma=0.08)
    n = len(x)
    cache = oracle.OracleCache(64, n, dtype)
    theta = np.float32(0.86)
    labels, seeds, margin = cache.cluster(x, theta, min_size)
    x64 = W.storage_to_f32(x, dtype).astype(np.float64)
    want, want_seeds, clusters, u = brute_force(x64, float(theta), min_size)
    assert labels.tolist() == want.tolist() and seeds.tolist() == want_seeds
    assert len(seeds) > 6 and (min_size == 1 or (labels < 0).any())
    # invariants that hold whatever the order was
    for k, members in enumerate(clusters):
        assert len(members) >= min_size
        assert all(m == seeds[k] or u[m] @ u[seeds[k]] > theta for m in members)   # a star around its seed
    cents, means, sizes = cache.export()
    assert sizes.tolist() == [len(m) for m in clusters]
    for k, members in enumerate(clusters):
        m = u[members].mean(axis=0)
        assert np.allclose(means[k], m, atol=1e-12)
        c = W.storage_to_f32(cents[k:k + 1], dtype)[0]
        assert np.allclose(c, m / np.linalg.norm(m), atol=4e-3 if dtype == "bf16" else 1e-7)
    s = (u @ u.T)[np.triu_indices(n, 1)]
    assert margin == pytest.approx(np.abs(s - float(theta)).min(), abs=1e-12)


def test_separate_topics_come_back_as_they_were_made(oracle):
    wl = W.c5_merge(n_groups=40, copies=6, dim=64, dtype="bf16", seed=17)
    cache = oracle.OracleCache(64, 64, "bf16")
    labels, seeds, _ = cache.cluster(wl.centroids, 0.86, 2)
    assert len(seeds) == 40 and (labels >= 0).all()
    for g in range(40):
        assert len(set(labels[wl.cluster_of == g].tolist())) == 1
    assert len(set(labels.tolist())) == 40
    # equal sizes: the clusters come in the order of their first members
    firsts = [int(np.flatnonzero(labels == k)[0]) for k in range(40)]
    assert firsts == sorted(firsts) and seeds.tolist() == firsts


def test_extreme_thresholds(oracle):
    x = W.uniform_directions(5, 1, 50, 32)
    cache = oracle.OracleCache(32, 64, "f32")
    labels, seeds, _ = cache.cluster(x, 1.0, 1)               # nothing exceeds 1: everyone alone, in order
    assert labels.tolist() == list(range(50)) and seeds.tolist() == list(range(50))
    cents, _, sizes = cache.export()
    assert np.allclose(cents, x, atol=1e-6) and sizes.tolist() == [1] * 50
    labels, seeds, _ = cache.cluster(x, 1.0, 2)
    assert (labels == -1).all() and len(seeds) == 0 and cache.count == 0
    labels, seeds, _ = cache.cluster(x, -1.5, 3)              # everything is a neighbour: one cluster, seed 0
    assert (labels == 0).all() and seeds.tolist() == [0]
    _, means, sizes = cache.export()
    assert sizes.tolist() == [50]
    assert np.allclose(means[0], x.astype(np.float64).mean(axis=0), atol=1e-7)


def test_cluster_rejects_what_it_cannot_place(oracle):
    cache = oracle.OracleCache(8, 2, "f32")
    x = plane([0, 90, 180])
    with pytest.raises(RuntimeError):
        cache.cluster(x, 0.9, 1)                              # three clusters, room for two
    bad = x.copy()
    bad[1] = 0
    big = oracle.OracleCache(8, 8, "f32")
    with pytest.raises(RuntimeError):
        big.cluster(bad, 0.9, 1)                              # a vector without a direction
    bad[1, 0] = np.nan
    with pytest.raises(RuntimeError):
        big.cluster(bad, 0.9, 1)


def test_representative_hand_worked(oracle):
    angles, cases = golden()
    # cluster 1 of the first example: 0, 15, 30 degrees -> the middle one, ahead by 1 - cos 15 degrees
    cache = oracle.OracleCache(8, 16, "f32")
    labels, seeds, _, rep, gap = cache.cluster(plane(angles), 0.94, 2, representatives=True)
    assert rep[1] == 1 and gap[1] == pytest.approx(1 - math.cos(math.radians(15)), abs=1e-6)
    assert all(labels[rep[k]] == k for k in range(len(seeds)))
    # the lopsided example
    c = cases["rep"]
    labels, seeds, _, rep, gap = cache.cluster(plane(c["angles"]), 0.94, 2, representatives=True)
    assert labels.tolist() == [0, 0, 0] and rep.tolist() == [c["rep"]]
    assert gap[0] == pytest.approx(c["gap"], abs=2e-5)
    # a cluster of one stands for itself; two exact copies: the lower index
    labels, seeds, _, rep, gap = cache.cluster(plane([10, 100, 100]), 0.94, 1, representatives=True)
    assert labels.tolist() == [1, 0, 0] and rep.tolist() == [1, 0] and gap[0] == 0.0 and np.isinf(gap[1])


def test_representative_against_numpy(oracle):
    x, _ = W.query_log_chains(n_chains=8, dim=64, dtype="bf16", seed=12, sigma=0.1)
    cache = oracle.OracleCache(64, len(x), "bf16")
    labels, seeds, _, rep, gap = cache.cluster(x, 0.86, 2, representatives=True)
    u = W.storage_to_f32(x, "bf16").astype(np.float64)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    for k in range(len(seeds)):
        mem = np.flatnonzero(labels == k)
        m = u[mem].mean(axis=0)
        cs = np.sort(u[mem] @ (m / np.linalg.norm(m)))
        best = mem[np.argmax(u[mem] @ m)]
        assert rep[k] == best or gap[k] < 1e-12
        assert gap[k] == pytest.approx(cs[-1] - cs[-2], abs=1e-12)


def test_clusters_are_stars_not_cliques(oracle):
    """What Table 2 reports for the method: members of a cluster are close to one common vector, not
    necessarily to each other, so the smallest similarity inside a cluster lies below the clustering
    threshold (0.80 against 0.86 in the paper) while the average stays high."""
    x, _ = W.query_log_chains(n_chains=12, dim=128, dtype="bf16", seed=21)
    cache = oracle.OracleCache(128, len(x), "bf16")
    labels, seeds, _ = cache.cluster(x, 0.86, 2)
    u = W.storage_to_f32(x, "bf16").astype(np.float64)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    inside = []
    for k in range(len(seeds)):
        mem = np.flatnonzero(labels == k)
        s = (u[mem] @ u[mem].T)[np.triu_indices(len(mem), 1)]
        inside.append(s)
        founder = seeds[k]
        assert all(u[m] @ u[founder] > 0.86 for m in mem if m != founder)
    inside = np.concatenate(inside)
    assert 0.70 < inside.min() < 0.86 and inside.mean() > 0.90

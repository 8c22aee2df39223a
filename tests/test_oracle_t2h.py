"""Pins for the oracle's threshold-to-hit-ratio table, the M/D/1 waiting time and the SLO-aware
choice of the retrieval threshold (section 4.3, equations 1 and 2).  CPU only."""

import math
import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))


def golden_rows():
    rows = []
    for line in open(os.path.join(HERE, "golden", "md1_wait_hand_computed.txt")):
        line = line.split("#")[0].strip()
        if line:
            rows.append([float(x) for x in line.split()])
    return rows


def test_md1_wait_matches_hand_computed_values(oracle):
    rows = golden_rows()
    assert len(rows) >= 6
    for L, lam, h, want in rows:
        assert oracle.md1_wait(L, lam, h) == pytest.approx(want, rel=1e-14, abs=0)


def test_md1_wait_limits_and_monotonicity(oracle):
    assert oracle.md1_wait(3.0, 0.0, 0.25) == 2.25  # no load: the bare serving time
    assert oracle.md1_wait(1.0, 1.0, 0.0) == math.inf  # rho = 1: unstable
    assert oracle.md1_wait(1.0, 2.0, 0.25) == math.inf  # rho > 1
    assert oracle.md1_wait(1.0, 2.0, 0.75) < math.inf  # enough hits make it stable again
    hs = np.linspace(0.0, 1.0, 41)
    ws = [oracle.md1_wait(2.0, 0.45, h) for h in hs]
    assert all(a > b for a, b in zip(ws, ws[1:]))  # more hits, shorter wait
    assert ws[-1] == 0.0  # everything from the cache


@pytest.mark.parametrize("lam,E", [(0.5, 1.0), (0.8, 1.0), (0.3, 2.5)])
def test_md1_wait_agrees_with_a_simulated_queue(oracle, lam, E):
    # Poisson arrivals, one server, the same serving time for everyone, first come first served:
    # waiting in the queue follows w' = max(0, w + E - gap); time in the system = w + E.
    rng = np.random.Generator(np.random.Philox(key=1234))
    n = 400_000
    gaps = rng.exponential(1.0 / lam, n)
    w, total = 0.0, 0.0
    for g in gaps:
        w = max(0.0, w + E - g)
        total += w + E
    simulated = total / n
    assert oracle.md1_wait(E, lam, 0.0) == pytest.approx(simulated, rel=0.02)


def numpy_top1(cents_f32, queries_f32):
    c = cents_f32.astype(np.float64)
    q = queries_f32.astype(np.float64)
    c /= np.linalg.norm(c, axis=1, keepdims=True)
    q /= np.linalg.norm(q, axis=1, keepdims=True)
    return (q @ c.T).max(axis=1)


def test_t2h_counts_match_an_independent_route(oracle):
    wl = W.c2_mid(n_clusters=32, per_cluster=8, n_queries=600, dim=128, seed=77)
    cache = oracle.OracleCache(wl.dim, wl.K, "bf16")
    cache.load(wl.centroids)
    thetas = np.round(np.arange(0.98, 0.599, -0.02), 2).astype(np.float32)  # 0.98 down to 0.60, as the paper sweeps
    hits = cache.t2h(wl.queries, thetas)
    top1 = numpy_top1(W.storage_to_f32(wl.centroids, "bf16"), W.storage_to_f32(wl.queries, "bf16"))
    near = np.array([(np.abs(top1 - float(t)) < 1e-12).sum() for t in thetas])
    assert near.sum() == 0  # no similarity sits on a threshold, so the counts are unambiguous
    want = np.array([(top1 > float(t)).sum() for t in thetas])
    assert (hits == want).all()
    assert all(a <= b for a, b in zip(hits, hits[1:]))  # lower threshold, more hits
    assert 0 < hits[0] < 600  # planted neighbours hit, uniform directions never do


def test_t2h_extremes_and_strictness(oracle):
    dim = 8
    eye = W.to_storage(np.eye(dim, dtype=np.float32), "f32")
    cache = oracle.OracleCache(dim, dim, "f32")
    cache.load(eye)
    q = np.zeros((3, dim), np.float32)
    q[0, 0] = 2.0  # cosine exactly 1 with centroid 0
    q[1, 1], q[1, 2] = 1.0, 1.0  # cosine 1/sqrt(2)
    q[2, 3] = -1.0  # best cosine 0 (all others), -1 with centroid 3
    thetas = np.array([-2.0, 0.0, 0.5, 1.0, 1.5], np.float32)
    hits = cache.t2h(q, thetas)
    assert list(hits) == [3, 2, 2, 0, 0]  # strict: 1 > 1 and 0 > 0 are no hits
    assert list(cache.t2h(q[:0], thetas)) == [0, 0, 0, 0, 0]
    empty = oracle.OracleCache(dim, dim, "f32")
    assert list(empty.t2h(q, thetas)) == [0, 0, 0, 0, 0]  # nothing cached, nothing hits


def brute_pick(thetas, hit_ratio, L, lam, slo):
    best = -1
    for j, (t, h) in enumerate(zip(thetas, hit_ratio)):
        E = L * (1.0 - h)
        if lam * E >= 1.0:
            continue
        wait = E + lam * E * E / (2.0 * (1.0 - lam * E))
        if slo > wait and (best < 0 or t > thetas[best]):
            best = j
    return best


def test_pick_threshold_against_brute_force(oracle):
    rng = np.random.Generator(np.random.Philox(key=99))
    thetas = np.round(np.arange(0.98, 0.599, -0.02), 2).astype(np.float32)
    for _ in range(300):
        h = np.sort(rng.uniform(0.0, 1.0, thetas.shape[0]))  # hit ratio grows as the threshold falls
        L, lam = rng.uniform(0.5, 5.0), rng.uniform(0.0, 1.5)
        slo = rng.uniform(0.1, 6.0)
        order = rng.permutation(thetas.shape[0])  # the table need not be sorted
        got = oracle.pick_threshold(thetas[order], h[order], L, lam, slo)
        assert got == brute_pick(list(thetas[order]), list(h[order]), L, lam, slo)


def test_pick_threshold_special_cases(oracle):
    thetas = np.array([0.9, 0.8, 0.7], np.float32)
    h = np.array([0.25, 0.5, 0.75])  # (binary fractions: the waiting times below are exact)
    # no load: W = L (1 - h) = 0.75, 0.5, 0.25 for L = 1
    assert oracle.pick_threshold(thetas, h, 1.0, 0.0, 10.0) == 0  # everything meets the SLO: highest threshold
    assert oracle.pick_threshold(thetas, h, 1.0, 0.0, 0.625) == 1
    assert oracle.pick_threshold(thetas, h, 1.0, 0.0, 0.5) == 2  # S > W is strict: W = 0.5 does not pass
    assert oracle.pick_threshold(thetas, h, 1.0, 0.0, 0.25) == -1  # nothing passes
    assert oracle.pick_threshold(thetas, h, 1.0, 1.5, 100.0) == 1  # 0.9 is unstable: rho = 1.125


def test_adjust_threshold_ten_percent_rule(oracle):
    thetas = np.array([0.9, 0.6, 0.8, 0.7], np.float32)  # positions: 0.9 -> 0, 0.8 -> 2, 0.7 -> 3, 0.6 -> 1
    assert oracle.adjust_threshold(thetas, 2, 1.0, 1.05) == 2  # within 10 %
    assert oracle.adjust_threshold(thetas, 2, 1.0, 0.95) == 2
    assert oracle.adjust_threshold(thetas, 2, 1.0, 1.1) == 2  # exactly 10 % is not "exceeds"
    assert oracle.adjust_threshold(thetas, 2, 1.0, 1.2) == 3  # waiting longer than estimated: next lower threshold
    assert oracle.adjust_threshold(thetas, 2, 1.0, 0.8) == 0  # shorter: next higher one
    assert oracle.adjust_threshold(thetas, 1, 1.0, 5.0) == 1  # already the lowest
    assert oracle.adjust_threshold(thetas, 0, 1.0, 0.1) == 0  # already the highest
    assert oracle.adjust_threshold(thetas, -1, 1.0, 5.0) == -1  # no position to move from

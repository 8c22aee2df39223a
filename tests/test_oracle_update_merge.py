"""Pins for the oracle's centroid update, pair search and group merge.  CPU only.

Closed forms (exact means written out independently in numpy float64), special
cases with hand-computable answers, brute force through numpy, and planted
near-duplicate groups with a known pair count."""

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W


def bf(x):
    return W.f32_to_bf16_bits(np.asarray(x, np.float32))


def f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def unit64(x):
    x = np.asarray(x, np.float64)
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


# ------------------------------------------------------------------ update
def test_update_hand_computed_and_bf16_rounding(oracle):
    # c = (1,0) with one member, fold q = (0,3): members are unit vectors, so the mean is (0.5, 0.5)
    oc = oracle.OracleCache(2, 4, "bf16")
    oc.load(bf([[1.0, 0.0], [0.0, 1.0]]))
    oc.update(bf([[0.0, 3.0]]), np.array([0]))
    cents, means, sizes = oc.export()
    assert np.array_equal(means[0], [0.5, 0.5]) and sizes[0] == 2 and sizes[1] == 1
    # 1/sqrt(2) = 0x3F3504F3 as float32 -> bf16 0x3F35 (remainder 0x04F3 is below half)
    assert cents[0, 0] == 0x3F35 and cents[0, 1] == 0x3F35
    assert np.array_equal(cents[1], bf([0.0, 1.0])) and np.array_equal(means[1], [0.0, 1.0])
    # fold two copies of (0,1) into the fresh (1,0): mean (1/3, 2/3); normalised (1,2)/sqrt(5)
    oc.load(bf([[1.0, 0.0]]))
    oc.update(bf([[0.0, 1.0], [5.0, 5.0], [0.0, 2.0]]), np.array([0, -1, 0]))
    cents, means, sizes = oc.export()
    assert sizes[0] == 3
    assert np.allclose(means[0], [1 / 3, 2 / 3], rtol=0, atol=1e-16)
    # 1/sqrt(5) = 0.4472136 = 0x3EE4F92E -> 0x3EE5 (remainder 0xF92E rounds up); 2/sqrt(5) = 0x3F64F92E -> 0x3F65
    assert cents[0, 0] == 0x3EE5 and cents[0, 1] == 0x3F65


def test_update_fp32_storage_and_identity(oracle):
    oc = oracle.OracleCache(3, 2, "f32")
    c = f32([[1.0, 2.0, 2.0]])
    oc.load(c)
    # folding the centroid itself (any length) leaves the mean direction unchanged
    oc.update(f32([[2.0, 4.0, 4.0]]), np.array([0]))
    cents, means, sizes = oc.export()
    assert sizes[0] == 2
    assert np.allclose(means[0], [1 / 3, 2 / 3, 2 / 3], rtol=0, atol=1e-16)
    assert np.array_equal(cents[0], f32([1 / 3, 2 / 3, 2 / 3]))


def test_update_is_exact_mean_of_members_over_many_batches(oracle):
    """After any sequence of batches the mean equals the count-weighted mean of the loaded
    centroid and every unit-normalised query folded into it, computed here from the log."""
    wl = W.c4_stream(n_clusters=8, per_cluster=4, batches=12, batch=16, dim=40, sigma=0.3, seed=21)
    counts = W.random_counts(21, wl.K, 1, 9)
    oc = oracle.OracleCache(wl.dim, wl.K, "bf16")
    oc.load(wl.centroids, counts)
    c0 = unit64(wl.centroids_f32())
    total = c0 * counts[:, None].astype(np.float64)
    n = counts.astype(np.float64).copy()
    q_all = wl.queries_f32().astype(np.float64)
    r = np.random.default_rng(5)
    for b in range(12):
        q = wl.queries[b * 16:(b + 1) * 16]
        idx, sim, hit, _ = oc.lookup(q, 0.85)
        sel = np.where(r.random(16) < 0.8, idx, -1).astype(np.int32)
        oc.update(q, sel)
        for i in range(16):
            if sel[i] >= 0:
                total[sel[i]] += unit64(q_all[b * 16 + i])
                n[sel[i]] += 1
    cents, means, sizes = oc.export()
    assert np.array_equal(sizes, n.astype(np.int32))
    assert n.sum() > counts.sum() + 100
    want = total / n[:, None]
    assert np.allclose(means, want, rtol=0, atol=1e-14)
    # stored centroid = normalised mean rounded to bf16, for the rows that were touched
    touched = n > counts
    stored = W.bf16_bits_to_f32(cents).astype(np.float64)
    assert np.max(np.abs(stored[touched] - unit64(want[touched]))) <= 2.0 ** -9  # half a bf16 step below 1
    assert np.array_equal(cents[~touched], wl.centroids[~touched])
    expect_bits = bf(unit64(want[touched]).astype(np.float32))
    assert (expect_bits != cents[touched]).mean() < 1e-3  # float32 detour can differ only at exact halves


def test_update_order_free_duplicates_and_errors(oracle):
    wl = W.c1_tiny(n_clusters=4, per_cluster=4, n_queries=64, dim=24, seed=22)
    idx = np.random.default_rng(6).integers(-1, wl.K, size=64).astype(np.int32)
    idx[:10] = 3  # many queries into one centroid
    res = []
    for perm in (np.arange(64), np.random.default_rng(7).permutation(64)):
        oc = oracle.OracleCache(wl.dim, wl.K, "f32")
        oc.load(wl.centroids)
        oc.update(wl.queries[perm].copy(), idx[perm].copy())
        res.append(oc.export())
    assert np.array_equal(res[0][2], res[1][2])
    assert np.allclose(res[0][1], res[1][1], rtol=0, atol=1e-15)
    assert np.allclose(res[0][0], res[1][0], rtol=0, atol=1e-7)
    # r copies of q into a count-1 centroid c: normalize((c + r q)/(1 + r))
    oc = oracle.OracleCache(wl.dim, wl.K, "f32")
    oc.load(wl.centroids)
    q = np.repeat(wl.queries[:1], 5, axis=0)
    oc.update(q, np.full(5, 2, np.int32))
    cents, means, sizes = oc.export()
    c = unit64(wl.centroids[2]); qq = unit64(wl.queries[0])
    assert sizes[2] == 6
    assert np.allclose(means[2], (c + 5 * qq) / 6, rtol=0, atol=1e-15)
    assert np.allclose(cents[2], unit64((c + 5 * qq) / 6), rtol=0, atol=1e-7)
    # zero and non-finite queries are not members; idx beyond the live rows is an error
    z = wl.queries[:3].copy(); z[0] = 0.0; z[1, 0] = np.nan
    before = oc.export()
    oc.update(z, np.array([1, 1, -1], np.int32))
    after = oc.export()
    assert np.array_equal(before[2], after[2]) and np.array_equal(before[1], after[1])
    with pytest.raises(RuntimeError):
        oc.update(wl.queries[:1], np.array([wl.K], np.int32))
    # antipodal member: mean becomes zero, stored centroid is kept
    oc2 = oracle.OracleCache(2, 1, "f32")
    oc2.load(f32([[1.0, 0.0]]))
    oc2.update(f32([[-2.0, 0.0]]), np.array([0], np.int32))
    cents, means, sizes = oc2.export()
    assert np.array_equal(cents[0], [1.0, 0.0]) and np.array_equal(means[0], [0.0, 0.0]) and sizes[0] == 2


# ------------------------------------------------------------------- merge
def numpy_pairs(cents64, theta):
    u = unit64(cents64)
    S = u @ u.T
    i, j = np.nonzero(np.triu(S > np.float64(np.float32(theta)), k=1))
    return np.stack([i, j], axis=1).astype(np.int32), S


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_merge_pairs_match_brute_force_and_closed_form_count(oracle, dtype):
    wl = W.c5_merge(n_groups=48, copies=8, dim=96, dtype=dtype, seed=23)
    oc = oracle.OracleCache(wl.dim, wl.K, dtype)
    oc.load(wl.centroids)
    pairs, total = oc.merge(0.90)
    want, S = numpy_pairs(wl.centroids_f32().astype(np.float64), 0.90)
    assert total == 48 * 28 == len(want)  # exactly the C(8,2) pairs inside each group
    assert np.array_equal(pairs, want)    # lexicographic order
    assert np.all(wl.cluster_of[pairs[:, 0]] == wl.cluster_of[pairs[:, 1]])
    # a capped call still reports the full count and writes a prefix
    few, total2 = oc.merge(0.90, cap=10)
    assert total2 == total and np.array_equal(few, want[:10])
    # no pair is emitted twice or mirrored
    assert np.all(pairs[:, 0] < pairs[:, 1])
    # a lower threshold on a looser mixture: still equal to brute force
    wl2 = W.c5_merge(n_groups=20, copies=6, dim=32, sigma=0.6, dtype=dtype, seed=24)
    oc2 = oracle.OracleCache(wl2.dim, wl2.K, dtype)
    oc2.load(wl2.centroids)
    for th in (0.5, 0.7, 0.8):
        pairs, total = oc2.merge(th)
        want, S = numpy_pairs(wl2.centroids_f32().astype(np.float64), th)
        margin = np.abs(S - np.float64(np.float32(th))).min()
        assert margin > 1e-12
        assert np.array_equal(pairs, want)


def test_merge_threshold_is_strict(oracle):
    oc = oracle.OracleCache(4, 3, "f32")
    oc.load(f32([[1, 1, 1, 1], [1, 0, 0, 0], [2, 0, 0, 0]]))  # cos(0,1) = cos(0,2) = 0.5, cos(1,2) = 1
    pairs, total = oc.merge(0.5)
    assert total == 1 and np.array_equal(pairs, [[1, 2]])
    pairs, total = oc.merge(0.4999999)
    assert total == 3
    pairs, total = oc.merge(1.0)
    assert total == 0


def test_merge_apply_groups_means_and_compaction(oracle):
    wl = W.c5_merge(n_groups=10, copies=4, dim=32, sigma=0.05, dtype="bf16", seed=25)
    counts = W.random_counts(25, wl.K, 1, 100)
    oc = oracle.OracleCache(wl.dim, wl.K, "bf16")
    oc.load(wl.centroids, counts)
    pairs, total = oc.merge(0.90)
    assert total == 10 * 6
    # hand the pairs over in a scrambled order, some mirrored: the grouping must not care
    pr = pairs[np.random.default_rng(8).permutation(total)]
    pr[::3] = pr[::3, ::-1]
    _, means0, _ = oc.export()
    surv = oc.merge_apply(pr)
    cents, means, sizes = oc.export()
    assert oc.count == 10
    # survivor = lowest index of the group; survivors keep their relative order
    first = {}
    for i, g in enumerate(wl.cluster_of):
        first.setdefault(int(g), i)
    order = sorted(first.values())
    for new, old in enumerate(order):
        g = wl.cluster_of[old]
        mem = np.nonzero(wl.cluster_of == g)[0]
        assert np.all(surv[mem] == new)
        w = counts[mem].astype(np.float64)
        want = (means0[mem] * w[:, None]).sum(0) / w.sum()   # count-weighted mean of the members' means
        assert np.allclose(means[new], want, rtol=0, atol=1e-15)
        assert sizes[new] == counts[mem].sum()               # cluster sizes add up (Algorithm 1, MergeCentroids)
        stored = W.bf16_bits_to_f32(cents[new]).astype(np.float64)
        assert np.max(np.abs(stored - unit64(want))) <= 2.0 ** -9


def test_merge_apply_chains_singletons_and_errors(oracle):
    d = 8
    rows = np.eye(d, dtype=np.float32)[:6]
    oc = oracle.OracleCache(d, 6, "f32")
    oc.load(rows, np.array([1, 2, 3, 4, 5, 6], np.int32))
    # chain 1~3, 3~4 (1 and 4 not paired directly) -> one group {1,3,4}; 0,2,5 untouched
    surv = oc.merge_apply(np.array([[3, 1], [3, 4]], np.int32))
    cents, means, sizes = oc.export()
    assert oc.count == 4
    assert np.array_equal(surv, [0, 1, 2, 1, 1, 3])
    assert np.array_equal(sizes, [1, 11, 3, 6])
    want = (2 * rows[1] + 4 * rows[3] + 5 * rows[4]).astype(np.float64) / 11
    assert np.allclose(means[1], want, rtol=0, atol=1e-16)
    assert np.allclose(cents[1], unit64(want), rtol=0, atol=1e-7)
    assert np.array_equal(cents[[0, 2, 3]], rows[[0, 2, 5]])
    # with all counts 1 the group mean is the plain mean
    oc.load(rows)
    oc.merge_apply(np.array([[0, 5]], np.int32))
    _, means, sizes = oc.export()
    assert np.allclose(means[0], (rows[0] + rows[5]) / 2) and sizes[0] == 2 and oc.count == 5
    # no pairs: nothing changes
    before = oc.export()
    oc.merge_apply(np.zeros((0, 2), np.int32))
    after = oc.export()
    assert all(np.array_equal(a, b) for a, b in zip(before, after))
    for bad in ([[0, 0]], [[0, 9]], [[-1, 2]]):
        with pytest.raises(RuntimeError):
            oc.merge_apply(np.array(bad, np.int32))


# ------------------------------------------------- group merge: cluster_size and access_count
def read_merge_meta_example():
    """tests/golden/merge_meta_hand_worked.txt -> (cluster_size, access_count, pairs, expected rows, survivor map)"""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "merge_meta_hand_worked.txt")

    def f32_of(tok):
        return np.array([int(tok, 16)], np.uint32).view(np.float32)[0] if tok.startswith("0x") else np.float32(tok)

    loc, acc, pairs, expect, surv = {}, {}, [], {}, None
    for line in open(path):
        t = line.split("#")[0].split()
        if not t:
            continue
        if t[0] == "row":
            loc[int(t[1])], acc[int(t[1])] = f32_of(t[3]), int(t[4], 0)
        elif t[0] == "pair":
            pairs.append((int(t[1]), int(t[2])))
        elif t[0] == "expect":
            expect[int(t[1])] = (f32_of(t[2]), int(t[3], 0))
        elif t[0] == "survivor_map":
            surv = np.array([int(x) for x in t[1:]], np.int32)
    k = len(loc)
    return (np.array([loc[i] for i in range(k)], np.float32), np.array([acc[i] for i in range(k)], np.uint32),
            np.array(pairs, np.int32), expect, surv)


def merge_meta_state(k, dim=4, seed=3):
    """Rows for the example: every row its own direction, weight 1 (the vectors do not enter the two sums)."""
    x = np.random.default_rng(seed).standard_normal((k, dim)).astype(np.float32)
    cents = f32(x / np.linalg.norm(x, axis=1, keepdims=True))
    return cents, cents.astype(np.float64), np.ones(k, np.int32)


def test_group_merge_adds_cluster_sizes_and_access_counts_hand_worked(oracle):
    loc, acc, pairs, expect, surv = read_merge_meta_example()
    k = len(loc)
    cents, means, sizes = merge_meta_state(k)
    oc = oracle.OracleCache(4, k, "f32")
    oc.import_state(cents, means, sizes, loc, acc)
    got_l, got_a = oc.export_meta()
    assert np.array_equal(got_l, loc) and np.array_equal(got_a, acc)      # the snapshot is taken over as it is
    got_surv = oc.merge_apply(pairs)
    assert np.array_equal(got_surv, surv) and oc.count == len(expect)
    got_l, got_a = oc.export_meta()
    for i, (want_l, want_a) in expect.items():
        assert got_l[i].view(np.uint32) == np.float32(want_l).view(np.uint32), f"cluster_size of survivor {i}"
        assert int(got_a[i]) == want_a, f"access_count of survivor {i}"
    # the weights of the means add up as before (six, two, three, two rows of weight 1; one row alone)
    assert np.array_equal(oc.export()[2], [6, 2, 3, 2, 1])


def test_group_merge_meta_does_not_depend_on_the_order_of_the_pairs(oracle):
    loc, acc, pairs, expect, surv = read_merge_meta_example()
    k = len(loc)
    cents, means, sizes = merge_meta_state(k)
    r = np.random.default_rng(11)
    for trial in range(5):
        p = pairs[r.permutation(len(pairs))]
        flip = r.random(len(p)) < 0.5
        p = np.where(flip[:, None], p[:, ::-1], p)
        oc = oracle.OracleCache(4, k, "f32")
        oc.import_state(cents, means, sizes, loc, acc)
        assert np.array_equal(oc.merge_apply(p), surv)
        got_l, got_a = oc.export_meta()
        assert [(float(l), int(a)) for l, a in zip(got_l, got_a)] == [(float(expect[i][0]), expect[i][1]) for i in range(5)]

"""GPU parity at the full sizes of the five configurations, in the launch configuration the
benchmark uses.  Where the oracle cannot run the whole problem in seconds it runs on a seeded
sample of queries (or rows), and properties that hold at any size cover the rest."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import DEV, SIM_TOL, check_lookup, to_dev, to_host

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(400)]


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


def unit64(x):
    x = np.asarray(x, np.float64)
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def sample_invariant(wl, gi, gs, rows, n_cent, seed):
    """The returned similarity is the maximum: no sampled centroid beats it (float64, library matmul)."""
    r = np.random.default_rng(seed)
    ks = r.choice(wl.K, size=n_cent, replace=False)
    c = unit64(W.storage_to_f32(wl.centroids[ks], wl.dtype))
    q = unit64(W.storage_to_f32(wl.queries[rows], wl.dtype))
    S = q @ c.T
    assert np.all(S.max(axis=1) <= gs[rows] + SIM_TOL[wl.dtype])
    # and it is the cosine of the centroid it names
    cw = unit64(W.storage_to_f32(wl.centroids[gi[rows]], wl.dtype))
    assert np.max(np.abs(np.einsum("ij,ij->i", q, cw) - gs[rows])) <= 1e-5


def test_c2_mid_full(siso, oracle):
    print("case: c2_mid full size", flush=True)
    wl = W.c2_mid()
    assert (wl.K, wl.n, wl.dim) == (65536, 4096, 768)
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    q = to_dev(wl.queries, "bf16")
    outs = [tuple(t.clone() for t in cache.lookup(q, th)) for th in wl.thresholds]
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o[0], outs[0][0]) and torch.equal(o[1], outs[0][1])
    hits = [o[2].cpu().numpy() for o in outs]
    assert np.all(hits[1] <= hits[0]) and np.all(hits[2] <= hits[1])
    gi, gs = outs[0][0].cpu().numpy(), outs[0][1].cpu().numpy().astype(np.float64)
    near = wl.planted >= 0
    assert (gi[near] == wl.planted[near]).mean() > 0.995 and gs[near].min() > 0.99 and gs[~near].max() < 0.5
    assert abs(hits[1].mean() - 0.7) < 0.03 and np.array_equal(hits[1].astype(bool), near)
    rows = np.arange(0, wl.n, 16)  # 256 sampled queries through the oracle
    for th, o in zip(wl.thresholds, outs):
        ora = oracle.lookup_rows(wl.centroids, wl.queries[rows], th, "bf16")
        st = check_lookup(tuple(t[rows] for t in o), ora, th, "bf16", f"c2 theta {th}")
        assert st["max_err"] < 1e-4 and st["clear"] > 100
    sample_invariant(wl, gi, gs, np.arange(0, wl.n, 32), 4096, 1)
    # fold the hits of the middle threshold, on the device
    cache.update(q, outs[1][0], outs[1][2])
    sizes = cache.export()[2].cpu().numpy()
    assert sizes.sum() == wl.K + int(hits[1].sum()) and cache.bad_indices() == 0


def test_c3_large_full(siso, oracle):
    print("case: c3_large full size (2 GiB of centroids)", flush=True)
    wl = W.c3_large()
    assert (wl.K, wl.n, wl.dim) == (1048576, 16384, 1024)
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    q = to_dev(wl.queries, "bf16")
    idx, sim, hit = cache.lookup(q, 0.85)
    torch.cuda.synchronize()
    print("lookup done", flush=True)
    gi, gs, gh = idx.cpu().numpy(), sim.cpu().numpy().astype(np.float64), hit.cpu().numpy()
    assert (gi == wl.planted).mean() > 0.995 and gs.min() > 0.99 and gh.all()
    assert np.array_equal(gh, (sim.cpu().numpy() > np.float32(0.85)).astype(np.uint8))
    rows = np.arange(0, wl.n, 64)  # 256 sampled queries through the oracle, against all 1,048,576 centroids
    ora = oracle.lookup_rows(wl.centroids, wl.queries[rows], 0.85, "bf16")
    print("oracle sample done", flush=True)
    st = check_lookup((idx[rows], sim[rows], hit[rows]), ora, 0.85, "bf16", "c3")
    assert st["max_err"] < 1e-4 and st["clear"] >= 128
    sample_invariant(wl, gi, gs, np.arange(0, wl.n, 128), 8192, 2)
    # Zipf popularity: the most popular cluster takes a visible share of the batch
    top = np.bincount(wl.cluster_of[gi]).max()
    assert top > 0.02 * wl.n


def test_c4_stream_full(siso, oracle):
    """The whole stream: 4,096 micro-batches of 64 with the update of the hit centroids between lookups,
    nothing synchronised in between, eight re-draws of the popularity ranking.  The first three and the last
    three batches run in lock-step with the oracle (the last three from the GPU's own state after 4,093
    batches, taken over by the oracle); the running means of touched centroids after the whole stream are
    compared with their closed form, computed in float64 from the log of (index, hit)."""
    print("case: c4_stream, 262,144 centroids, 4,096 micro-batches of 64 with update in between", flush=True)
    wl = W.c4_stream()
    B, nb = 64, 4096
    assert (wl.K, wl.dim, wl.batch, wl.n) == (262144, 768, B, B * nb) and wl.meta["drift_every"] == 512
    th = 0.85
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.reserve(B)
    cache.load(to_dev(wl.centroids, "bf16"))
    oc = oracle.OracleCache(wl.dim, wl.K, "bf16")
    oc.load(wl.centroids)
    q_all = to_dev(wl.queries, "bf16")
    idx_log = torch.empty((nb, B), dtype=torch.int32, device=DEV)
    sim_log = torch.empty((nb, B), dtype=torch.float32, device=DEV)
    hit_log = torch.empty((nb, B), dtype=torch.uint8, device=DEV)

    def gpu_step(b):
        q = q_all[b * B:(b + 1) * B]
        if b % 2 == 0:   # the step as one call (its tail is one kernel) and as two: the same arithmetic, bit for bit
            cache.lookup_update(q, th, idx_log[b], sim_log[b], hit_log[b])
        else:
            cache.lookup(q, th, idx_log[b], sim_log[b], hit_log[b])
            cache.update(q, idx_log[b], hit_log[b])          # no host synchronisation between the two

    def lockstep(b, label):
        gpu_step(b)
        qs = wl.queries[b * B:(b + 1) * B]
        ora = oc.lookup(qs, th)
        check_lookup((idx_log[b], sim_log[b], hit_log[b]), ora, th, "bf16", f"c4 batch {b}")
        assert np.array_equal(idx_log[b].cpu().numpy(), ora[0]) and np.array_equal(hit_log[b].cpu().numpy(), ora[2])
        oc.update(qs, np.where(ora[2] == 1, ora[0], -1).astype(np.int32))
        print(f"batch {b} matches the oracle ({label})", flush=True)
        return np.unique(ora[0][ora[2] == 1])

    def compare_touched(touched, label, mean_tol):
        gc, gm, gsz = cache.export()
        oc_c, oc_m, oc_s = oc.export()
        assert np.array_equal(gsz.cpu().numpy(), oc_s), label
        err = np.abs(gm[touched].cpu().numpy().astype(np.float64) - oc_m[touched]).max()
        assert err < mean_tol, f"{label}: mean error {err:.3e}"
        g = to_host(gc, "bf16")
        assert (g[touched] != oc_c[touched]).mean() < 2e-3, label
        rest = np.ones(wl.K, bool)
        rest[touched] = False
        assert np.array_equal(g[rest], oc_c[rest]), label
        return err

    first = [lockstep(b, "from the start") for b in range(3)]
    compare_touched(np.unique(np.concatenate(first)), "first three batches", 2e-6)
    for b in range(3, nb - 3):
        gpu_step(b)
    torch.cuda.synchronize()
    print("4,093 batches done on the GPU", flush=True)

    # closed form of the running means after 4,093 batches, from the log
    gi = idx_log[:nb - 3].cpu().numpy().reshape(-1)
    gh = hit_log[:nb - 3].cpu().numpy().reshape(-1).astype(bool)
    assert (gi == wl.planted[:len(gi)]).mean() > 0.99 and gh.mean() > 0.95
    gc, gm, gsz = cache.export()
    sizes = gsz.cpu().numpy()
    folds = np.bincount(gi[gh], minlength=wl.K)
    assert np.array_equal(sizes, 1 + folds) and cache.bad_indices() == 0
    r = np.random.default_rng(44)
    hot = np.argsort(-folds)[:48]
    some = r.choice(np.nonzero(folds > 0)[0], size=208, replace=False)
    worst = 0.0
    for k in np.unique(np.concatenate([hot, some])):
        members = np.nonzero(gh & (gi == k))[0]
        u = unit64(W.bf16_bits_to_f32(wl.queries[members]))
        want = (unit64(W.bf16_bits_to_f32(wl.centroids[k])) + u.sum(axis=0)) / (1 + len(members))
        worst = max(worst, np.abs(gm[k].cpu().numpy().astype(np.float64) - want).max())
    print(f"hottest centroid folded {folds.max()} queries; worst mean error against the closed form {worst:.2e}", flush=True)
    assert folds.max() > 300 and worst < 2e-6
    # the popularity ranking was re-drawn: the hottest cluster of the first epoch is not that of the last
    top = lambda lo, hi: np.bincount(wl.cluster_of[gi[lo * B:hi * B]]).argmax()
    assert top(0, 512) != top(3584, nb - 3)
    norms = torch.linalg.vector_norm(gc.float(), dim=1)
    assert float((norms - 1).abs().max()) < 3e-3

    # the oracle takes over the GPU's state (fp32 means widened exactly) and the last three batches run in lock-step
    gl, ga = cache.export_meta()
    oc.import_state(to_host(gc, "bf16"), gm.cpu().numpy().astype(np.float64), sizes, gl.cpu().numpy(),
                    ga.cpu().numpy().astype(np.uint32))
    del gc, gm
    last = [lockstep(b, "after 4,093 batches") for b in range(nb - 3, nb)]
    compare_touched(np.unique(np.concatenate(last)), "last three batches", 2e-6)
    ol, oa = oc.export_meta()
    gl, ga = cache.export_meta()
    assert np.array_equal(ga.cpu().numpy().astype(np.uint32), oa) and np.array_equal(gl.cpu().numpy(), ol)
    assert int(oa.sum()) == int(hit_log.sum().item())   # every hit of the stream was counted as a reference


def test_c5_merge_full(siso, oracle):
    print("case: c5_merge full size", flush=True)
    wl = W.c5_merge()
    assert (wl.K, wl.dim) == (131072, 768)
    th = 0.90
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    expected = wl.meta["expected_pairs"]
    assert expected == 458752
    pairs, total = cache.merge(th, cap=expected + 4096)
    assert total == expected            # closed form: C(8,2) pairs in each of the 16,384 groups
    p = pairs.cpu().numpy()
    assert np.all(p[:, 0] < p[:, 1]) and len(np.unique(p.astype(np.int64) @ np.array([1 << 20, 1]))) == expected
    assert np.array_equal(wl.cluster_of[p[:, 0]], wl.cluster_of[p[:, 1]])
    assert np.all(np.bincount(wl.cluster_of[p[:, 0]], minlength=16384) == 28)
    # oracle on a subset of rows: 96 whole groups plus 1,280 other rows
    r = np.random.default_rng(3)
    groups = r.choice(16384, size=96, replace=False)
    rows = np.union1d(np.nonzero(np.isin(wl.cluster_of, groups))[0], r.choice(wl.K, size=1280, replace=False))
    oc = oracle.OracleCache(wl.dim, len(rows), "bf16")
    oc.load(wl.centroids[rows])
    want, _ = oc.merge(th)
    pos = -np.ones(wl.K, np.int64); pos[rows] = np.arange(len(rows))
    both = (pos[p[:, 0]] >= 0) & (pos[p[:, 1]] >= 0)
    got = np.stack([pos[p[both, 0]], pos[p[both, 1]]], 1)
    got = got[np.lexsort((got[:, 1], got[:, 0]))]
    assert np.array_equal(got, want) and len(want) >= 96 * 28
    print("pairs match", flush=True)
    # group merge
    surv = cache.merge_apply(pairs).cpu().numpy()
    assert cache.count == 16384
    first = np.full(16384, wl.K, np.int64)
    np.minimum.at(first, wl.cluster_of, np.arange(wl.K))
    order = np.argsort(first)                      # groups in the order of their lowest row
    newidx = np.empty(16384, np.int64); newidx[order] = np.arange(16384)
    assert np.array_equal(surv, newidx[wl.cluster_of])
    gc, gm, gsz = cache.export()
    assert bool((gsz == 8).all())
    check = r.choice(16384, size=256, replace=False)
    u = unit64(W.bf16_bits_to_f32(wl.centroids))
    gm_h = gm.cpu().numpy().astype(np.float64)
    gc_h = W.bf16_bits_to_f32(to_host(gc, "bf16")).astype(np.float64)
    for g in check:
        mem = np.nonzero(wl.cluster_of == g)[0]
        want_m = u[mem].mean(axis=0)
        assert np.abs(gm_h[newidx[g]] - want_m).max() < 2e-6
        assert np.abs(gc_h[newidx[g]] - unit64(want_m)).max() <= 2.0 ** -8


def test_refresh_mid_size_vs_oracle(siso, oracle):
    """Cache replacement at a size where the MFMA lookup and the MFMA pair search serve it: 16,384 cached
    centroids, a repository of 2,048 (half near cached ones, half new directions, a few duplicates of
    each other), more rows than the cache may keep."""
    import torch
    from gpu_util import SIM_TOL, to_dev, to_host
    dim, K, r = 768, 16384, 2048
    print(f"case: refresh K={K} r={r} dim={dim}", flush=True)
    wl = W.c2_mid(n_clusters=4096, per_cluster=4, n_queries=8, dim=dim, seed=333)
    rng = np.random.Generator(np.random.Philox(key=334))
    near = W.spread_sample(wl.centroids, "bf16", r // 2, sigma_lo=0.02, sigma_hi=0.1, seed=335)
    fresh = W.to_storage(W.uniform_directions(336, 7, r // 2 - 64, dim), "bf16")
    twins = W.spread_sample(fresh[:64], "bf16", 64, sigma_lo=0.02, sigma_hi=0.05, seed=337)  # near other new rows
    repo = np.concatenate([near, fresh, twins])[rng.permutation(r)]
    sizes = rng.integers(1, 40, size=r).astype(np.float32)
    counts = rng.integers(1, 40, size=K).astype(np.int32)
    M = K + 600
    ora = oracle.OracleCache(dim, K + r, "bf16")
    ora.load(wl.centroids, counts)
    gpu = siso.SisoCache(dim, K + r, siso.BF16)
    gpu.load(to_dev(wl.centroids, "bf16"), torch.from_numpy(counts).to("cuda:0"))
    want = ora.refresh(repo, sizes, 0.9, M, want_gap=True)
    got = gpu.refresh(to_dev(repo, "bf16"), torch.from_numpy(sizes).to("cuda:0"), 0.9, M)
    print(f"  oracle (merged, added, evicted, margin, lead of the closest) = {want}; gpu = {got}", flush=True)
    assert want[3] > 10 * SIM_TOL["bf16"]
    assert want[4] > 1e-6     # every closest centroid leads by more than single precision can blur
    assert got == want[:3] and want[1] > 900 and want[2] > 300
    oc, _, osz = ora.export()
    gc, _, gsz = gpu.export()
    assert gpu.count == ora.count == M
    assert (to_host(gc, "bf16") == oc).all() and (gsz.cpu().numpy() == osz).all()
    ol, oa = ora.export_meta()
    gl, ga = gpu.export_meta()
    assert (gl.cpu().numpy() == ol).all() and (ga.cpu().numpy().astype(np.uint32) == oa).all()


def test_cluster_mid_size_vs_oracle(siso, oracle):
    """Clustering at a size of many tile pairs: about 6,000 vectors in chains of overlapping topics."""
    from gpu_util import SIM_TOL
    from test_gpu_update_merge import compare_state
    dim = 512
    x, topic = W.query_log_chains(n_chains=150, chain_len=6, members_lo=2, members_hi=11, n_noise=300, dim=dim,
                                  dtype="bf16", seed=4242)
    n = len(x)
    print(f"case: cluster n={n} dim={dim}", flush=True)
    ora = oracle.OracleCache(dim, n, "bf16")
    want, seeds, margin = ora.cluster(x, 0.86, 2)
    print(f"  oracle: {len(seeds)} clusters, margin {margin:.4f}", flush=True)
    assert margin > 5 * SIM_TOL["bf16"] and n > 5500 and len(seeds) > 400
    gpu = siso.SisoCache(dim, n, siso.BF16)
    labels, clusters, pairs = gpu.cluster(to_dev(x, "bf16"), 0.86, 2)
    assert clusters == len(seeds) and np.array_equal(labels.cpu().numpy(), want)
    compare_state(gpu, ora, "bf16", "repository")


def test_cluster_full_size(siso, oracle):
    """The 131,072 rows of the merge workload taken as a query log: 16,384 topics of 8 near-duplicates."""
    print("case: cluster full size", flush=True)
    wl = W.c5_merge()
    gpu = siso.SisoCache(wl.dim, 16384, siso.BF16)
    labels, clusters, pairs = gpu.cluster(to_dev(wl.centroids, "bf16"), 0.86, 2)
    lab = labels.cpu().numpy()
    assert clusters == 16384 and pairs == wl.meta["expected_pairs"] and (lab >= 0).all()
    # all candidates have 8 vectors, so the clusters come in the order of their lowest rows
    first = np.full(16384, wl.K, np.int64)
    np.minimum.at(first, wl.cluster_of, np.arange(wl.K))
    newidx = np.empty(16384, np.int64); newidx[np.argsort(first)] = np.arange(16384)
    assert np.array_equal(lab, newidx[wl.cluster_of])
    gc, gm, gsz = gpu.export()
    sizes, acc = gpu.export_meta()
    assert bool((gsz == 8).all()) and bool((sizes == 8.0).all()) and bool((acc == 0).all())
    r = np.random.default_rng(5)
    u = unit64(W.bf16_bits_to_f32(wl.centroids))
    gm_h = gm.cpu().numpy().astype(np.float64)
    gc_h = W.bf16_bits_to_f32(to_host(gc, "bf16")).astype(np.float64)
    for g in r.choice(16384, size=256, replace=False):
        want_m = u[np.nonzero(wl.cluster_of == g)[0]].mean(axis=0)
        assert np.abs(gm_h[newidx[g]] - want_m).max() < 2e-6
        assert np.abs(gc_h[newidx[g]] - unit64(want_m)).max() <= 2.0 ** -8
    # the oracle on 64 whole topics plus 700 other rows clusters them the same way
    groups = r.choice(16384, size=64, replace=False)
    rows = np.union1d(np.nonzero(np.isin(wl.cluster_of, groups))[0], r.choice(wl.K, size=700, replace=False))
    oc = oracle.OracleCache(wl.dim, len(rows), "bf16")
    want, seeds, margin = oc.cluster(wl.centroids[rows], 0.86, 2)
    for g in groups:
        sel = wl.cluster_of[rows] == g
        assert len(set(want[sel].tolist())) == 1 and want[sel][0] >= 0 and (want[sel][0] != want[~sel]).all()


def test_cluster_a_million_vectors(siso):
    """The 1,048,576 rows of the large workload as a query log: 32,768 topics of 32 near-duplicates,
    16 million neighbour pairs.  Properties that hold by construction: the topics come back as
    generated, in the order of their first rows, every cluster with 32 members."""
    print("case: cluster 1,048,576 vectors", flush=True)
    wl = W.c3_large(n_queries=64)
    repo = siso.SisoCache(wl.dim, 32768, siso.BF16)
    labels, clusters, pairs = repo.cluster(to_dev(wl.centroids, "bf16"), 0.86, 2)
    assert clusters == 32768 and pairs == 32768 * (32 * 31 // 2)
    first = np.full(32768, wl.K, np.int64)
    np.minimum.at(first, wl.cluster_of, np.arange(wl.K))
    newidx = np.empty(32768, np.int64); newidx[np.argsort(first)] = np.arange(32768)
    assert np.array_equal(labels.cpu().numpy(), newidx[wl.cluster_of])
    assert bool((repo.export()[2] == 32).all())

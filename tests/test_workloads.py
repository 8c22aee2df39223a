"""The seeded input generators: storage conversions against torch's bf16 cast,
determinism, and the structure the recipes promise.  CPU only."""

import numpy as np
import torch

from paper_2508_18736_amd import workloads as W


def test_bf16_conversion_matches_library_cast():
    r = np.random.default_rng(0)
    x = np.concatenate([r.standard_normal(4096).astype(np.float32) * 10.0 ** r.integers(-30, 30, 4096),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.4e38, 1e-40],
                                 np.float32)]).astype(np.float32)
    got = W.f32_to_bf16_bits(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)
    # halfway cases go to the even neighbour
    assert W.f32_to_bf16_bits(np.array([1.00390625], np.float32))[0] == 0x3F80   # 1 + 2^-8  -> 1
    assert W.f32_to_bf16_bits(np.array([1.01171875], np.float32))[0] == 0x3F82   # 1 + 3*2^-8 -> 1 + 2^-6
    back = W.bf16_bits_to_f32(got)
    assert np.array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy(), equal_nan=True)
    assert W.f32_to_bf16_bits(np.array([np.nan], np.float32))[0] == 0x7FC0


def test_generators_are_deterministic_and_unit_norm(monkeypatch):
    a = W.c2_mid(n_clusters=16, per_cluster=8, n_queries=64, dim=64)
    monkeypatch.setattr(W, "_workers", lambda: 1)
    b = W.c2_mid(n_clusters=16, per_cluster=8, n_queries=64, dim=64)
    assert np.array_equal(a.centroids, b.centroids) and np.array_equal(a.queries, b.queries)
    assert np.array_equal(a.planted, b.planted)
    c = W.c2_mid(n_clusters=16, per_cluster=8, n_queries=64, dim=64, seed=999)
    assert not np.array_equal(a.centroids, c.centroids)
    for wl in (a, W.c1_tiny(n_clusters=4, per_cluster=4, n_queries=8, dim=32)):
        assert np.allclose(np.linalg.norm(wl.centroids_f32(), axis=1), 1.0, atol=2e-3)
        assert np.allclose(np.linalg.norm(wl.queries_f32(), axis=1), 1.0, atol=2e-3)


def test_mixture_structure():
    wl = W.c5_merge(n_groups=32, copies=8, dim=256)
    c = wl.centroids_f32().astype(np.float64)
    S = c @ c.T
    same = wl.cluster_of[:, None] == wl.cluster_of[None, :]
    off = ~np.eye(wl.K, dtype=bool)
    # copies of one mean: cosine about 1/(1+sigma^2); different means: about N(0, 1/dim)
    assert abs(S[same & off].mean() - 1 / (1 + 0.03 ** 2)) < 2e-3
    assert np.abs(S[~same]).max() < 0.5
    assert wl.meta["expected_pairs"] == 32 * 28
    # members of a cluster are spread over the array, not adjacent
    assert np.mean(np.diff(wl.cluster_of) == 0) < 0.2


def test_zipf_stream_and_drift():
    wl = W.c4_stream(n_clusters=64, per_cluster=4, batches=32, batch=16, dim=32, drift_every=8)
    assert wl.queries.shape == (32 * 16, 32) and wl.batch == 16
    p = W.zipf_probabilities(64, 1.2)
    assert abs(p.sum() - 1) < 1e-12 and abs(p[0] / p[1] - 2 ** 1.2) < 1e-12
    cl = wl.cluster_of[wl.planted]
    tops = [np.bincount(cl[e * 128:(e + 1) * 128], minlength=64).argmax() for e in range(4)]
    assert len(set(tops)) > 1  # the popular cluster changes between epochs
    # every query sits next to the centroid it was planted on
    q = wl.queries_f32(); c = wl.centroids_f32()
    cos = np.einsum("ij,ij->i", q, c[wl.planted])
    assert cos.min() > 0.98


def test_query_log_chains_structure():
    """The clustering log: members of a topic are close, neighbouring topics of a chain overlap at the
    clustering threshold, second neighbours and unrelated directions do not; same seed, same log."""
    x, topic = W.query_log_chains(n_chains=5, chain_len=4, dim=256, seed=9, n_noise=10)
    x2, topic2 = W.query_log_chains(n_chains=5, chain_len=4, dim=256, seed=9, n_noise=10)
    assert np.array_equal(x, x2) and np.array_equal(topic, topic2)
    u = W.storage_to_f32(x, "bf16").astype(np.float64)
    assert np.allclose(np.linalg.norm(u, axis=1), 1.0, atol=4e-3)
    s = u @ u.T
    related = topic >= 0
    assert (topic == -1).sum() == 10 and related.sum() > 40
    for i in np.flatnonzero(related):
        for j in np.flatnonzero(related):
            if i >= j:
                continue
            a, b = topic[i], topic[j]
            same_chain = a // 4 == b // 4
            if a == b:
                assert s[i, j] > 0.97
            elif same_chain and abs(a - b) == 1:
                assert 0.87 < s[i, j] < 0.93
            elif same_chain and abs(a - b) == 2:
                assert s[i, j] < 0.85
            elif not same_chain:
                assert abs(s[i, j]) < 0.4
    assert np.abs(s[~related][:, related]).max() < 0.4


def test_cone_moves_unrelated_directions_together():
    x = W.uniform_directions(3, 1, 200, 512)
    y = W.into_cone(x, 3, 1.28)
    s = (y @ y.T)[np.triu_indices(200, 1)]
    assert abs(np.median(s) - 1.28 ** 2 / (1 + 1.28 ** 2)) < 0.02 and np.allclose(np.linalg.norm(y, axis=1), 1, atol=1e-5)
    assert W.into_cone(x, 3, 0.0) is x

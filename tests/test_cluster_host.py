"""The library's host-side choice of the communities (section 4.1; the walk over the neighbour pairs that
siso_cluster does between its kernels) against the oracle.  The pairs come from numpy here, so no GPU work
is involved: these run wherever the library loads."""

import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2508_18736_amd", "libsiso.so")


@pytest.fixture(scope="module")
def siso():
    if not os.path.exists(LIB):
        from paper_2508_18736_amd import build
        build.build(verbose=False)
    from paper_2508_18736_amd import siso as binding
    return binding


def neighbour_pairs(x, dtype, theta, rng):
    u = W.storage_to_f32(x, dtype).astype(np.float64)
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    i, j = np.nonzero(np.triu(u @ u.T > theta, 1))
    pairs = np.stack([i, j], 1).astype(np.int32)
    flip = rng.random(len(pairs)) < 0.5                      # either order, any sequence
    pairs[flip] = pairs[flip][:, ::-1]
    return pairs[rng.permutation(len(pairs))]


@pytest.mark.parametrize("min_size,seed", [(1, 3), (2, 4), (3, 5), (5, 6)])
def test_communities_match_oracle(siso, oracle, min_size, seed):
    rng = np.random.default_rng(seed)
    x, _ = W.query_log_chains(n_chains=10, chain_len=5, n_noise=30, dim=64, dtype="bf16", seed=seed, sigma=0.08)
    ora = oracle.OracleCache(64, len(x), "bf16")
    want, seeds, _ = ora.cluster(x, 0.86, min_size)
    labels, clusters = siso.choose_communities(neighbour_pairs(x, "bf16", 0.86, rng), len(x), min_size)
    assert clusters == len(seeds) and np.array_equal(labels, want)


def test_hand_worked_example_and_edges(siso):
    # the example of tests/golden/cluster_hand_worked.txt as pairs: chain 0-1-2-3-4, pair 5-6, clique 9..12
    pairs = [(0, 1), (2, 1), (2, 3), (4, 3), (6, 5), (9, 10), (9, 11), (9, 12), (10, 11), (12, 10), (11, 12)]
    labels, clusters = siso.choose_communities(pairs, 13, 2)
    assert labels.tolist() == [1, 1, 1, 2, 2, 3, 3, -1, -1, 0, 0, 0, 0] and clusters == 4
    labels, clusters = siso.choose_communities(pairs, 13, 1)
    assert labels.tolist() == [1, 1, 1, 2, 3, 4, 4, 5, 6, 0, 0, 0, 0] and clusters == 7
    labels, clusters = siso.choose_communities(np.zeros((0, 2), np.int32), 4, 1)   # no pairs: everyone alone
    assert labels.tolist() == [0, 1, 2, 3] and clusters == 4
    labels, clusters = siso.choose_communities(np.zeros((0, 2), np.int32), 4, 2)
    assert labels.tolist() == [-1] * 4 and clusters == 0
    assert siso.choose_communities(np.zeros((0, 2), np.int32), 0, 1)[1] == 0
    for bad in ([(0, 0)], [(0, 4)], [(-1, 2)]):
        with pytest.raises(siso.SisoError):
            siso.choose_communities(bad, 4, 1)

"""GPU parity of the clustering (section 4.1: community detection at the clustering threshold, one
repository row per cluster) against the CPU oracle, through the C ABI.  The greedy choice makes
every cluster depend on the ones before it, so one neighbour decided differently could change
everything behind it: the query logs keep every cosine well away from the threshold (the oracle
reports the smallest margin, the test requires it far above the similarity tolerance), and then
labels, cluster sizes and the order of the clusters must agree exactly; means and stored centroids
to the bar of the centroid update."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import SIM_TOL, siso_dtype, to_dev
from test_gpu_update_merge import compare_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


def run_both(siso, oracle, x, dtype, dim, theta, min_size, capacity=None):
    """Clusters on both sides; the representatives (the member closest to each centroid) are compared here:
    equal wherever the oracle's best member leads the second best by more than single precision can blur."""
    n = len(x)
    capacity = capacity or max(n, 1)
    ora = oracle.OracleCache(dim, capacity, dtype)
    want_labels, seeds, margin, want_rep, rep_gap = ora.cluster(x, theta, min_size, representatives=True)
    gpu = siso.SisoCache(dim, capacity, siso_dtype(dtype))
    labels, clusters, pairs, rep = gpu.cluster(to_dev(x, dtype), theta, min_size, representatives=True)
    torch.cuda.synchronize()
    got_labels, rep = labels.cpu().numpy(), rep.cpu().numpy()
    if clusters == len(seeds) and np.array_equal(got_labels, want_labels):
        clear = rep_gap > 1e-5
        assert np.array_equal(rep[clear], want_rep[clear]), "representatives differ"
        assert all(got_labels[rep[k]] == k for k in range(clusters)), "a representative outside its cluster"
        print(f"  representatives: {int(clear.sum())} of {clusters} compared", flush=True)
    return ora, gpu, want_labels, seeds, margin, got_labels, clusters, pairs


@pytest.mark.parametrize("dtype,dim,chains,min_size,seed", [
    ("bf16", 256, 24, 1, 31),     # MFMA pair search; every vector ends somewhere
    ("bf16", 256, 40, 3, 32),     # small candidates dropped, vectors left over
    ("bf16", 768, 60, 2, 33),     # several 256-row tiles with a ragged tail
    ("f32", 160, 12, 2, 34),      # scalar pair search
])
def test_cluster_vs_oracle(siso, oracle, dtype, dim, chains, min_size, seed):
    print(f"case: cluster dtype={dtype} dim={dim} chains={chains} min_size={min_size}", flush=True)
    x, topic = W.query_log_chains(n_chains=chains, dim=dim, dtype=dtype, seed=seed, n_noise=37)
    ora, gpu, want, seeds, margin, got, clusters, pairs = run_both(siso, oracle, x, dtype, dim, 0.86, min_size)
    print(f"  n={len(x)} clusters={len(seeds)} pairs={pairs} margin={margin:.4f} unassigned={(want < 0).sum()}", flush=True)
    assert margin > 5 * SIM_TOL[dtype]
    assert clusters == len(seeds) and np.array_equal(got, want)
    assert sum(want[seeds[k]] != k for k in range(len(seeds))) > 0     # the order mattered somewhere
    compare_state(gpu, ora, dtype, "repository after clustering")
    ol, oa = ora.export_meta()
    gl, ga = gpu.export_meta()
    assert np.array_equal(gl.cpu().numpy(), ol) and np.array_equal(ga.cpu().numpy().astype(np.uint32), oa)
    # the repository answers lookups: every member finds its own cluster's centroid or a closer one
    idx, sim, hit = gpu.lookup(to_dev(x, dtype), 0.5)
    assert (idx.cpu().numpy()[want >= 0] >= 0).all()


def test_cluster_feeds_a_refresh(siso, oracle):
    print("case: cluster -> export -> refresh", flush=True)
    dtype, dim = "bf16", 128
    wl = W.c5_merge(n_groups=200, copies=5, dim=dim, dtype=dtype, seed=77)
    ora, gpu, want, seeds, margin, got, clusters, pairs = run_both(siso, oracle, wl.centroids, dtype, dim, 0.86, 1)
    assert margin > 5 * SIM_TOL[dtype] and clusters == 200 and np.array_equal(got, want)
    assert pairs == 200 * 10
    for g in range(200):
        assert len(set(got[wl.cluster_of == g].tolist())) == 1
    rows, _, _ = gpu.export()
    sizes, _ = gpu.export_meta()
    assert sizes.cpu().numpy().tolist() == [5.0] * 200
    serving = siso.SisoCache(dim, 256, siso.BF16)
    merged, added, evicted = serving.refresh(rows, sizes, 0.86, 128)
    assert (merged, added, evicted) == (0, 200, 72) and serving.count == 128


def test_cluster_edge_cases(siso, oracle):
    print("case: cluster edge cases", flush=True)
    dim = 64
    gpu = siso.SisoCache(dim, 8, siso.BF16)
    x = W.to_storage(W.uniform_directions(9, 1, 40, dim), "bf16")
    # more clusters than the cache holds: an error, and the cache keeps what it had
    gpu.load(to_dev(x[:3], "bf16"))
    with pytest.raises(RuntimeError):
        gpu.cluster(to_dev(x, "bf16"), 0.86, 1)
    assert gpu.count == 3
    # nothing reaches the smallest size: an empty repository, every label -1
    labels, clusters, pairs = gpu.cluster(to_dev(x, "bf16"), 0.86, 2)
    assert clusters == 0 and pairs == 0 and gpu.count == 0 and (labels.cpu().numpy() == -1).all()
    idx, sim, hit = gpu.lookup(to_dev(x[:4], "bf16"), 0.5)
    assert (idx.cpu().numpy() == -1).all()
    # everything is a neighbour of everything: one cluster; its mean is the mean of the directions
    labels, clusters, pairs = gpu.cluster(to_dev(x, "bf16"), -1.5, 3)
    assert clusters == 1 and pairs == 40 * 39 // 2 and (labels.cpu().numpy() == 0).all()
    ora = oracle.OracleCache(dim, 8, "bf16")
    ora.cluster(x, -1.5, 3)
    compare_state(gpu, ora, "bf16", "one cluster")
    # no vectors at all
    labels, clusters, pairs = gpu.cluster(torch.empty((0, dim), dtype=torch.bfloat16, device="cuda:0"), 0.86, 1)
    assert clusters == 0 and gpu.count == 0
    # a vector without a direction or with a NaN is refused and nothing changes
    gpu.load(to_dev(x[:5], "bf16"))
    bad = x.copy()
    bad[7] = 0
    with pytest.raises(RuntimeError):
        gpu.cluster(to_dev(bad, "bf16"), 0.86, 1)
    bad[7] = 0x7FC0
    with pytest.raises(RuntimeError):
        gpu.cluster(to_dev(bad, "bf16"), 0.86, 1)
    assert gpu.count == 5


@pytest.mark.parametrize("dtype,dim", [("f32", 98), ("bf16", 100), ("f32", 7), ("bf16", 4096)])
def test_cluster_odd_dimensions(siso, oracle, dtype, dim):
    """Dimensions that the MFMA pair search does not take (scalar kernels), the smallest and the largest."""
    print(f"case: cluster dtype={dtype} dim={dim}", flush=True)
    if dim >= 64:
        x, _ = W.query_log_chains(n_chains=6, dim=dim, dtype=dtype, seed=dim)
    else:
        x = W.to_storage(W.uniform_directions(dim, 1, 120, dim), dtype)
    ora, gpu, want, seeds, margin, got, clusters, pairs = run_both(siso, oracle, x, dtype, dim, 0.86, 1)
    assert margin > 1e-3 and clusters == len(seeds) and np.array_equal(got, want)
    compare_state(gpu, ora, dtype, "odd dimension")

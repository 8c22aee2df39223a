"""GPU parity of the threshold-to-hit-ratio table (section 4.3) against the CPU oracle, through
the C ABI.  A count can only differ from the oracle's by sample queries whose similarity lies
within the lookup tolerance of that threshold; on these workloads there are none for most
thresholds, and the test says how many there were."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import SIM_TOL, siso_dtype, to_dev

pytestmark = pytest.mark.gpu

SWEEP = np.round(np.arange(0.98, 0.599, -0.02), 2).astype(np.float32)  # 0.98 down to 0.60


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


@pytest.mark.parametrize("dtype,dim,n_clusters,per_cluster,n", [("bf16", 256, 64, 16, 1500), ("f32", 384, 16, 8, 333),
                                                                ("bf16", 768, 128, 8, 40)])
def test_t2h_counts_vs_oracle(siso, oracle, dtype, dim, n_clusters, per_cluster, n):
    print(f"case: t2h dtype={dtype} dim={dim} K={n_clusters * per_cluster} n={n}", flush=True)
    wl = W.c2_mid(n_clusters=n_clusters, per_cluster=per_cluster, n_queries=n, dim=dim, dtype=dtype, sigma=0.35,
                  seed=501 + dim)
    ora = oracle.OracleCache(wl.dim, wl.K, dtype)
    ora.load(wl.centroids)
    want = ora.t2h(wl.queries, SWEEP)
    _, sim, _, _ = ora.lookup(wl.queries, 0.0)
    near = np.array([(np.abs(sim - float(t)) <= SIM_TOL[dtype]).sum() for t in SWEEP])
    cache = siso.SisoCache(wl.dim, wl.K, siso_dtype(dtype))
    cache.load(to_dev(wl.centroids, dtype))
    got = cache.t2h(to_dev(wl.queries, dtype), SWEEP)
    print(f"  oracle hits {want.tolist()}\n  gpu hits    {got.tolist()}\n  near a threshold {near.tolist()}", flush=True)
    assert (np.abs(got - want) <= near).all()
    assert (got[near == 0] == want[near == 0]).all() and (near == 0).sum() >= len(SWEEP) // 2
    assert all(a <= b for a, b in zip(got, got[1:]))  # lower threshold, more hits
    assert 0 < want[-1] and want[0] < n  # the sweep crosses the similarities of this workload


def test_t2h_gradual_curve_vs_oracle(siso, oracle):
    """Sample with similarities spread over the whole sweep: every threshold cuts through it."""
    wl = W.c2_mid(n_clusters=256, per_cluster=8, n_queries=8, dim=256, seed=91)
    sample = W.spread_sample(wl.centroids, "bf16", 3000, seed=92)
    ora = oracle.OracleCache(wl.dim, wl.K, "bf16")
    ora.load(wl.centroids)
    want = ora.t2h(sample, SWEEP)
    _, sim, _, _ = ora.lookup(sample, 0.0)
    near = np.array([(np.abs(sim - float(t)) <= SIM_TOL["bf16"]).sum() for t in SWEEP])
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    got = cache.t2h(to_dev(sample, "bf16"), SWEEP)
    print(f"  oracle hits {want.tolist()}\n  gpu hits    {got.tolist()}\n  near a threshold {near.tolist()}", flush=True)
    assert (np.abs(got - want) <= near).all()
    assert (np.diff(want) > 0).all()  # strictly more hits at every lower threshold
    assert np.abs(got - want).sum() <= 3  # fp32 accumulation of exact products: far inside the bar


def test_t2h_is_the_lookup_hit_count(siso):
    """The table's entry for a threshold is exactly the number of hit flags siso_lookup sets at it."""
    wl = W.c2_mid(n_clusters=64, per_cluster=16, n_queries=700, dim=256, sigma=0.35, seed=77)
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    q = to_dev(wl.queries, "bf16")
    hits = cache.t2h(q, SWEEP)
    for j in (0, 7, 19):
        _, _, hit = cache.lookup(q, float(SWEEP[j]))
        assert int(hit.sum().item()) == hits[j]


def test_t2h_edges(siso):
    dim = 64
    cache = siso.SisoCache(dim, 16, siso.F32)
    q = torch.zeros((5, dim), device="cuda:0")
    q[0, 0], q[1, 1], q[2, 2] = 1.0, 3.0, -2.0
    thetas = np.array([-2.0, 0.5, 1.5], np.float32)
    assert cache.t2h(q, thetas).tolist() == [0, 0, 0]  # empty cache: nothing hits
    cache.load(torch.eye(16, dim, device="cuda:0"))
    # rows 0, 1 match a centroid exactly (1 > 0.5), row 2 is opposite to one (best 0), rows 3, 4 are zero (0)
    assert cache.t2h(q, thetas).tolist() == [5, 2, 0]
    assert cache.t2h(q[:0], thetas).tolist() == [0, 0, 0]
    assert cache.t2h(q, thetas[:0]).tolist() == []
    with pytest.raises(siso.SisoError):
        cache.t2h(q, np.zeros(2000, np.float32))  # more thresholds than the table holds


def test_probe_reports_plausible_rates(siso):
    """The chip's own ceilings, as the benchmark reports them beside the published peaks."""
    random_ops, constant_ops, stream = siso.probe(0), siso.probe(1), siso.probe(2)
    print(f"  MFMA loop: {random_ops:.0f} TFLOP/s on random operands, {constant_ops:.0f} on constant ones; "
          f"streaming read {stream:.0f} GB/s", flush=True)
    assert 500 < random_ops <= 2600 and random_ops <= constant_ops * 1.05 <= 2600 * 1.05
    assert 2000 < stream <= 8200
    with pytest.raises(siso.SisoError):
        siso.probe(3)

"""The lookup that allocates nothing (siso_lookup_static) against siso_lookup, through the C ABI: two calls in
a row, the second with a smaller input; the paths for large, mid-size and small batches and the fp32 kernel;
a batch beyond the static workspace is rejected."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import DEV, check_lookup, siso_dtype, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


def outputs(n):
    return (torch.full((n,), -7, dtype=torch.int32, device=DEV), torch.full((n,), -7.0, dtype=torch.float32, device=DEV),
            torch.full((n,), 7, dtype=torch.uint8, device=DEV))


@pytest.mark.parametrize("dtype,dim,K,n1,n2", [("bf16", 768, 9000, 1500, 300), ("bf16", 256, 70000, 64, 9),
                                                ("bf16", 512, 3000, 128, 100), ("f32", 384, 1024, 256, 31)])
def test_static_lookup_equals_lookup(siso, oracle, dtype, dim, K, n1, n2):
    print(f"case: static lookup {dtype} dim={dim} K={K} n={n1} then {n2}", flush=True)
    wl = W.c2_mid(n_clusters=128, per_cluster=(K + 127) // 128, n_queries=n1, dim=dim, dtype=dtype, seed=97)
    wl.centroids = wl.centroids[:K].copy()
    cache = siso.SisoCache(dim, K, siso_dtype(dtype))
    cache.load(to_dev(wl.centroids, dtype))
    q1 = to_dev(wl.queries, dtype)
    q2 = q1[n1 - n2:].clone()          # a smaller batch of other rows: the workspace still holds the first call's keys
    th = 0.85
    got1, got2 = outputs(n1), outputs(n2)
    cache.lookup_static(q1, th, *got1)
    cache.lookup_static(q2, th, *got2)  # two calls in a row, no synchronisation in between
    torch.cuda.synchronize()
    ref1 = cache.lookup(q1, th)
    ref2 = cache.lookup(q2, th)
    torch.cuda.synchronize()
    for g, r in zip(got1 + got2, ref1 + ref2):
        assert torch.equal(g, r)        # the same kernels: bit-identical
    ora = oracle.lookup_rows(wl.centroids, wl.queries, th, dtype)
    check_lookup(got1, ora, th, dtype, "static lookup")
    check_lookup(got2, tuple(a[n1 - n2:] for a in ora), th, dtype, "static lookup, second call")
    # hits are references to their centroids in this call as well: four lookups counted
    _, acc = cache.export_meta()
    hits1, hits2 = int(ref1[2].sum().item()), int(ref2[2].sum().item())
    assert int(acc.sum().item()) == 2 * (hits1 + hits2)


def test_static_lookup_edges(siso):
    print("case: static lookup edges", flush=True)
    dim, K = 1024, 300000
    cache = siso.SisoCache(dim, K, siso.BF16)
    rows = W.to_storage(W.uniform_directions(98, 2, 4096, dim), "bf16")
    cache.load(to_dev(np.tile(rows, (K // 4096 + 1, 1))[:K], "bf16"))
    # 8,192 queries against 300,000 centroids of 1,024 elements need more keys than the static workspace holds: an error, no fault
    big = torch.zeros((8192, dim), dtype=torch.bfloat16, device=DEV)
    with pytest.raises(siso.SisoError, match="static workspace"):
        cache.lookup_static(big, 0.5, *outputs(8192))
    # n = 0 is a no-op; an empty cache answers as siso_lookup does
    cache.lookup_static(big[:0], 0.5, *outputs(0))
    empty = siso.SisoCache(dim, 8, siso.BF16)
    o = outputs(5)
    empty.lookup_static(big[:5], 0.5, *o)
    torch.cuda.synchronize()
    assert (o[0] == -1).all() and torch.isneginf(o[1]).all() and (o[2] == 0).all()

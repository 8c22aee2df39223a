"""GPU parity of the lookup kernels against the CPU oracle, through the C ABI."""

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


def run_lookup(siso, wl, threshold, path, opts=None, capacity=None):
    cache = siso.SisoCache(wl.dim, capacity or max(wl.K, 1), siso_dtype(wl.dtype))
    cache.set_lookup_path(path)
    for k, v in (opts or {}).items():
        cache.set_option(k, v)
    cache.load(to_dev(wl.centroids, wl.dtype))
    out = cache.lookup(to_dev(wl.queries, wl.dtype), threshold)
    torch.cuda.synchronize()
    return cache, out


def test_c1_tiny_fp32_scalar(siso, oracle):
    print("case: c1_tiny fp32 scalar path", flush=True)
    wl = W.c1_tiny()
    assert (wl.K, wl.n, wl.dim) == (1024, 256, 384)
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.80, "f32")
    cache, out = run_lookup(siso, wl, 0.80, siso.PATH_SCALAR)
    # the members of a cluster sit within about 1e-3 of each other, so the stated bar (gap > 1e-3)
    # decides few indices here; fp32 arithmetic is good for a far tighter one
    check_lookup(out, ora, 0.80, "f32", "c1")
    st = check_lookup(out, ora, 0.80, "f32", "c1 tight", gap_bar=1e-5)
    assert st["clear"] > 200 and ora[2].sum() > 200 and st["max_err"] < 2e-6
    # auto path on fp32 must give the same answer
    cache2, out2 = run_lookup(siso, wl, 0.80, siso.PATH_AUTO)
    assert all(torch.equal(a, b) for a, b in zip(out, out2))


@pytest.mark.parametrize("dtype,dim,K,n", [("bf16", 72, 1013, 77), ("f32", 100, 300, 130), ("bf16", 768, 2100, 65)])
def test_scalar_path_ragged_shapes(siso, oracle, dtype, dim, K, n):
    print(f"case: scalar {dtype} dim={dim} K={K} n={n}", flush=True)
    wl = W.c2_mid(n_clusters=64, per_cluster=(K + 63) // 64, n_queries=n, dim=dim, dtype=dtype, seed=31)
    wl.centroids = wl.centroids[:K].copy()
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, dtype)
    cache, out = run_lookup(siso, wl, 0.85, siso.PATH_SCALAR)
    check_lookup(out, ora, 0.85, dtype, "scalar ragged")


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("dim,K,n,tps", [(128, 5000, 300, 0), (768, 2049, 513, 3), (192, 700, 1, 1), (1024, 1500, 257, 2),
                                          (4096, 600, 130, 0), (320, 37, 700, 0), (64 * 7, 3000, 2000, 5)])
def test_mfma_path_vs_oracle(siso, oracle, cfg, dim, K, n, tps):
    print(f"case: mfma cfg={cfg} dim={dim} K={K} n={n} tiles_per_slice={tps}", flush=True)
    wl = W.c2_mid(n_clusters=128, per_cluster=(K + 127) // 128, n_queries=n, dim=dim, seed=32 + cfg)
    wl.centroids = wl.centroids[:K].copy()
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    cache, out = run_lookup(siso, wl, 0.85, siso.PATH_MFMA, {"mfma_config": cfg, "tiles_per_slice": tps},
                            capacity=K + 7)
    st = check_lookup(out, ora, 0.85, "bf16", f"mfma cfg {cfg}")
    assert st["max_err"] < 1e-4  # fp32 accumulation of exact bf16 products is far inside the bar
    # scalar path on the same data agrees on everything the bar fixes
    cache.set_lookup_path(siso.PATH_SCALAR)
    out_s = cache.lookup(to_dev(wl.queries, "bf16"), 0.85)
    check_lookup(out_s, ora, 0.85, "bf16", "scalar on mfma data")
    # determinism: a second call is bit-identical
    cache.set_lookup_path(siso.PATH_MFMA)
    out2 = cache.lookup(to_dev(wl.queries, "bf16"), 0.85)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(out, out2))


@pytest.mark.parametrize("n,K,dim", [(700, 5000, 256), (1300, 9000, 128), (1700, 40000, 128), (2305, 3000, 256), (2400, 70000, 128),
                                     (5000, 2049, 128)])
def test_numbers_of_query_tiles_that_do_not_fill_the_blocks(siso, oracle, n, K, dim):
    """3, 6, 7, 10 and 20 tiles of queries: the blocks of query tiles that share an XCD's centroid tiles are of even
    size then (a number that need not divide the 32 places of a unit), and the slice length is chosen for an even
    load on the XCDs.  Every query against the oracle, also through the k closest (whose second pass lists each
    row once)."""
    print(f"case: ragged query tiles n={n} K={K} dim={dim}", flush=True)
    wl = W.c2_mid(n_clusters=64, per_cluster=(K + 63) // 64, n_queries=n, dim=dim, seed=47)
    wl.centroids = wl.centroids[:K].copy()
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    for cfg in (0, 1):
        cache, out = run_lookup(siso, wl, 0.85, siso.PATH_MFMA, {"mfma_config": cfg}, capacity=K)
        st = check_lookup(out, ora, 0.85, "bf16", f"ragged cfg {cfg}")
        assert st["max_err"] < 1e-4
    oc = oracle.OracleCache(dim, K, "bf16")
    oc.load(wl.centroids)
    from gpu_util import check_topk
    tk = cache.lookup_topk(to_dev(wl.queries, "bf16"), 6)
    torch.cuda.synchronize()
    check_topk(tk, oc.lookup_topk(wl.queries, 7), "bf16", "ragged top 6")


@pytest.mark.parametrize("storage,cfg,n", [("bf16", 3, 50), ("bf16", 2, 128), ("bf16", 1, 300), ("bf16", 5, 700), ("fp8", 8, 64), ("fp8", 7, 100),
                                            ("fp8", 6, 300), ("fp8", 3, 33)])
def test_streaming_mark_changes_nothing(siso, oracle, storage, cfg, n):
    """The centroid loads of the eight-wave kernels with and without the non-temporal mark (two instantiations,
    chosen per launch by size): the same outputs bit for bit, the lookup and the k closest."""
    print(f"case: streaming mark {storage} cfg={cfg} n={n}", flush=True)
    wl = W.c2_mid(n_clusters=64, per_cluster=50, n_queries=n, dim=256, seed=61)
    outs = []
    for hint in (0, 1, 2):
        cache = siso.SisoCache(wl.dim, wl.K, siso.FP8 if storage == "fp8" else siso.BF16)
        cache.set_option("mfma_config", cfg)
        cache.set_option("stream_hint", hint)
        cache.load(to_dev(wl.centroids, "bf16"))
        q = to_dev(wl.queries, "bf16")
        outs.append(tuple(cache.lookup(q, 0.85)) + tuple(cache.lookup_topk(q, 5)))
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert all(torch.equal(a, b) for a, b in zip(o, outs[0]))
    if storage == "bf16":
        check_lookup(outs[1][:3], oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16"), 0.85, "bf16", "marked")
    with pytest.raises(siso.SisoError):
        cache.set_option("stream_hint", 3)


@pytest.mark.parametrize("cfg,n", [(2, 100), (3, 40), (1, 300), (4, 300), (5, 300)])
@pytest.mark.parametrize("tps", [3, 7])
def test_two_slab_tiles_with_scaled_rows(siso, oracle, cfg, n, tps):
    """The smallest dimension of the MFMA path (two slabs per tile) with workgroups that walk through
    several tiles, a ragged last tile and stored rows of very different lengths: a tile scaled by another
    tile's inverse lengths would lose its winners."""
    dim, K = 128, 256 * 9 + 77
    print(f"case: two-slab tiles cfg={cfg} n={n} tiles_per_slice={tps}", flush=True)
    wl = W.c2_mid(n_clusters=128, per_cluster=(K + 127) // 128, n_queries=n, dim=dim, seed=77 + cfg)
    r = np.random.default_rng(5 + tps)
    c = wl.centroids_f32()[:K] * np.exp2(r.integers(-6, 7, size=K)).astype(np.float32)[:, None]
    wl.centroids = W.f32_to_bf16_bits(c)
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    cache, out = run_lookup(siso, wl, 0.85, siso.PATH_MFMA, {"mfma_config": cfg, "tiles_per_slice": tps}, capacity=K + 5)
    st = check_lookup(out, ora, 0.85, "bf16", f"two-slab cfg {cfg}")
    assert st["max_err"] < 1e-4 and st["clear"] > n // 2
    if n <= 64:  # the small-batch path proper (one workgroup per compute unit) on the same rows
        cache.set_option("mfma_config", 0)
        cache.set_lookup_path(siso.PATH_SKINNY)
        out2 = cache.lookup(to_dev(wl.queries, "bf16"), 0.85)
        check_lookup(out2, ora, 0.85, "bf16", "two-slab skinny")


@pytest.mark.parametrize("dim,K,n", [(256, 5013, 64), (768, 4099, 7), (1024, 2048, 33), (768, 31, 1), (512, 70000, 32)])
def test_skinny_path_vs_oracle(siso, oracle, dim, K, n):
    print(f"case: skinny dim={dim} K={K} n={n}", flush=True)
    wl = W.c4_stream(n_clusters=128, per_cluster=(K + 127) // 128, batches=1, batch=n, dim=dim, seed=60)
    wl.centroids = wl.centroids[:K].copy()
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    cache, out = run_lookup(siso, wl, 0.85, siso.PATH_SKINNY, capacity=K + 3)
    st = check_lookup(out, ora, 0.85, "bf16", "skinny")
    assert st["max_err"] < 1e-4
    # the automatic choice for a small batch is this path and gives the same bits
    cache.set_lookup_path(siso.PATH_AUTO)
    out2 = cache.lookup(to_dev(wl.queries, "bf16"), 0.85)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(out, out2))
    # a batch that is too large for this path is an error, not a fault
    cache.set_lookup_path(siso.PATH_SKINNY)
    with pytest.raises(siso.SisoError):
        cache.lookup(torch.zeros((65, dim), dtype=torch.bfloat16, device=DEV), 0.5)


@pytest.mark.parametrize("path,cfg", [(1, 0), (2, 1), (2, 2), (2, 3), (2, 4), (2, 5), (3, 0)])
def test_exact_duplicates_lowest_index_wins(siso, oracle, path, cfg):
    """Bit-identical copies of a centroid at distant rows (other tiles, other slices) tie
    exactly; the lowest index must be returned."""
    print(f"case: duplicates path={path} cfg={cfg}", flush=True)
    nq = 64 if path == 3 else 200
    wl = W.c2_mid(n_clusters=64, per_cluster=40, n_queries=nq, dim=256, seed=40)
    K = wl.K
    r = np.random.default_rng(9)
    src = r.choice(K, size=60, replace=False)
    for a in src:
        for b in r.choice(K, size=2, replace=False):
            wl.centroids[b] = wl.centroids[a]
    # queries near the duplicated rows
    cf = wl.centroids_f32()
    wl.queries = W.jitter(41, 3, cf, np.resize(src, nq), 0.08, "total", "bf16")
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    cache, out = run_lookup(siso, wl, 0.85, path, {"mfma_config": cfg, "tiles_per_slice": 1})
    gi = out[0].cpu().numpy()
    tie = ora[1] == ora[3]
    assert tie.sum() > 0.75 * nq
    assert np.array_equal(gi[tie], ora[0][tie])  # exact ties: the lowest index, bit-exactly
    check_lookup(out, (ora[0], ora[1], ora[2], np.where(tie, -np.inf, ora[3])), 0.85, "bf16", "duplicates")


@pytest.mark.parametrize("path", [1, 2, 3])
def test_special_values_and_edges(siso, oracle, path):
    print(f"case: special values path={path}", flush=True)
    dim = 256
    wl = W.c2_mid(n_clusters=8, per_cluster=40, n_queries=64 if path == 3 else 70, dim=dim, seed=42)
    q = wl.queries_f32().copy()
    q[0] = 0.0                      # zero-length query
    q[1, 5] = np.nan                # NaN query
    q[2, 7] = np.inf                # infinite query
    q[3] *= 1e-3                    # not normalised
    q[4] *= 250.0
    wl.queries = W.f32_to_bf16_bits(q)
    c = wl.centroids_f32().copy()
    c[10] = 0.0                     # zero centroid: similarity 0
    c[11, 3] = np.nan               # NaN centroid never wins
    c[12] *= 7.0                    # centroid that is not unit length
    wl.centroids = W.f32_to_bf16_bits(c)
    ora = oracle.lookup_rows(wl.centroids, wl.queries, 0.85, "bf16")
    cache, out = run_lookup(siso, wl, 0.85, path)
    check_lookup(out, ora, 0.85, "bf16", "special")
    gi = out[0].cpu().numpy(); gs = out[1].cpu().numpy()
    assert gi[0] == 0 and gs[0] == 0.0 and gi[1] == -1 and np.isnan(gs[1]) and gi[2] == -1 and np.isnan(gs[2])
    # thresholds: -2 hits everything finite, 1.5 nothing
    assert cache.lookup(to_dev(wl.queries, "bf16"), -2.0)[2].cpu().numpy()[3:].all()
    assert not cache.lookup(to_dev(wl.queries, "bf16"), 1.5)[2].cpu().numpy().any()
    # n = 0 is a no-op; an empty cache answers -1 / -inf / miss
    cache.lookup(to_dev(wl.queries[:0], "bf16"), 0.5)
    empty = siso.SisoCache(dim, 16, siso.BF16)
    ei, es, eh = empty.lookup(to_dev(wl.queries[3:9], "bf16"), 0.5)
    assert (ei.cpu().numpy() == -1).all() and np.isneginf(es.cpu().numpy()).all() and not eh.cpu().numpy().any()
    # wrong shapes and capacity overflow are errors, not faults
    with pytest.raises(ValueError):
        cache.lookup(torch.zeros((4, dim + 1), dtype=torch.bfloat16, device=DEV), 0.5)
    with pytest.raises(siso.SisoError):
        small = siso.SisoCache(dim, 4, siso.BF16)
        small.load(to_dev(wl.centroids[:5], "bf16"))


def test_threshold_sweep_is_one_similarity(siso):
    """The similarity does not depend on the threshold: idx/sim are bit-identical over a sweep,
    and the hit set shrinks as the threshold grows."""
    print("case: threshold sweep", flush=True)
    wl = W.c2_mid(n_clusters=64, per_cluster=16, n_queries=512, dim=256, sigma=0.5, seed=43)
    cache = siso.SisoCache(wl.dim, wl.K, siso.BF16)
    cache.load(to_dev(wl.centroids, "bf16"))
    q = to_dev(wl.queries, "bf16")
    outs = [tuple(t.clone() for t in cache.lookup(q, th)) for th in (0.75, 0.85, 0.92)]
    torch.cuda.synchronize()
    for o in outs[1:]:
        assert torch.equal(o[0], outs[0][0]) and torch.equal(o[1], outs[0][1])
    h = [o[2].cpu().numpy() for o in outs]
    assert np.all(h[1] <= h[0]) and np.all(h[2] <= h[1]) and h[0].sum() > h[2].sum()

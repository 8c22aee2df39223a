"""GPU parity where byte offsets into the stored centroids pass 2^32: more than 4 GiB of bf16 rows (and more than
8 GiB of running means).  The oracle cannot scan four million rows per query in seconds, so it runs on a sample of
the rows that holds every row a query was made from; a wrong 32-bit offset anywhere in the lookup, its final step or
the update would name, score or rewrite a row far from the one meant."""

import numpy as np
import pytest
import torch

from paper_2508_18736_amd import workloads as W
from gpu_util import DEV, check_lookup, to_dev, to_host

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(400)]

BLOCK = 65536
DIM = 512
K = (1 << 22) + 777       # 4 GiB + 777 KiB of bf16 rows
MEAN_TOL = 2e-6


@pytest.fixture(scope="module")
def siso():
    from paper_2508_18736_amd import siso as m
    return m


def rows_of(base: np.ndarray, ks: np.ndarray) -> np.ndarray:
    """Row k of the big matrix: row k mod 65,536 of the base block, rotated by k div 65,536 columns."""
    out = np.empty((len(ks), DIM), base.dtype)
    for j, k in enumerate(ks):
        out[j] = np.roll(base[k % BLOCK], k // BLOCK)
    return out


def test_rows_beyond_four_gib(siso, oracle):
    print(f"case: {K} centroids of {DIM} bf16 values: offsets beyond 2^32 bytes", flush=True)
    r = np.random.default_rng(2025)
    base = W.to_storage(W.uniform_directions(2025, 1, BLOCK, DIM), "bf16")
    dev_base = to_dev(base, "bf16")
    big = torch.empty((K, DIM), dtype=torch.bfloat16, device=DEV)
    for b in range((K + BLOCK - 1) // BLOCK):
        lo, hi = b * BLOCK, min(K, (b + 1) * BLOCK)
        big[lo:hi] = torch.roll(dev_base[:hi - lo], shifts=b, dims=1)
    cache = siso.SisoCache(DIM, K, siso.BF16)
    cache.load(big)
    torch.cuda.synchronize()
    print("loaded", flush=True)

    # queries near chosen rows: the ends, both sides of the 2 GiB and 4 GiB marks of the stored rows and of the means,
    # and rows spread over everything
    edge = np.array([0, 1, 255, 256, K - 1, K - 2, K - 256, K - 777, K - 778,
                     (1 << 21) - 1, 1 << 21, (1 << 21) + 1, (1 << 22) - 1, 1 << 22, (1 << 22) + 1, (1 << 22) + 300], np.int64)
    spread = r.choice(K, size=184, replace=False)
    targets = np.concatenate([edge, spread, edge[:8]])          # 208 queries, some rows asked for twice
    n = len(targets)
    noise = r.standard_normal((n, DIM)).astype(np.float32) * np.float32(0.25 / np.sqrt(DIM))
    q32 = W.storage_to_f32(rows_of(base, targets), "bf16") * r.uniform(0.5, 2.0, (n, 1)).astype(np.float32) + noise
    q32[-3:] = r.standard_normal((3, DIM)).astype(np.float32)     # three queries near nothing: misses
    queries = W.to_storage(q32, "bf16")
    q = to_dev(queries, "bf16")

    theta = 0.85
    idx, sim, hit = cache.lookup(q, theta)
    torch.cuda.synchronize()
    gi = idx.cpu().numpy()
    assert np.array_equal(gi[:-3], targets[:-3]) and hit.cpu().numpy()[:-3].all() and not hit.cpu().numpy()[-3:].any()

    # the oracle on a sample of the rows, in index order: the targets, what the three far queries were given, and 20,000 others
    sample = np.unique(np.concatenate([targets, gi[-3:].astype(np.int64), r.choice(K, size=20000, replace=False)]))
    sub = rows_of(base, sample)
    oc = oracle.OracleCache(DIM, len(sample), "bf16")
    oc.load(sub)
    ora = oc.lookup(queries, theta)
    where = np.searchsorted(sample, gi)
    assert np.array_equal(sample[where], gi)
    st = check_lookup((torch.from_numpy(where.astype(np.int32)), sim, hit), ora, theta, "bf16", "rows beyond 4 GiB")
    assert st["max_err"] < 1e-4 and st["clear"] >= n - 3

    # the same through the kernels for small batches (one block of queries, slices over all rows) and the k closest
    i64, s64, h64 = cache.lookup(q[:64], theta)
    ti, ts = cache.lookup_topk(q[:16], 4)
    torch.cuda.synchronize()
    assert torch.equal(i64, idx[:64]) and torch.equal(h64, hit[:64]) and (s64 - sim[:64]).abs().max().item() < 1e-5
    assert torch.equal(ti[:, 0], idx[:16]) and (ts[:, 0] - sim[:16]).abs().max().item() < 1e-5

    # fold the hits in, then one step of lookup and update in one call; compare the touched rows and their neighbours
    cache.update(q, idx, hit)
    oc.update(queries, np.where(ora[2] != 0, ora[0], -1))
    i2, s2, h2 = cache.lookup_update(q[:64], theta)
    torch.cuda.synchronize()
    o2 = oc.lookup(queries[:64], theta)
    check_lookup((torch.from_numpy(np.searchsorted(sample, i2.cpu().numpy()).astype(np.int32)), s2, h2), o2, theta, "bf16", "second step")
    oc.update(queries[:64], np.where(o2[2] != 0, o2[0], -1))
    assert cache.bad_indices() == 0
    gc, gm, gs = cache.export()
    torch.cuda.synchronize()
    oc_c, oc_m, oc_s = oc.export()
    pick = torch.from_numpy(sample).to(DEV)
    assert np.array_equal(gs[pick].cpu().numpy(), oc_s)
    assert int(gs.sum().item()) == K + int(hit.sum().item()) + int(h2.sum().item())
    err = np.abs(gm[pick].cpu().numpy().astype(np.float64) - oc_m).max()
    assert err <= MEAN_TOL, f"mean error {err:.3e}"
    g = to_host(gc[pick], "bf16")
    diff = g != oc_c
    assert diff.mean() < 2e-3
    assert np.abs(W.bf16_bits_to_f32(g).astype(np.float64) - W.bf16_bits_to_f32(oc_c).astype(np.float64)).max() <= 2.0 ** -8
    # nothing else was rewritten: every stored row outside the touched ones is still what was loaded
    touched = torch.zeros(K, dtype=torch.bool, device=DEV)
    touched[idx[hit.bool()].long()] = True
    touched[i2[h2.bool()].long()] = True
    same = (gc.view(torch.int16) == big.view(torch.int16)).all(dim=1)
    assert bool((same | touched).all()) and int(touched.sum().item()) == len(np.unique(targets[:-3]))


def test_codes_beyond_four_gib(siso, oracle):
    import gpu_util
    gpu_util.SIM_TOL.setdefault("fp8", 5e-4)
    K8 = (1 << 23) + 300      # 4 GiB + 150 KiB of 8-bit codes
    print(f"case: {K8} centroids of {DIM} 8-bit codes: offsets beyond 2^32 bytes", flush=True)
    r = np.random.default_rng(2026)
    base = W.to_storage(W.uniform_directions(2026, 1, BLOCK, DIM), "bf16")
    dev_base = to_dev(base, "bf16")
    cache = siso.SisoCache(DIM, K8, siso.FP8)
    big = torch.empty((K8, DIM), dtype=torch.bfloat16, device=DEV)
    for b in range((K8 + BLOCK - 1) // BLOCK):
        lo, hi = b * BLOCK, min(K8, (b + 1) * BLOCK)
        big[lo:hi] = torch.roll(dev_base[:hi - lo], shifts=b, dims=1)
    cache.load(big)
    torch.cuda.synchronize()
    del big
    print("loaded", flush=True)
    edge = np.array([0, 255, 256, K8 - 1, K8 - 300, K8 - 301, (1 << 22) - 1, 1 << 22, (1 << 23) - 1, 1 << 23, (1 << 23) + 1], np.int64)
    targets = np.concatenate([edge, r.choice(K8, size=139, replace=False)])
    n = len(targets)
    noise = r.standard_normal((n, DIM)).astype(np.float32) * np.float32(0.25 / np.sqrt(DIM))
    queries = W.to_storage(W.storage_to_f32(rows_of(base, targets), "bf16") + noise, "bf16")
    q = to_dev(queries, "bf16")
    idx, sim, hit = cache.lookup(q, 0.85)
    i64, s64, h64 = cache.lookup(q[:64], 0.85)
    ti, ts = cache.lookup_topk(q[:16], 4)
    torch.cuda.synchronize()
    gi = idx.cpu().numpy()
    assert np.array_equal(gi, targets) and hit.cpu().numpy().all()
    assert torch.equal(i64, idx[:64]) and torch.equal(h64, hit[:64]) and (s64 - sim[:64]).abs().max().item() < 1e-5
    assert torch.equal(ti[:, 0], idx[:16]) and (ts[:, 0] - sim[:16]).abs().max().item() < 1e-5
    sample = np.unique(np.concatenate([targets, r.choice(K8, size=20000, replace=False)]))
    oc, os_ = oracle.fp8_quantize(rows_of(base, sample), "bf16")
    codes, scales, _ = cache.export_fp8()
    pick = torch.from_numpy(sample).to(DEV)
    assert np.array_equal(codes[pick].cpu().numpy(), oc) and np.array_equal(scales[pick].cpu().numpy().view(np.uint32), os_.view(np.uint32))
    ora = oracle.fp8_lookup_rows(oc, os_, queries, 0.85)
    where = np.searchsorted(sample, gi)
    st = check_lookup((torch.from_numpy(where.astype(np.int32)), sim, hit), ora, 0.85, "fp8", "codes beyond 4 GiB")
    assert st["max_err"] < 2e-5 and st["clear"] == n

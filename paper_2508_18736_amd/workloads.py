"""Seeded synthetic inputs for the centroid-cache hot path.

Real query embeddings (the paper clusters question datasets into roughly one
centroid per ten queries, section 3.1, and observes skewed, slowly drifting
centroid popularity, section 3.2) are replaced by Gaussian mixtures on the unit
sphere.  This module only *draws inputs*: it contains no part of the lookup,
update or merge arithmetic, and it is the one module that both the CPU oracle's
tests and the GPU path's tests may import.

Everything is generated on the host with numpy's counter-based Philox
generator, keyed by ``(seed, stream, chunk)`` so that the result does not depend
on the number of worker threads.  Vectors are normalised in float32 and then
rounded (round-to-nearest-even) to the storage type.  bf16 arrays are carried
as ``uint16`` bit patterns, because numpy has no bf16 type.

``sigma_mode``:
  ``"total"``   - the noise *vector* has expected length ``sigma`` (per-dimension
                  standard deviation ``sigma / sqrt(dim)``); members of one
                  cluster then have cosine about ``1 / (1 + sigma**2)``.
  ``"per_dim"`` - every coordinate gets standard deviation ``sigma``; at the
                  dimensions used here members of one cluster are then almost
                  orthogonal and nothing ever crosses a threshold.
"""

from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

BASE_SEED = 0x5150

_STREAM_MEANS = 1
_STREAM_MEMBERS = 2
_STREAM_QUERIES = 3
_STREAM_PERM = 4
_STREAM_POP = 5
_STREAM_MISC = 6


# --------------------------------------------------------------------------- #
# storage formats
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even.

    NaN inputs become a quiet NaN; finite inputs that round past the largest
    bf16 become infinity, as the format prescribes."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    out = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32, exact."""
    u = np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(x)
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------- #
# random streams
# --------------------------------------------------------------------------- #
def _rng(seed: int, stream: int, chunk: int = 0) -> np.random.Generator:
    key = (np.uint64(seed) << np.uint64(32)) | (np.uint64(stream) << np.uint64(24)) | np.uint64(chunk)
    return np.random.Generator(np.random.Philox(key=int(key)))


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _unit_rows(x: np.ndarray) -> np.ndarray:
    n = np.sqrt(np.einsum("ij,ij->i", x, x, dtype=np.float32))[:, None]
    return x / n


def _noise_scale(sigma: float, dim: int, sigma_mode: str) -> np.float32:
    if sigma_mode == "total":
        return np.float32(sigma / np.sqrt(dim))
    if sigma_mode == "per_dim":
        return np.float32(sigma)
    raise ValueError(f"unknown sigma_mode {sigma_mode!r}")


_CHUNK_ROWS = 8192


def uniform_directions(seed: int, stream: int, n: int, dim: int) -> np.ndarray:
    """``n`` float32 unit vectors, uniform on the sphere (normalised Gaussians)."""
    out = np.empty((n, dim), dtype=np.float32)

    def work(c: int) -> None:
        lo, hi = c * _CHUNK_ROWS, min(n, (c + 1) * _CHUNK_ROWS)
        g = _rng(seed, stream, c).standard_normal((hi - lo, dim), dtype=np.float32)
        out[lo:hi] = _unit_rows(g)

    chunks = range((n + _CHUNK_ROWS - 1) // _CHUNK_ROWS)
    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(work, chunks))
    return out


def jitter(seed: int, stream: int, base: np.ndarray, rows: np.ndarray, sigma: float,
           sigma_mode: str, dtype: str) -> np.ndarray:
    """``normalize(base[rows[i]] + noise_i)`` for every i, rounded to ``dtype``.

    ``base`` holds float32 unit vectors; the result has ``len(rows)`` rows in the
    storage type."""
    n, dim = len(rows), base.shape[1]
    s = _noise_scale(sigma, dim, sigma_mode)
    out = np.empty((n, dim), dtype=np.float32 if dtype == "f32" else np.uint16)

    def work(c: int) -> None:
        lo, hi = c * _CHUNK_ROWS, min(n, (c + 1) * _CHUNK_ROWS)
        g = _rng(seed, stream, c).standard_normal((hi - lo, dim), dtype=np.float32)
        g *= s
        g += base[rows[lo:hi]]
        out[lo:hi] = to_storage(_unit_rows(g), dtype)

    chunks = range((n + _CHUNK_ROWS - 1) // _CHUNK_ROWS)
    with ThreadPoolExecutor(_workers()) as ex:
        list(ex.map(work, chunks))
    return out


def zipf_probabilities(n: int, s: float) -> np.ndarray:
    """p(rank r) proportional to r**-s for r = 1..n (float64, sums to 1)."""
    p = np.arange(1, n + 1, dtype=np.float64) ** (-s)
    return p / p.sum()


# --------------------------------------------------------------------------- #
# workloads
# --------------------------------------------------------------------------- #
@dataclass
class Workload:
    """One synthetic configuration.

    ``centroids``: ``[K, dim]`` in the storage type (float32, or uint16 bf16 bits).
    ``queries``:   ``[n, dim]`` in the storage type (for the streaming workload
                   ``n = batches * batch`` and batch b is rows ``b*batch .. (b+1)*batch``).
    ``planted``:   for each query the centroid index it was drawn next to, or -1
                   for a fresh uniform direction.
    ``cluster_of``: for each centroid the mixture component it came from.
    """

    name: str
    dim: int
    dtype: str
    centroids: np.ndarray
    cluster_of: np.ndarray
    queries: Optional[np.ndarray] = None
    planted: Optional[np.ndarray] = None
    thresholds: Sequence[float] = ()
    batch: Optional[int] = None
    meta: Dict[str, object] = field(default_factory=dict)

    @property
    def K(self) -> int:
        return int(self.centroids.shape[0])

    @property
    def n(self) -> int:
        return 0 if self.queries is None else int(self.queries.shape[0])

    def centroids_f32(self) -> np.ndarray:
        return storage_to_f32(self.centroids, self.dtype)

    def queries_f32(self) -> np.ndarray:
        return storage_to_f32(self.queries, self.dtype)


def into_cone(x: np.ndarray, seed: int, cone: float) -> np.ndarray:
    """``normalize(x_i + cone * e)`` with one seeded unit direction ``e`` shared by all rows: two
    unrelated rows then have cosine about ``cone^2 / (1 + cone^2)`` instead of about 0, the way
    text embeddings of unrelated sentences sit in a cone (``cone`` = 1.28 gives 0.62)."""
    if cone == 0.0:
        return x
    e = uniform_directions(seed, _STREAM_MISC + 1, 1, x.shape[1])[0]
    return _unit_rows(x + np.float32(cone) * e)


def mixture_centroids(seed: int, n_clusters: int, per_cluster: int, dim: int, sigma: float,
                      sigma_mode: str, dtype: str, shuffle: bool = True, cone: float = 0.0):
    """Cluster means uniform on the sphere (or in a cone, see ``into_cone``); every centroid is a
    jittered copy of its mean.  Returns ``(centroids_storage, cluster_of, means_f32)``.  With
    ``shuffle`` the rows are put in a seeded random order, so that members of a
    cluster are spread over the array instead of sitting side by side."""
    means = into_cone(uniform_directions(seed, _STREAM_MEANS, n_clusters, dim), seed, cone)
    cluster_of = np.repeat(np.arange(n_clusters, dtype=np.int32), per_cluster)
    if shuffle:
        cluster_of = cluster_of[_rng(seed, _STREAM_PERM).permutation(len(cluster_of))]
    cents = jitter(seed, _STREAM_MEMBERS, means, cluster_of, sigma, sigma_mode, dtype)
    return cents, cluster_of, means


def _members_by_cluster(cluster_of: np.ndarray, n_clusters: int):
    order = np.argsort(cluster_of, kind="stable").astype(np.int64)
    starts = np.searchsorted(cluster_of[order], np.arange(n_clusters + 1))
    return order, starts


def _queries_near(seed: int, cents_f32: np.ndarray, targets: np.ndarray, sigma: float,
                  sigma_mode: str, dtype: str) -> np.ndarray:
    return jitter(seed, _STREAM_QUERIES, cents_f32, targets, sigma, sigma_mode, dtype)


def c1_tiny(n_clusters: int = 64, per_cluster: int = 16, n_queries: int = 256, dim: int = 384,
            sigma: float = 0.1, sigma_mode: str = "total", seed: int = BASE_SEED + 1) -> Workload:
    """Tiny fp32 lookup: a 64-component mixture, 1,024 centroids, 256 queries drawn
    as further members of random components; threshold 0.80."""
    cents, cluster_of, means = mixture_centroids(seed, n_clusters, per_cluster, dim, sigma, sigma_mode, "f32")
    r = _rng(seed, _STREAM_POP)
    qc = r.integers(0, n_clusters, size=n_queries).astype(np.int64)
    queries = jitter(seed, _STREAM_QUERIES, means, qc, sigma, sigma_mode, "f32")
    return Workload("c1_tiny", dim, "f32", cents, cluster_of, queries,
                    np.full(n_queries, -1, np.int64), (0.80,),
                    meta={"query_cluster": qc, "sigma": sigma, "sigma_mode": sigma_mode})


def c2_mid(n_clusters: int = 4096, per_cluster: int = 16, n_queries: int = 4096, dim: int = 768,
           sigma: float = 0.08, near_fraction: float = 0.7, sigma_mode: str = "total",
           dtype: str = "bf16", seed: int = BASE_SEED + 2, cone: float = 0.0) -> Workload:
    """Mid lookup: 65,536 bf16 centroids; 70 % of the queries are jittered copies of
    a random existing centroid (its index is recorded in ``planted``), 30 % are
    fresh uniform directions.  Thresholds 0.75 / 0.85 / 0.92."""
    cents, cluster_of, _ = mixture_centroids(seed, n_clusters, per_cluster, dim, sigma, sigma_mode, dtype, cone=cone)
    K = cents.shape[0]
    r = _rng(seed, _STREAM_POP)
    near = r.random(n_queries) < near_fraction
    targets = r.integers(0, K, size=n_queries).astype(np.int64)
    cf = storage_to_f32(cents, dtype)
    queries = _queries_near(seed, cf, targets, sigma, sigma_mode, dtype)
    fresh = to_storage(into_cone(uniform_directions(seed, _STREAM_MISC, n_queries, dim), seed, cone), dtype)
    queries[~near] = fresh[~near]
    planted = np.where(near, targets, -1)
    return Workload("c2_mid", dim, dtype, cents, cluster_of, queries, planted, (0.75, 0.85, 0.92),
                    meta={"sigma": sigma, "sigma_mode": sigma_mode, "cone": cone})


def spread_sample(centroids: np.ndarray, dtype: str, n_queries: int, sigma_lo: float = 0.1,
                  sigma_hi: float = 1.3, seed: int = BASE_SEED + 6) -> np.ndarray:
    """Sample queries for a threshold-to-hit-ratio table: query i is a jittered copy of a random
    stored centroid with its own noise length, drawn uniformly from ``[sigma_lo, sigma_hi]`` (the
    length of the whole noise vector), so that the top-1 similarities spread over roughly
    ``1/sqrt(1 + sigma^2)`` = 0.61 .. 0.995 and the hit ratio falls gradually as the threshold
    rises, like the curves measured on text embeddings.  Returns rows in the storage type."""
    K, dim = centroids.shape
    r = _rng(seed, _STREAM_POP)
    targets = r.integers(0, K, size=n_queries).astype(np.int64)
    lengths = r.uniform(sigma_lo, sigma_hi, size=n_queries).astype(np.float32)
    cf = storage_to_f32(centroids, dtype)
    out = np.empty((n_queries, dim), dtype=np.float32 if dtype == "f32" else np.uint16)
    for c in range((n_queries + _CHUNK_ROWS - 1) // _CHUNK_ROWS):
        lo, hi = c * _CHUNK_ROWS, min(n_queries, (c + 1) * _CHUNK_ROWS)
        g = _rng(seed, _STREAM_QUERIES, c).standard_normal((hi - lo, dim), dtype=np.float32)
        g *= (lengths[lo:hi] / np.sqrt(np.float32(dim)))[:, None]
        g += cf[targets[lo:hi]]
        out[lo:hi] = to_storage(_unit_rows(g), dtype)
    return out


def _popular_targets(r: np.random.Generator, p: np.ndarray, rank_to_cluster: np.ndarray,
                     order: np.ndarray, starts: np.ndarray, n: int) -> np.ndarray:
    ranks = r.choice(len(p), size=n, p=p)
    cl = rank_to_cluster[ranks]
    size = starts[cl + 1] - starts[cl]
    pick = (r.random(n) * size).astype(np.int64)
    return order[starts[cl] + np.minimum(pick, size - 1)]


def c3_large(n_clusters: int = 32768, per_cluster: int = 32, n_queries: int = 16384, dim: int = 1024,
             sigma: float = 0.06, zipf_s: float = 1.1, sigma_mode: str = "total",
             dtype: str = "bf16", seed: int = BASE_SEED + 3) -> Workload:
    """Large lookup: 1,048,576 bf16 centroids (2 GiB at dim 1,024); the cluster of each
    query follows a Zipf law over a seeded ranking of the clusters, and the query is
    a jittered copy of a random centroid of that cluster.  Threshold 0.85."""
    cents, cluster_of, _ = mixture_centroids(seed, n_clusters, per_cluster, dim, sigma, sigma_mode, dtype)
    order, starts = _members_by_cluster(cluster_of, n_clusters)
    r = _rng(seed, _STREAM_POP)
    rank_to_cluster = r.permutation(n_clusters)
    targets = _popular_targets(r, zipf_probabilities(n_clusters, zipf_s), rank_to_cluster, order, starts, n_queries)
    # only the rows that are needed are widened (the full array would be 4 GiB)
    uniq, inv = np.unique(targets, return_inverse=True)
    base = storage_to_f32(cents[uniq], dtype)
    queries = jitter(seed, _STREAM_QUERIES, base, inv, sigma, sigma_mode, dtype)
    return Workload("c3_large", dim, dtype, cents, cluster_of, queries, targets, (0.85,),
                    meta={"sigma": sigma, "sigma_mode": sigma_mode, "zipf_s": zipf_s})


def c4_stream(n_clusters: int = 16384, per_cluster: int = 16, batches: int = 4096, batch: int = 64,
              dim: int = 768, sigma: float = 0.08, zipf_s: float = 1.2, drift_every: int = 512,
              sigma_mode: str = "total", dtype: str = "bf16", seed: int = BASE_SEED + 4) -> Workload:
    """Streaming lookup: 262,144 bf16 centroids and a stream of micro-batches of 64
    queries.  Cluster popularity is Zipf(1.2); the ranking of the clusters is re-drawn
    every ``drift_every`` batches.  Threshold 0.85."""
    cents, cluster_of, _ = mixture_centroids(seed, n_clusters, per_cluster, dim, sigma, sigma_mode, dtype)
    order, starts = _members_by_cluster(cluster_of, n_clusters)
    r = _rng(seed, _STREAM_POP)
    p = zipf_probabilities(n_clusters, zipf_s)
    targets = np.empty(batches * batch, dtype=np.int64)
    for e0 in range(0, batches, drift_every):
        e1 = min(batches, e0 + drift_every)
        rank_to_cluster = r.permutation(n_clusters)
        targets[e0 * batch:e1 * batch] = _popular_targets(r, p, rank_to_cluster, order, starts, (e1 - e0) * batch)
    uniq, inv = np.unique(targets, return_inverse=True)
    base = storage_to_f32(cents[uniq], dtype)
    queries = jitter(seed, _STREAM_QUERIES, base, inv, sigma, sigma_mode, dtype)
    return Workload("c4_stream", dim, dtype, cents, cluster_of, queries, targets, (0.85,), batch=batch,
                    meta={"sigma": sigma, "sigma_mode": sigma_mode, "zipf_s": zipf_s,
                          "drift_every": drift_every, "batches": batches})


def c5_merge(n_groups: int = 16384, copies: int = 8, dim: int = 768, sigma: float = 0.03,
             sigma_mode: str = "total", dtype: str = "bf16", seed: int = BASE_SEED + 5) -> Workload:
    """Merge workload: every cluster mean appears as ``copies`` jittered near-duplicates,
    in a seeded random order.  With the default noise the copies of one mean have
    cosine about 0.999 and different means are almost orthogonal, so at threshold
    0.90 the pairs above threshold are exactly the ``n_groups * C(copies, 2)`` pairs
    inside groups (``cluster_of`` gives the group of each row)."""
    cents, cluster_of, _ = mixture_centroids(seed, n_groups, copies, dim, sigma, sigma_mode, dtype)
    return Workload("c5_merge", dim, dtype, cents, cluster_of, None, None, (0.90,),
                    meta={"sigma": sigma, "sigma_mode": sigma_mode, "copies": copies,
                          "expected_pairs": n_groups * copies * (copies - 1) // 2})


def random_counts(seed: int, k: int, lo: int = 1, hi: int = 100) -> np.ndarray:
    """Seeded per-centroid cluster sizes in ``[lo, hi]`` (int32)."""
    return _rng(seed, _STREAM_MISC, 7).integers(lo, hi + 1, size=k).astype(np.int32)


FULL_CONFIGS = {
    "c1_tiny": c1_tiny,
    "c2_mid": c2_mid,
    "c3_large": c3_large,
    "c4_stream": c4_stream,
    "c5_merge": c5_merge,
}


def query_log_chains(n_chains: int = 24, chain_len: int = 5, members_lo: int = 2, members_hi: int = 12,
                     n_noise: int = 64, dim: int = 256, step_cos: float = 0.90, sigma: float = 0.1,
                     dtype: str = "bf16", seed: int = BASE_SEED + 8):
    """A query log for clustering: topics whose members are jittered copies of a topic direction
    (noise of total length ``sigma``: cosine to the direction about ``1/sqrt(1+sigma^2)``), the
    topics strung into chains in which neighbouring directions have cosine ``step_cos`` and
    directions two apart about ``step_cos**2``; plus ``n_noise`` unrelated directions; all in a
    seeded random order.  With the defaults members of one topic have cosine about 0.99, members
    of neighbouring topics about 0.89, two apart at most 0.84: at a clustering threshold of 0.86
    neighbourhoods overlap along a chain, so what a greedy clustering returns depends on its
    order, and no cosine comes close to the threshold.  Returns ``(rows in the storage type,
    topic of every row, -1 for the unrelated ones)``."""
    r = _rng(seed, _STREAM_MISC, 11)
    topics = n_chains * chain_len
    start = uniform_directions(seed, _STREAM_MEANS, n_chains, dim)
    turn = uniform_directions(seed, _STREAM_MEMBERS, topics, dim)
    dirs = np.empty((topics, dim), np.float32)
    side = np.float32(np.sqrt(1.0 - step_cos * step_cos))
    for c in range(n_chains):
        cur = start[c]
        for s in range(chain_len):
            t = c * chain_len + s
            if s > 0:
                u = turn[t] - np.dot(turn[t], cur) * cur          # a direction at right angles to the last one
                u /= np.sqrt(np.dot(u, u))
                cur = np.float32(step_cos) * cur + side * u
                cur /= np.sqrt(np.dot(cur, cur))
            dirs[t] = cur
    members = r.integers(members_lo, members_hi + 1, size=topics)
    topic_of = np.concatenate([np.repeat(np.arange(topics), members), np.full(n_noise, -1)]).astype(np.int64)
    base = np.concatenate([dirs, uniform_directions(seed, _STREAM_PERM, max(n_noise, 1), dim)[:n_noise]])
    rows_of = np.where(topic_of >= 0, topic_of, topics + np.arange(len(topic_of)) - int(members.sum()))
    perm = r.permutation(len(topic_of))
    topic_of, rows_of = topic_of[perm], rows_of[perm]
    noise = np.where(topic_of >= 0, np.float32(sigma), np.float32(0.0))
    out = np.empty((len(topic_of), dim), dtype=np.float32 if dtype == "f32" else np.uint16)
    g = _rng(seed, _STREAM_QUERIES, 1).standard_normal((len(topic_of), dim), dtype=np.float32)
    g *= (noise / np.sqrt(np.float32(dim)))[:, None]
    g += base[rows_of]
    out[:] = to_storage(_unit_rows(g), dtype)
    return out, topic_of

"""ctypes binding of the CPU oracle (``siso_oracle.c``).

TEST INFRASTRUCTURE: only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package.  It shares no code
with the GPU library.  All arrays are numpy host arrays; bf16 data is carried as
``uint16`` bit patterns.
"""

from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "siso_oracle.c")
_LIB = os.path.join(_HERE, "libsiso_oracle.so")

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (generic x86-64 code, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        vp, lg, it, fl = C.c_void_p, C.c_long, C.c_int, C.c_float
        L.oracle_lookup_rows.argtypes = [vp, lg, it, it, vp, lg, fl, vp, vp, vp, vp]
        L.oracle_lookup_rows.restype = it
        L.oracle_create.argtypes = [it, lg, it, C.POINTER(vp)]
        L.oracle_create.restype = it
        L.oracle_destroy.argtypes = [vp]
        L.oracle_destroy.restype = None
        L.oracle_count.argtypes = [vp]
        L.oracle_count.restype = lg
        L.oracle_load.argtypes = [vp, vp, vp, lg]
        L.oracle_load.restype = it
        L.oracle_lookup.argtypes = [vp, vp, lg, fl, vp, vp, vp, vp]
        L.oracle_lookup.restype = it
        L.oracle_update.argtypes = [vp, vp, vp, lg]
        L.oracle_update.restype = it
        L.oracle_merge.argtypes = [vp, fl, vp, lg]
        L.oracle_merge.restype = lg
        L.oracle_merge_apply.argtypes = [vp, vp, lg, vp]
        L.oracle_merge_apply.restype = it
        L.oracle_export.argtypes = [vp, vp, vp, vp]
        L.oracle_export.restype = it
        L.oracle_threads.argtypes = []
        L.oracle_threads.restype = it
        L.oracle_export_meta.argtypes = [vp, vp, vp]
        L.oracle_export_meta.restype = it
        L.oracle_lookup_multi.argtypes = [vp, vp, lg, vp, it, it, vp, vp, vp, vp]
        L.oracle_lookup_multi.restype = it
        L.oracle_lookup_topk.argtypes = [vp, vp, lg, it, vp, vp]
        L.oracle_lookup_topk.restype = it
        L.oracle_fp8_quantize.argtypes = [vp, it, lg, it, vp, vp]
        L.oracle_fp8_quantize.restype = it
        L.oracle_fp8_lookup_rows.argtypes = [vp, vp, lg, it, vp, it, lg, fl, vp, vp, vp, vp]
        L.oracle_fp8_lookup_rows.restype = it
        L.oracle_fp8_lookup_topk_rows.argtypes = [vp, vp, lg, it, vp, it, lg, it, vp, vp]
        L.oracle_fp8_lookup_topk_rows.restype = it
        L.oracle_import.argtypes = [vp, vp, vp, vp, vp, vp, lg]
        L.oracle_import.restype = it
        L.oracle_refresh.argtypes = [vp, vp, vp, lg, fl, lg, vp, vp]
        L.oracle_refresh.restype = it
        L.oracle_refresh_gap.argtypes = [vp, vp, vp, lg, fl, lg, vp, vp, vp]
        L.oracle_refresh_gap.restype = it
        db = C.c_double
        L.oracle_t2h.argtypes = [vp, vp, lg, vp, it, vp]
        L.oracle_t2h.restype = it
        L.oracle_md1_wait.argtypes = [db, db, db]
        L.oracle_md1_wait.restype = db
        L.oracle_pick_threshold.argtypes = [vp, vp, it, db, db, db]
        L.oracle_pick_threshold.restype = it
        L.oracle_adjust_threshold.argtypes = [vp, it, it, db, db]
        L.oracle_adjust_threshold.restype = it
        L.oracle_cluster.argtypes = [vp, vp, lg, fl, it, vp, vp, vp, vp, vp]
        L.oracle_cluster.restype = lg
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().oracle_threads())


def _storage(x: np.ndarray, dtype: str, dim: int) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    x = np.ascontiguousarray(x)
    if x.dtype != want:
        raise TypeError(f"expected {want} rows for dtype {dtype}, got {x.dtype}")
    if x.ndim != 2 or x.shape[1] != dim:
        raise ValueError(f"expected [*, {dim}] rows, got {x.shape}")
    return x


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def lookup_rows(centroids: np.ndarray, queries: np.ndarray, threshold: float, dtype: str,
                want_second: bool = True):
    """Stateless lookup.  Returns ``(idx int32, sim float64, hit uint8, second float64|None)``."""
    dim = int(queries.shape[1]) if queries.ndim == 2 else int(centroids.shape[1])
    cents = _storage(centroids, dtype, dim)
    qs = _storage(queries, dtype, dim)
    n = qs.shape[0]
    idx = np.empty(n, np.int32)
    sim = np.empty(n, np.float64)
    hit = np.empty(n, np.uint8)
    second = np.empty(n, np.float64) if want_second else None
    rc = lib().oracle_lookup_rows(_ptr(cents), cents.shape[0], dim, _DT[dtype], _ptr(qs), n,
                                  float(threshold), _ptr(idx), _ptr(sim), _ptr(hit), _ptr(second))
    if rc != 0:
        raise RuntimeError(f"oracle_lookup_rows failed ({rc})")
    return idx, sim, hit, second


def fp8_quantize(rows: np.ndarray, dtype: str):
    """Rows of the input type -> ``(codes uint8 [n, dim], scales float32 [n])`` in the 8-bit storage format."""
    x = _storage(rows, dtype, rows.shape[1])
    n, dim = x.shape
    codes = np.zeros((n, dim), np.uint8)
    scales = np.zeros(n, np.float32)
    rc = lib().oracle_fp8_quantize(_ptr(x), _DT[dtype], n, dim, _ptr(codes), _ptr(scales))
    if rc != 0:
        raise RuntimeError(f"oracle_fp8_quantize failed ({rc})")
    return codes, scales


def fp8_lookup_rows(cent_codes: np.ndarray, cent_scales: np.ndarray, queries: np.ndarray, threshold: float,
                    qdtype: str = "bf16"):
    """Lookup over rows stored in the 8-bit format (queries are quantised the same way).
    Returns ``(idx int32, sim float64, hit uint8, second float64)``."""
    cc = np.ascontiguousarray(cent_codes, dtype=np.uint8)
    cs = np.ascontiguousarray(cent_scales, dtype=np.float32)
    k, dim = cc.shape
    qs = _storage(queries, qdtype, dim)
    n = qs.shape[0]
    idx = np.empty(n, np.int32)
    sim = np.empty(n, np.float64)
    hit = np.empty(n, np.uint8)
    second = np.empty(n, np.float64)
    rc = lib().oracle_fp8_lookup_rows(_ptr(cc), _ptr(cs), k, dim, _ptr(qs), _DT[qdtype], n, float(threshold), _ptr(idx),
                                      _ptr(sim), _ptr(hit), _ptr(second))
    if rc != 0:
        raise RuntimeError(f"oracle_fp8_lookup_rows failed ({rc})")
    return idx, sim, hit, second


def fp8_lookup_topk_rows(cent_codes: np.ndarray, cent_scales: np.ndarray, queries: np.ndarray, k: int,
                         qdtype: str = "bf16"):
    """The k closest rows of an 8-bit store per query: ``(idx int32 [n, k], sim float64 [n, k])``."""
    cc = np.ascontiguousarray(cent_codes, dtype=np.uint8)
    cs = np.ascontiguousarray(cent_scales, dtype=np.float32)
    rows, dim = cc.shape
    qs = _storage(queries, qdtype, dim)
    n = qs.shape[0]
    idx = np.empty((n, int(k)), np.int32)
    sim = np.empty((n, int(k)), np.float64)
    rc = lib().oracle_fp8_lookup_topk_rows(_ptr(cc), _ptr(cs), rows, dim, _ptr(qs), _DT[qdtype], n, int(k), _ptr(idx),
                                           _ptr(sim))
    if rc != 0:
        raise RuntimeError(f"oracle_fp8_lookup_topk_rows failed ({rc})")
    return idx, sim


def md1_wait(L: float, lam: float, h: float) -> float:
    """Expected M/D/1 waiting time at hit ratio ``h`` (inf when the queue is unstable)."""
    return float(lib().oracle_md1_wait(float(L), float(lam), float(h)))


def pick_threshold(thetas, hit_ratio, L: float, lam: float, slo: float) -> int:
    """Position of the highest threshold with ``slo > W``; -1 if none."""
    th = np.ascontiguousarray(thetas, dtype=np.float32)
    hr = np.ascontiguousarray(hit_ratio, dtype=np.float64)
    assert th.shape == hr.shape and th.ndim == 1
    return int(lib().oracle_pick_threshold(_ptr(th), _ptr(hr), th.shape[0], float(L), float(lam), float(slo)))


def adjust_threshold(thetas, index: int, w_est: float, w_actual: float) -> int:
    """Position after the 10 % correction."""
    th = np.ascontiguousarray(thetas, dtype=np.float32)
    return int(lib().oracle_adjust_threshold(_ptr(th), th.shape[0], int(index), float(w_est), float(w_actual)))


class OracleCache:
    """The oracle's cache object: stored centroids, exact means (float64), cluster sizes."""

    def __init__(self, dim: int, capacity: int, dtype: str = "bf16"):
        self.dim, self.capacity, self.dtype = int(dim), int(capacity), dtype
        h = C.c_void_p()
        rc = lib().oracle_create(self.dim, self.capacity, _DT[dtype], C.byref(h))
        if rc != 0:
            raise RuntimeError(f"oracle_create failed ({rc})")
        self._h = h

    def close(self) -> None:
        if self._h:
            lib().oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def count(self) -> int:
        return int(lib().oracle_count(self._h))

    def load(self, centroids: np.ndarray, counts: Optional[np.ndarray] = None) -> None:
        cents = _storage(centroids, self.dtype, self.dim)
        cn = None if counts is None else np.ascontiguousarray(counts, dtype=np.int32)
        rc = lib().oracle_load(self._h, _ptr(cents), _ptr(cn), cents.shape[0])
        if rc != 0:
            raise RuntimeError(f"oracle_load failed ({rc})")

    def import_state(self, centroids: np.ndarray, means: np.ndarray, sizes: np.ndarray,
                     cluster_size: Optional[np.ndarray] = None, access_count: Optional[np.ndarray] = None) -> None:
        """Take over a snapshot as it is: stored rows, means (float64), sizes, and the two numbers of
        Algorithm 1 per row (default: cluster_size = size, access_count = 0)."""
        cents = _storage(centroids, self.dtype, self.dim)
        k = cents.shape[0]
        mm = np.ascontiguousarray(means, dtype=np.float64)
        sz = np.ascontiguousarray(sizes, dtype=np.int32)
        loc = None if cluster_size is None else np.ascontiguousarray(cluster_size, dtype=np.float32)
        acc = None if access_count is None else np.ascontiguousarray(access_count, dtype=np.uint32)
        assert mm.shape == (k, self.dim) and sz.shape == (k,)
        assert loc is None or loc.shape == (k,)
        assert acc is None or acc.shape == (k,)
        rc = lib().oracle_import(self._h, _ptr(cents), _ptr(mm), _ptr(sz), _ptr(loc), _ptr(acc), k)
        if rc != 0:
            raise RuntimeError(f"oracle_import failed ({rc})")

    def export_meta(self):
        """``(cluster_size float32, access_count uint32)`` of the live rows; 0xFFFFFFFF = infinity."""
        k = self.count
        loc = np.empty(k, np.float32)
        acc = np.empty(k, np.uint32)
        rc = lib().oracle_export_meta(self._h, _ptr(loc), _ptr(acc))
        if rc != 0:
            raise RuntimeError(f"oracle_export_meta failed ({rc})")
        return loc, acc

    def refresh(self, repo: np.ndarray, repo_size, theta_c: float, max_centroids: int, want_gap: bool = False):
        """Algorithm 1.  Returns ``(merged, added, evicted, min_margin)``; with ``want_gap`` a fifth entry: the
        smallest lead of the closest centroid over the second-closest among the rows that were merged."""
        rows = _storage(repo, self.dtype, self.dim)
        sizes = np.ascontiguousarray(repo_size, dtype=np.float32)
        assert sizes.shape == (rows.shape[0],)
        stats = np.zeros(3, np.int64)
        margin = C.c_double(0.0)
        gap = C.c_double(0.0)
        rc = lib().oracle_refresh_gap(self._h, _ptr(rows), _ptr(sizes), rows.shape[0], float(theta_c),
                                      int(max_centroids), _ptr(stats), C.byref(margin), C.byref(gap) if want_gap else None)
        if rc != 0:
            raise RuntimeError(f"oracle_refresh failed ({rc})")
        out = (int(stats[0]), int(stats[1]), int(stats[2]), float(margin.value))
        return out + (float(gap.value),) if want_gap else out

    def cluster(self, vectors: np.ndarray, theta_c: float, min_size: int = 1, representatives: bool = False):
        """Community detection; the cache becomes the repository of the clusters.
        Returns ``(labels int32 [n], seeds int32 [clusters], min_margin)``, with ``representatives``
        also ``(rep int32 [clusters], rep_gap float64 [clusters])``: the member closest to each centroid."""
        rows = _storage(vectors, self.dtype, self.dim)
        n = rows.shape[0]
        labels = np.full(n, -1, np.int32)
        seeds = np.zeros(max(n, 1), np.int32)
        rep = np.zeros(max(n, 1), np.int32)
        gap = np.zeros(max(n, 1), np.float64)
        margin = C.c_double(0.0)
        rc = lib().oracle_cluster(self._h, _ptr(rows), n, float(theta_c), int(min_size), _ptr(labels), _ptr(seeds),
                                  _ptr(rep), _ptr(gap), C.byref(margin))
        if rc < 0:
            raise RuntimeError(f"oracle_cluster failed ({rc})")
        if representatives:
            return labels, seeds[:rc].copy(), float(margin.value), rep[:rc].copy(), gap[:rc].copy()
        return labels, seeds[:rc].copy(), float(margin.value)

    def t2h(self, queries: np.ndarray, thetas) -> np.ndarray:
        """Hits per threshold (int64) of the sample queries."""
        qs = _storage(queries, self.dtype, self.dim)
        th = np.ascontiguousarray(thetas, dtype=np.float32)
        hits = np.zeros(th.shape[0], np.int64)
        rc = lib().oracle_t2h(self._h, _ptr(qs), qs.shape[0], _ptr(th), th.shape[0], _ptr(hits))
        if rc != 0:
            raise RuntimeError(f"oracle_t2h failed ({rc})")
        return hits

    def lookup(self, queries: np.ndarray, threshold: float, want_second: bool = True):
        qs = _storage(queries, self.dtype, self.dim)
        n = qs.shape[0]
        idx = np.empty(n, np.int32)
        sim = np.empty(n, np.float64)
        hit = np.empty(n, np.uint8)
        second = np.empty(n, np.float64) if want_second else None
        rc = lib().oracle_lookup(self._h, _ptr(qs), n, float(threshold), _ptr(idx), _ptr(sim), _ptr(hit),
                                 _ptr(second))
        if rc != 0:
            raise RuntimeError(f"oracle_lookup failed ({rc})")
        return idx, sim, hit, second

    def lookup_multi(self, queries: np.ndarray, thetas, count_index: int = -1):
        """One lookup against several thresholds: ``(idx, sim, hit uint8 [n, m], second)``."""
        qs = _storage(queries, self.dtype, self.dim)
        th = np.ascontiguousarray(thetas, dtype=np.float32)
        n, m = qs.shape[0], th.shape[0]
        idx = np.empty(n, np.int32)
        sim = np.empty(n, np.float64)
        hit = np.zeros((n, m), np.uint8)
        second = np.empty(n, np.float64)
        rc = lib().oracle_lookup_multi(self._h, _ptr(qs), n, _ptr(th), m, int(count_index), _ptr(idx), _ptr(sim),
                                       _ptr(hit), _ptr(second))
        if rc != 0:
            raise RuntimeError(f"oracle_lookup_multi failed ({rc})")
        return idx, sim, hit, second

    def lookup_topk(self, queries: np.ndarray, k: int):
        """The k closest centroids per query: ``(idx int32 [n, k], sim float64 [n, k])``."""
        qs = _storage(queries, self.dtype, self.dim)
        n = qs.shape[0]
        idx = np.empty((n, int(k)), np.int32)
        sim = np.empty((n, int(k)), np.float64)
        rc = lib().oracle_lookup_topk(self._h, _ptr(qs), n, int(k), _ptr(idx), _ptr(sim))
        if rc != 0:
            raise RuntimeError(f"oracle_lookup_topk failed ({rc})")
        return idx, sim

    def update(self, queries: np.ndarray, idx: np.ndarray) -> None:
        qs = _storage(queries, self.dtype, self.dim)
        ix = np.ascontiguousarray(idx, dtype=np.int32)
        if ix.shape != (qs.shape[0],):
            raise ValueError("idx must have one entry per query")
        rc = lib().oracle_update(self._h, _ptr(qs), _ptr(ix), qs.shape[0])
        if rc != 0:
            raise RuntimeError(f"oracle_update failed ({rc})")

    def merge(self, threshold: float, cap: Optional[int] = None) -> Tuple[np.ndarray, int]:
        """Returns ``(pairs[min(total, cap), 2] int32 in lexicographic order, total)``."""
        if cap is None:
            total = int(lib().oracle_merge(self._h, float(threshold), None, 0))
            if total < 0:
                raise RuntimeError(f"oracle_merge failed ({total})")
            cap = total
        pairs = np.empty((max(cap, 1), 2), np.int32)
        total = int(lib().oracle_merge(self._h, float(threshold), _ptr(pairs), cap))
        if total < 0:
            raise RuntimeError(f"oracle_merge failed ({total})")
        return pairs[:min(total, cap)].copy(), total

    def merge_apply(self, pairs: np.ndarray) -> np.ndarray:
        """Merges connected groups; returns the survivor map (new index of each old row)."""
        pr = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
        surv = np.empty(self.count, np.int32)
        rc = lib().oracle_merge_apply(self._h, _ptr(pr), pr.shape[0], _ptr(surv))
        if rc != 0:
            raise RuntimeError(f"oracle_merge_apply failed ({rc})")
        return surv

    def export(self):
        """Returns ``(centroids storage, means float64, sizes int32)`` of the live rows."""
        k = self.count
        cents = np.empty((k, self.dim), np.float32 if self.dtype == "f32" else np.uint16)
        means = np.empty((k, self.dim), np.float64)
        sizes = np.empty(k, np.int32)
        rc = lib().oracle_export(self._h, _ptr(cents), _ptr(means), _ptr(sizes))
        if rc != 0:
            raise RuntimeError(f"oracle_export failed ({rc})")
        return cents, means, sizes

"""Thin binding over the C-ABI library ``libsiso.so`` (declared in ``include/siso.h``; the tuning and
timing calls in ``include/siso_bench.h``).

Argument marshalling only: every step of the hot path runs in the library's HIP
kernels.  PyTorch supplies device memory (``tensor.data_ptr()``) and the stream.
There is no CPU fallback: importing this module without a built library raises.
"""

from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsiso.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_2508_18736_amd.build` "
        "(there is no fallback path)")

_lib = C.CDLL(LIB_PATH)

F32, BF16, FP8 = 0, 1, 2
PATH_AUTO, PATH_SCALAR, PATH_MFMA, PATH_SKINNY = 0, 1, 2, 3
OK, EINVAL, ECAPACITY, EHIP, ENOMEM = 0, -1, -2, -3, -4

# every symbol the headers under include/ declare, with its signature
_vp, _lg, _it, _fl = C.c_void_p, C.c_long, C.c_int, C.c_float
SYMBOLS = {
    "siso_create": ([_it, _lg, C.POINTER(_vp)], _it),
    "siso_create_ex": ([_it, _lg, _it, C.POINTER(_vp)], _it),
    "siso_destroy": ([_vp], None),
    "siso_set_stream": ([_vp, _vp], _it),
    "siso_set_lookup_path": ([_vp, _it], _it),
    "siso_set_option": ([_vp, C.c_char_p, _lg], _it),
    "siso_load": ([_vp, _vp, _vp, _lg], _it),
    "siso_count": ([_vp], _lg),
    "siso_reserve": ([_vp, _lg], _it),
    "siso_lookup": ([_vp, _vp, _lg, _fl, _vp, _vp, _vp], _it),
    "siso_lookup_update": ([_vp, _vp, _lg, _fl, _vp, _vp, _vp], _it),
    "siso_lookup_multi": ([_vp, _vp, _lg, _vp, _it, _it, _vp, _vp, _vp], _it),
    "siso_lookup_topk": ([_vp, _vp, _lg, _it, _vp, _vp], _it),
    "siso_lookup_static": ([_vp, _vp, _lg, _fl, _vp, _vp, _vp], _it),
    "siso_update": ([_vp, _vp, _vp, _lg], _it),
    "siso_update_hits": ([_vp, _vp, _vp, _vp, _lg], _it),
    "siso_bad_indices": ([_vp], _lg),
    "siso_merge": ([_vp, _fl, _vp, _lg], _lg),
    "siso_merge_apply": ([_vp, _vp, _lg, _vp], _it),
    "siso_export": ([_vp, _vp, _vp, _vp], _it),
    "siso_profile_enable": ([_vp, _it], _it),
    "siso_profile_read": ([_vp, C.POINTER(C.c_double), C.POINTER(C.c_long)], _it),
    "siso_last_error": ([_vp], C.c_char_p),
    "siso_probe": ([_it, C.POINTER(C.c_double)], _it),
    "siso_refresh": ([_vp, _vp, _vp, _lg, _fl, _lg, _vp], _it),
    "siso_cluster": ([_vp, _vp, _lg, _fl, _it, _vp, _vp, _vp], _lg),
    "siso_choose_communities": ([_vp, _lg, _lg, _it, _vp], _lg),
    "siso_refresh_plan": ([_lg, _vp, _vp, _lg, _vp, _vp, _vp, _vp, _vp, _lg, _fl, _lg, _vp, _vp, _vp], _lg),
    "siso_export_meta": ([_vp, _vp, _vp], _it),
    "siso_export_scales": ([_vp, _vp], _it),
    "siso_fp8_follow": ([_vp, _vp, _vp, _vp, _lg], _it),
    "siso_fp8_lookup_update": ([_vp, _vp, _vp, _lg, _fl, _vp, _vp, _vp], _it),
    "siso_fp8_hand_counts": ([_vp, _vp], _it),
    "siso_fp8_resync": ([_vp, _vp], _it),
    "siso_import": ([_vp, _vp, _vp, _vp, _vp, _vp, _lg], _it),
    "siso_t2h": ([_vp, _vp, _lg, _vp, _it, _vp], _it),
    "siso_md1_wait": ([C.c_double, C.c_double, C.c_double], C.c_double),
    "siso_pick_threshold": ([_vp, _vp, _it, C.c_double, C.c_double, C.c_double, C.POINTER(_it)], _it),
    "siso_adjust_threshold": ([_vp, _it, _it, C.c_double, C.c_double], _it),
}
for _name, (_args, _res) in SYMBOLS.items():
    _fn = getattr(_lib, _name)
    _fn.argtypes = _args
    _fn.restype = _res


def md1_wait(llm_time: float, arrival_rate: float, hit_ratio: float) -> float:
    return float(_lib.siso_md1_wait(float(llm_time), float(arrival_rate), float(hit_ratio)))


def choose_communities(pairs, n: int, min_size: int = 1):
    """The host part of the clustering: labels (numpy int32 [n]) and the number of clusters from the
    neighbour pairs (host array [P, 2])."""
    import numpy as np
    pr = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
    labels = np.full(int(n), -1, np.int32)
    rc = _lib.siso_choose_communities(pr.ctypes.data_as(_vp), pr.shape[0], int(n), int(min_size),
                                      labels.ctypes.data_as(_vp))
    if rc < 0:
        raise SisoError(int(rc), "siso_choose_communities: bad pairs or sizes")
    return labels, int(rc)


def refresh_plan(cluster_size, access_count, repo_size, best_idx, best_sim, pairs, pair_cosine, theta_c: float,
                 max_centroids: int):
    """The host part of a refresh (host arrays in, host arrays out):
    ``(source int32 [survivors], cluster_size float32 [survivors], (merged, added, evicted))``."""
    import numpy as np
    cs = np.ascontiguousarray(cluster_size, dtype=np.float32)
    ac = np.ascontiguousarray(access_count, dtype=np.uint32)
    rs = np.ascontiguousarray(repo_size, dtype=np.float32)
    bi = np.ascontiguousarray(best_idx, dtype=np.int32)
    bs = np.ascontiguousarray(best_sim, dtype=np.float32)
    pr = np.ascontiguousarray(pairs, dtype=np.int32).reshape(-1, 2)
    pc = np.ascontiguousarray(pair_cosine, dtype=np.float32)
    k0, r = cs.shape[0], rs.shape[0]
    assert ac.shape == (k0,) and bi.shape == (r,) and bs.shape == (r,) and pc.shape == (pr.shape[0],)
    src = np.empty(k0 + r, np.int32)
    out = np.empty(k0 + r, np.float32)
    stats = (C.c_long * 3)()
    p = lambda a: a.ctypes.data_as(_vp)
    rc = _lib.siso_refresh_plan(k0, p(cs), p(ac), r, p(rs), p(bi), p(bs), p(pr), p(pc), pr.shape[0], float(theta_c),
                                int(max_centroids), p(src), p(out), stats)
    if rc < 0:
        raise SisoError(int(rc), "siso_refresh_plan: bad arguments")
    return src[:rc].copy(), out[:rc].copy(), (int(stats[0]), int(stats[1]), int(stats[2]))


def pick_threshold(thetas, hit_ratio, llm_time: float, arrival_rate: float, slo: float) -> int:
    """Position of the highest threshold of the table that meets the SLO, -1 if none."""
    import numpy as np
    th = np.ascontiguousarray(thetas, dtype=np.float32)
    hr = np.ascontiguousarray(hit_ratio, dtype=np.float64)
    if th.ndim != 1 or th.shape != hr.shape:
        raise ValueError("thetas and hit_ratio: one-dimensional arrays of the same length")
    out = _it(-1)
    rc = _lib.siso_pick_threshold(th.ctypes.data_as(_vp), hr.ctypes.data_as(_vp), th.shape[0], float(llm_time),
                                  float(arrival_rate), float(slo), C.byref(out))
    if rc != OK:
        raise SisoError(rc, "siso_pick_threshold failed")
    return int(out.value)


def adjust_threshold(thetas, index: int, wait_estimated: float, wait_measured: float) -> int:
    import numpy as np
    th = np.ascontiguousarray(thetas, dtype=np.float32)
    return int(_lib.siso_adjust_threshold(th.ctypes.data_as(_vp), th.shape[0], int(index), float(wait_estimated),
                                          float(wait_measured)))


def probe(which: int) -> float:
    """What the chip delivers: 0 = bf16 MFMA loop, random operands (TFLOP/s); 1 = the same with constant
    operands; 2 = streaming read from HBM (GB/s).  Runs on the current device's null stream."""
    v = C.c_double(0.0)
    rc = _lib.siso_probe(int(which), C.byref(v))
    if rc != OK:
        raise SisoError(rc, "siso_probe failed")
    return float(v.value)


def to_dev(arr, dtype: str, device: str = "cuda:0") -> torch.Tensor:
    """Host rows (numpy; bf16 as uint16 bit patterns, as the workload generators carry them) -> device tensor."""
    import numpy as np
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(device)


def to_host(t: torch.Tensor, dtype: str):
    """Device tensor -> host rows (numpy; bf16 as uint16 bit patterns)."""
    import numpy as np
    t = t.detach().cpu().contiguous()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


class SisoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"siso error {code}: {msg}")
        self.code = code


_TORCH_DT = {F32: torch.float32, BF16: torch.bfloat16, FP8: torch.bfloat16}  # what the rows handed in are made of


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


class SisoCache:
    """Device-resident centroid cache.  Method names follow the C ABI."""

    def __init__(self, dim: int, capacity: int, dtype: int = BF16, device: str = "cuda:0"):
        self.dim, self.capacity, self.dtype = int(dim), int(capacity), int(dtype)
        self.device = torch.device(device)
        self._h = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = _lib.siso_create_ex(self.dim, self.capacity, self.dtype, C.byref(self._h))
        if rc != OK:
            self._h = C.c_void_p()
            raise SisoError(rc, "siso_create_ex failed")
        self.set_stream(torch.cuda.current_stream(self.device))

    # ------------------------------------------------------------------ plumbing
    def _check(self, rc: int) -> int:
        if rc < 0:
            raise SisoError(rc, _lib.siso_last_error(self._h).decode())
        return rc

    def _rows(self, t: torch.Tensor, what: str) -> torch.Tensor:
        if t.device != self.device or t.dtype != _TORCH_DT[self.dtype] or t.dim() != 2 or t.shape[1] != self.dim:
            raise ValueError(f"{what}: expected a [*, {self.dim}] {_TORCH_DT[self.dtype]} tensor on {self.device}")
        return t if t.is_contiguous() else t.contiguous()

    def _vec(self, t: Optional[torch.Tensor], dtype: torch.dtype, n: int, what: str) -> Optional[torch.Tensor]:
        if t is None:
            return None
        if t.device != self.device or t.dtype != dtype or t.shape != (n,) or not t.is_contiguous():
            raise ValueError(f"{what}: expected a contiguous [{n}] {dtype} tensor on {self.device}")
        return t

    def close(self) -> None:
        if getattr(self, "_h", None):
            _lib.siso_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_stream(self, stream: torch.cuda.Stream) -> None:
        self._stream = stream
        self._check(_lib.siso_set_stream(self._h, C.c_void_p(stream.cuda_stream)))

    def set_lookup_path(self, path: int) -> None:
        self._check(_lib.siso_set_lookup_path(self._h, int(path)))

    def set_option(self, name: str, value: int) -> None:
        self._check(_lib.siso_set_option(self._h, name.encode(), int(value)))

    def reserve(self, n: int) -> None:
        """Room for lookups and updates of up to ``n`` queries, so that those calls never allocate."""
        self._check(_lib.siso_reserve(self._h, int(n)))

    @property
    def count(self) -> int:
        return int(_lib.siso_count(self._h))

    # ---------------------------------------------------------------------- calls
    def load(self, centroids: torch.Tensor, counts: Optional[torch.Tensor] = None) -> None:
        cents = self._rows(centroids, "centroids")
        cn = self._vec(counts, torch.int32, cents.shape[0], "counts")
        self._check(_lib.siso_load(self._h, _ptr(cents), _ptr(cn), cents.shape[0]))

    def lookup(self, queries: torch.Tensor, threshold: float, out_idx: Optional[torch.Tensor] = None,
               out_sim: Optional[torch.Tensor] = None, out_hit: Optional[torch.Tensor] = None
               ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        q = self._rows(queries, "queries")
        n = q.shape[0]
        if out_idx is None:
            out_idx = torch.empty(n, dtype=torch.int32, device=self.device)
        if out_sim is None:
            out_sim = torch.empty(n, dtype=torch.float32, device=self.device)
        if out_hit is None:
            out_hit = torch.empty(n, dtype=torch.uint8, device=self.device)
        self._vec(out_idx, torch.int32, n, "out_idx")
        self._vec(out_sim, torch.float32, n, "out_sim")
        self._vec(out_hit, torch.uint8, n, "out_hit")
        self._check(_lib.siso_lookup(self._h, _ptr(q), n, float(threshold), _ptr(out_idx), _ptr(out_sim),
                                     _ptr(out_hit)))
        return out_idx, out_sim, out_hit

    def lookup_update(self, queries: torch.Tensor, threshold: float, out_idx: Optional[torch.Tensor] = None,
                      out_sim: Optional[torch.Tensor] = None, out_hit: Optional[torch.Tensor] = None
                      ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        """``lookup`` and ``update(queries, idx, hit)`` with its outputs, as one call."""
        q = self._rows(queries, "queries")
        n = q.shape[0]
        if out_idx is None:
            out_idx = torch.empty(n, dtype=torch.int32, device=self.device)
        if out_sim is None:
            out_sim = torch.empty(n, dtype=torch.float32, device=self.device)
        if out_hit is None:
            out_hit = torch.empty(n, dtype=torch.uint8, device=self.device)
        self._vec(out_idx, torch.int32, n, "out_idx")
        self._vec(out_sim, torch.float32, n, "out_sim")
        self._vec(out_hit, torch.uint8, n, "out_hit")
        self._check(_lib.siso_lookup_update(self._h, _ptr(q), n, float(threshold), _ptr(out_idx), _ptr(out_sim),
                                            _ptr(out_hit)))
        return out_idx, out_sim, out_hit

    def lookup_multi(self, queries: torch.Tensor, thetas, count_index: int = -1
                     ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        """One lookup against several thresholds (host values): ``(idx [n], sim [n], hit uint8 [n, m])``."""
        import numpy as np
        q = self._rows(queries, "queries")
        n = q.shape[0]
        th = np.ascontiguousarray(thetas, dtype=np.float32)
        idx = torch.empty(n, dtype=torch.int32, device=self.device)
        sim = torch.empty(n, dtype=torch.float32, device=self.device)
        hit = torch.empty((n, th.shape[0]), dtype=torch.uint8, device=self.device)
        self._check(_lib.siso_lookup_multi(self._h, _ptr(q), n, th.ctypes.data_as(_vp), th.shape[0], int(count_index),
                                           _ptr(idx), _ptr(sim), _ptr(hit)))
        return idx, sim, hit

    def lookup_topk(self, queries: torch.Tensor, k: int) -> Tuple[torch.Tensor, torch.Tensor]:
        """The k closest centroids per query: ``(idx int32 [n, k], sim float32 [n, k])``."""
        q = self._rows(queries, "queries")
        n = q.shape[0]
        idx = torch.empty((n, max(int(k), 1)), dtype=torch.int32, device=self.device)
        sim = torch.empty((n, max(int(k), 1)), dtype=torch.float32, device=self.device)
        self._check(_lib.siso_lookup_topk(self._h, _ptr(q), n, int(k), _ptr(idx), _ptr(sim)))
        return idx, sim

    def lookup_static(self, queries: torch.Tensor, threshold: float, out_idx: torch.Tensor, out_sim: torch.Tensor,
                      out_hit: Optional[torch.Tensor] = None) -> None:
        """``siso_lookup_static``: the lookup that allocates nothing; the caller brings every output."""
        q = self._rows(queries, "queries")
        if q.data_ptr() != queries.data_ptr():
            raise ValueError("queries: must be contiguous (this call does not copy)")
        n = q.shape[0]
        self._vec(out_idx, torch.int32, n, "out_idx")
        self._vec(out_sim, torch.float32, n, "out_sim")
        self._vec(out_hit, torch.uint8, n, "out_hit")
        self._check(_lib.siso_lookup_static(self._h, _ptr(q), n, float(threshold), _ptr(out_idx), _ptr(out_sim),
                                            _ptr(out_hit)))

    def update(self, queries: torch.Tensor, idx: torch.Tensor, hit: Optional[torch.Tensor] = None) -> None:
        q = self._rows(queries, "queries")
        n = q.shape[0]
        self._vec(idx, torch.int32, n, "idx")
        if hit is None:
            self._check(_lib.siso_update(self._h, _ptr(q), _ptr(idx), n))
        else:
            self._vec(hit, torch.uint8, n, "hit")
            self._check(_lib.siso_update_hits(self._h, _ptr(q), _ptr(idx), _ptr(hit), n))

    def bad_indices(self) -> int:
        return self._check(_lib.siso_bad_indices(self._h))

    def merge(self, threshold: float, cap: int) -> Tuple[torch.Tensor, int]:
        """Returns ``(pairs[min(total, cap), 2] int32 on the device, total)``."""
        pairs = torch.empty((max(int(cap), 1), 2), dtype=torch.int32, device=self.device)
        total = self._check(_lib.siso_merge(self._h, float(threshold), _ptr(pairs), int(cap)))
        return pairs[:min(total, int(cap))], total

    def merge_apply(self, pairs: torch.Tensor) -> torch.Tensor:
        """Merges the connected groups; returns the survivor map (int32, old count)."""
        if pairs.device != self.device or pairs.dtype != torch.int32 or pairs.dim() != 2 or pairs.shape[1] != 2:
            raise ValueError("pairs: expected a [*, 2] int32 tensor on the cache's device")
        pr = pairs.contiguous()
        surv = torch.empty(self.count, dtype=torch.int32, device=self.device)
        self._check(_lib.siso_merge_apply(self._h, _ptr(pr), pr.shape[0], _ptr(surv)))
        return surv

    def refresh(self, repo: torch.Tensor, repo_size: torch.Tensor, theta_c: float, max_centroids: int):
        """Algorithm 1 (merge, filtering, update).  Returns ``(merged, added, evicted)``."""
        rows = self._rows(repo, "repo")
        sizes = self._vec(repo_size, torch.float32, rows.shape[0], "repo_size")
        stats = (C.c_long * 3)()
        self._check(_lib.siso_refresh(self._h, _ptr(rows), _ptr(sizes), rows.shape[0], float(theta_c),
                                      int(max_centroids), stats))
        return int(stats[0]), int(stats[1]), int(stats[2])

    def cluster(self, vectors: torch.Tensor, theta_c: float, min_size: int = 1, representatives: bool = False):
        """Community detection over the vectors; this cache becomes the repository of the clusters.
        Returns ``(labels int32 [n] on the device, number of clusters, pairs above the threshold)``; with
        ``representatives`` also the member closest to each centroid (int32 [clusters] on the device)."""
        rows = self._rows(vectors, "vectors")
        labels = torch.empty(rows.shape[0], dtype=torch.int32, device=self.device)
        rep = torch.empty(min(rows.shape[0], self.capacity), dtype=torch.int32, device=self.device) if representatives else None
        stats = (C.c_long * 2)()
        rc = _lib.siso_cluster(self._h, _ptr(rows), rows.shape[0], float(theta_c), int(min_size), _ptr(labels),
                               _ptr(rep) if representatives else None, stats)
        if rc < 0:
            self._check(int(rc))
        if representatives:
            return labels, int(rc), int(stats[0]), rep[:int(rc)]
        return labels, int(rc), int(stats[0])

    def export_meta(self) -> Tuple[torch.Tensor, torch.Tensor]:
        """``(cluster_size float32, access_count int64)`` of the live centroids; infinity = 0xFFFFFFFF."""
        k = self.count
        loc = torch.empty(k, dtype=torch.float32, device=self.device)
        acc = torch.empty(k, dtype=torch.int32, device=self.device)
        self._check(_lib.siso_export_meta(self._h, _ptr(loc), _ptr(acc)))
        return loc, acc.to(torch.int64) & 0xFFFFFFFF

    def import_state(self, centroids: torch.Tensor, means: torch.Tensor, counts: torch.Tensor,
                     cluster_size: Optional[torch.Tensor] = None, access_count: Optional[torch.Tensor] = None) -> None:
        """Take over a snapshot (what ``export`` and ``export_meta`` returned) as it is.  ``access_count`` may be
        the int64 tensor ``export_meta`` returns (0xFFFFFFFF = infinity)."""
        cents = self._rows(centroids, "centroids")
        k = cents.shape[0]
        if means.device != self.device or means.dtype != torch.float32 or means.shape != cents.shape:
            raise ValueError("means: expected a float32 tensor of the centroids' shape on the cache's device")
        mm = means.contiguous()
        cn = self._vec(counts, torch.int32, k, "counts")
        loc = self._vec(cluster_size, torch.float32, k, "cluster_size")
        acc = None
        if access_count is not None:
            # the low 32 bits as they are (0xFFFFFFFF stays 0xFFFFFFFF)
            acc = (access_count.to(torch.int64) & 0xFFFFFFFF).to(torch.uint32).view(torch.int32).contiguous()
            self._vec(acc, torch.int32, k, "access_count")
        self._check(_lib.siso_import(self._h, _ptr(cents), _ptr(mm), _ptr(cn), _ptr(loc), _ptr(acc), k))

    def t2h(self, queries: torch.Tensor, thetas):
        """Hits per threshold (numpy int64) of the sample queries; thresholds are host values."""
        import numpy as np
        q = self._rows(queries, "queries")
        th = np.ascontiguousarray(thetas, dtype=np.float32)
        hits = np.zeros(th.shape[0], dtype=np.int64)
        self._check(_lib.siso_t2h(self._h, _ptr(q), q.shape[0], th.ctypes.data_as(_vp), th.shape[0],
                                  hits.ctypes.data_as(_vp)))
        return hits

    def profile_enable(self, on) -> None:
        """0/False = off; N = bracket the dominant kernel of every N-th call with events."""
        self._check(_lib.siso_profile_enable(self._h, int(on)))

    def profile_read(self) -> Tuple[float, int]:
        """Sum of the bracketed kernel durations (ms) and their number since the last read."""
        ms, cnt = C.c_double(0.0), C.c_long(0)
        self._check(_lib.siso_profile_read(self._h, C.byref(ms), C.byref(cnt)))
        return float(ms.value), int(cnt.value)

    def follow(self, master: "SisoCache", idx: torch.Tensor, hit: Optional[torch.Tensor] = None) -> None:
        """8-bit serving copy: quantise the centroids ``idx`` (where ``hit``) again from the bf16 ``master``."""
        n = idx.shape[0]
        self._vec(idx, torch.int32, n, "idx")
        if hit is not None:
            self._vec(hit, torch.uint8, n, "hit")
        self._check(_lib.siso_fp8_follow(self._h, master._h, _ptr(idx), _ptr(hit) if hit is not None else None, n))

    def hand_counts(self, master: "SisoCache") -> None:
        """8-bit serving copy: the references its lookups counted go to the ``master``'s access counts."""
        self._check(_lib.siso_fp8_hand_counts(self._h, master._h))

    def resync(self, master: "SisoCache") -> None:
        """8-bit serving copy: become the image of the ``master`` as it stands (after its merge or refresh)."""
        self._check(_lib.siso_fp8_resync(self._h, master._h))

    def lookup_update_with(self, master: "SisoCache", queries: torch.Tensor, threshold: float,
                           out_idx: Optional[torch.Tensor] = None, out_sim: Optional[torch.Tensor] = None,
                           out_hit: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        """8-bit serving copy: ``lookup`` here, ``update`` of the hits on the bf16 ``master``, ``follow``: one call."""
        q = master._rows(queries, "queries")
        n = q.shape[0]
        if out_idx is None:
            out_idx = torch.empty(n, dtype=torch.int32, device=self.device)
        if out_sim is None:
            out_sim = torch.empty(n, dtype=torch.float32, device=self.device)
        if out_hit is None:
            out_hit = torch.empty(n, dtype=torch.uint8, device=self.device)
        self._vec(out_idx, torch.int32, n, "out_idx")
        self._vec(out_sim, torch.float32, n, "out_sim")
        self._vec(out_hit, torch.uint8, n, "out_hit")
        self._check(_lib.siso_fp8_lookup_update(self._h, master._h, _ptr(q), n, float(threshold), _ptr(out_idx), _ptr(out_sim),
                                                _ptr(out_hit)))
        return out_idx, out_sim, out_hit

    def export_fp8(self) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        """8-bit caches: ``(codes uint8 [count, dim], scales float32 [count], sizes int32 [count])``."""
        k = self.count
        codes = torch.empty((k, self.dim), dtype=torch.uint8, device=self.device)
        scales = torch.empty(k, dtype=torch.float32, device=self.device)
        sizes = torch.empty(k, dtype=torch.int32, device=self.device)
        self._check(_lib.siso_export(self._h, _ptr(codes), None, _ptr(sizes)))
        self._check(_lib.siso_export_scales(self._h, _ptr(scales)))
        return codes, scales, sizes

    def export(self) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
        k = self.count
        cents = torch.empty((k, self.dim), dtype=_TORCH_DT[self.dtype], device=self.device)
        means = torch.empty((k, self.dim), dtype=torch.float32, device=self.device)
        sizes = torch.empty(k, dtype=torch.int32, device=self.device)
        self._check(_lib.siso_export(self._h, _ptr(cents), _ptr(means), _ptr(sizes)))
        return cents, means, sizes

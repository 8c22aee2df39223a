"""Pins for the oracle's 8-bit storage variant.  CPU only.  Codes worked by hand from the definition of the
format; an independent decode table written here from the same definition; the cosine of the stored vectors
through numpy float64; invariants of the blocked scaling."""

import os

import numpy as np
import pytest

from paper_2508_18736_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fp8_e4m3_hand_worked.txt")


def f32(x):
    return np.ascontiguousarray(x, dtype=np.float32)


def decode_table():
    """All 256 codes from the definition: sign, exponent field e, mantissa m."""
    t = np.zeros(256, np.float64)
    for code in range(256):
        s, e, m = code >> 7, (code >> 3) & 15, code & 7
        if e == 15 and m == 7:
            v = np.nan
        elif e == 0:
            v = m / 8.0 * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[code] = -v if s else v
    return t


def read_golden():
    out = []
    for line in open(GOLDEN):
        t = line.split("#")[0].split()
        if len(t) == 2:
            out.append((float(t[0]), int(t[1], 16)))
    return out


def test_codes_worked_by_hand(oracle):
    cases = read_golden()
    assert len(cases) >= 20
    rows = f32([[448.0, v] for v, _ in cases])
    codes, scales = oracle.fp8_quantize(rows, "f32")
    assert np.all(scales == 1.0) and np.all(codes[:, 0] == 0x7E)
    for (v, want), got in zip(cases, codes[:, 1]):
        assert got == want, f"{v} -> {got:#04x}, expected {want:#04x}"
    # the table itself: 448 is the largest value, the values ascend with the codes, every value encodes to itself
    tab = decode_table()
    assert tab[0x7E] == 448.0 and tab[0x38] == 1.0 and tab[0x01] == 2.0 ** -9 and np.isnan(tab[0x7F])
    assert np.all(np.diff(tab[:0x7F]) > 0)
    rows = f32([[448.0, tab[c]] for c in range(0x7F)] + [[448.0, -tab[c]] for c in range(1, 0x7F)])
    codes, _ = oracle.fp8_quantize(rows, "f32")
    assert codes[:0x7F, 1].tolist() == list(range(0x7F)) and codes[0x7F:, 1].tolist() == [c | 0x80 for c in range(1, 0x7F)]


def test_rounding_is_to_the_nearest_value_everywhere(oracle):
    """Brute force: 20,000 values against the nearest entry of the decode table (ties excluded: they are in the
    hand-worked list)."""
    tab = decode_table()[:0x7F]
    r = np.random.default_rng(3)
    v = np.concatenate([r.uniform(0, 448, 8000), r.uniform(0, 2, 8000), 2.0 ** r.uniform(-12, 9, 4000)]).astype(np.float32)
    v = np.minimum(v, np.float32(448))
    codes, scales = oracle.fp8_quantize(f32(np.stack([np.full_like(v, 448.0), v], 1)), "f32")
    err = np.abs(tab[None, :] - v.astype(np.float64)[:, None])
    nearest = err.argmin(axis=1)
    two = np.sort(err, axis=1)[:, :2]
    clear = two[:, 1] - two[:, 0] > 0
    assert clear.mean() > 0.999 and np.array_equal(codes[clear, 1], nearest[clear])


def test_scale_is_the_largest_element_over_448_and_scaling_a_row_changes_only_the_scale(oracle):
    wl = W.c2_mid(n_clusters=4, per_cluster=8, n_queries=4, dim=64, dtype="bf16", seed=401)
    codes, scales = oracle.fp8_quantize(wl.centroids, "bf16")
    x = wl.centroids_f32()
    assert np.array_equal(scales, np.abs(x).max(axis=1) / np.float32(448.0))
    assert np.all(np.abs(decode_table()[codes]).max(axis=1) == 448.0)      # the largest element maps to +-448
    codes2, scales2 = oracle.fp8_quantize(W.f32_to_bf16_bits(x * np.float32(8.0)), "bf16")   # a power of two: exact
    assert np.array_equal(codes2, codes) and np.array_equal(scales2, scales * np.float32(8.0))
    # the stored row is close to the row: relative step 2^-4 per element at worst (3 mantissa bits), much less in length
    back = decode_table()[codes] * scales[:, None].astype(np.float64)
    assert np.abs(back - x).max() <= np.abs(x).max() * 2.0 ** -4
    cos = np.einsum("ij,ij->i", back, x) / np.linalg.norm(back, axis=1) / np.linalg.norm(x.astype(np.float64), axis=1)
    assert cos.min() > 0.999
    # degenerate rows
    z = np.zeros((3, 8), np.float32)
    z[1, 2] = np.nan
    z[2, 5] = np.inf
    c, s = oracle.fp8_quantize(z, "f32")
    assert s[0] == 0.0 and np.isnan(s[1]) and np.isnan(s[2]) and not c.any()


@pytest.mark.parametrize("dim,K,n", [(64, 300, 40), (128, 1000, 25)])
def test_fp8_lookup_is_the_cosine_of_the_stored_vectors(oracle, dim, K, n):
    wl = W.c2_mid(n_clusters=16, per_cluster=(K + 15) // 16, n_queries=n, dim=dim, dtype="bf16", sigma=0.4, seed=402)
    wl.centroids = wl.centroids[:K].copy()
    wl.centroids[7] = wl.centroids[3]           # an exact duplicate: the lower index wins
    cc, cs = oracle.fp8_quantize(wl.centroids, "bf16")
    idx, sim, hit, second = oracle.fp8_lookup_rows(cc, cs, wl.queries, 0.8)
    tab = decode_table()
    qc, qs = oracle.fp8_quantize(wl.queries, "bf16")
    C = tab[cc] * cs[:, None].astype(np.float64)      # the stored vectors, scales included
    Q = tab[qc] * qs[:, None].astype(np.float64)
    S = (Q / np.linalg.norm(Q, axis=1, keepdims=True)) @ (C / np.linalg.norm(C, axis=1, keepdims=True)).T
    assert np.abs(S.max(axis=1) - sim).max() < 1e-12
    gap = np.sort(S, axis=1)[:, -1] - np.sort(S, axis=1)[:, -2]
    clear = gap > 1e-9
    assert np.array_equal(idx[clear], S.argmax(axis=1)[clear])
    assert np.array_equal(hit, (sim > np.float64(np.float32(0.8))).astype(np.uint8)) and 0 < hit.sum() < n
    assert not (idx == 7).any()
    # close to, but not the same as, the lookup at the input precision: the error of the 8-bit storage
    ref = oracle.lookup_rows(wl.centroids, wl.queries, 0.8, "bf16")
    assert np.abs(ref[1] - sim).max() < 0.02 and (ref[0] == idx).mean() > 0.7


def test_fp8_lookup_degenerate_rows(oracle):
    dim = 16
    c = np.zeros((4, dim), np.float32)
    c[0, 0] = 1.0
    c[1, 1] = 3.0
    c[2, :] = 0.0              # no length: similarity 0
    c[3, 0] = np.nan           # never chosen
    cc, cs = oracle.fp8_quantize(c, "f32")
    q = np.zeros((4, dim), np.float32)
    q[0, 1] = 5.0              # equals centroid 1 in direction
    q[1, :] = 0.0              # no length: similarity 0 to everything, index 0
    q[2, 3] = np.inf
    q[3, 0] = -2.0             # opposite to centroid 0: best is a similarity of 0 (centroid 1 or 2: the lower index)
    idx, sim, hit, second = oracle.fp8_lookup_rows(cc, cs, q, 0.5, "f32")
    assert idx.tolist() == [1, 0, -1, 1] and sim[0] == 1.0 and sim[1] == 0.0 and np.isnan(sim[2]) and sim[3] == 0.0
    assert hit.tolist() == [1, 0, 0, 0]
    idx, sim, hit, second = oracle.fp8_lookup_rows(cc[:0], cs[:0], q, 0.5, "f32")
    assert (idx[[0, 1, 3]] == -1).all() and np.isneginf(sim[[0, 1, 3]]).all()


@pytest.mark.parametrize("dim,K,n,k", [(64, 300, 30, 5), (128, 700, 12, 9)])
def test_fp8_topk_is_the_ranking_of_the_cosines_of_the_stored_vectors(oracle, dim, K, n, k):
    """numpy route: decode table from the format's definition, cosines in float64, a stable sort (equal cosines keep
    their index order); planted exact duplicates must come out in index order."""
    wl = W.c2_mid(n_clusters=16, per_cluster=(K + 15) // 16, n_queries=n, dim=dim, dtype="bf16", sigma=0.4, seed=404)
    wl.centroids = wl.centroids[:K].copy()
    wl.centroids[211] = wl.centroids[5]
    wl.centroids[90] = wl.centroids[5]
    wl.queries[0] = wl.centroids[5]              # its three copies tie at the top: 5, 90, 211
    cc, cs = oracle.fp8_quantize(wl.centroids, "bf16")
    idx, sim = oracle.fp8_lookup_topk_rows(cc, cs, wl.queries, k)
    assert idx.shape == (n, k) and idx[0, :3].tolist() == [5, 90, 211] and np.all(sim[0, :3] == sim[0, 0])
    tab = decode_table()
    qc, _ = oracle.fp8_quantize(wl.queries, "bf16")
    C, Q = tab[cc], tab[qc]
    S = (Q / np.linalg.norm(Q, axis=1, keepdims=True)) @ (C / np.linalg.norm(C, axis=1, keepdims=True)).T
    order = np.argsort(-S, axis=1, kind="stable")[:, :k]
    top = np.take_along_axis(S, order, axis=1)
    assert np.abs(top - sim).max() < 1e-12
    clear = np.abs(np.diff(np.take_along_axis(S, np.argsort(-S, axis=1, kind="stable")[:, :k + 1], axis=1), axis=1)).min(axis=1) > 1e-9
    assert clear.sum() >= n // 2 and np.array_equal(idx[clear], order[clear])
    assert np.all(np.diff(sim, axis=1) <= 0)
    # k = 1 is the lookup
    one_idx, one_sim = oracle.fp8_lookup_topk_rows(cc, cs, wl.queries, 1)
    ref = oracle.fp8_lookup_rows(cc, cs, wl.queries, 0.5)
    assert np.array_equal(one_idx[:, 0], ref[0]) and np.array_equal(one_sim[:, 0], ref[1])


def test_fp8_topk_degenerate_rows(oracle):
    dim = 16
    c = np.zeros((4, dim), np.float32)
    c[0, 0] = 1.0
    c[1, 1] = 3.0
    c[3, 0] = np.nan           # never chosen; row 2 has no length: similarity 0
    cc, cs = oracle.fp8_quantize(c, "f32")
    q = np.zeros((3, dim), np.float32)
    q[0, 1] = 5.0              # row 1, then the zeros of rows 0 and 2 in index order
    q[2, 3] = np.inf           # q[1] has no length: similarity 0 to every row that can be chosen
    idx, sim = oracle.fp8_lookup_topk_rows(cc, cs, q, 4, "f32")
    assert idx[0].tolist() == [1, 0, 2, -1] and sim[0, 0] == 1.0 and sim[0, 1] == 0.0 and np.isneginf(sim[0, 3])
    assert idx[1].tolist() == [0, 1, 2, -1] and np.all(sim[1, :3] == 0.0)
    assert (idx[2] == -1).all() and np.isnan(sim[2]).all()

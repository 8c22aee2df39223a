// The k closest centroids of every query (FindClosestCentroid of Algorithm 1 taken k times).
//
// Fast path (bf16 and 8-bit caches the MFMA kernels can serve, at least 512 * k centroids): two passes of the
// fused GEMM.  Pass 1 is the first phase of an ordinary lookup: per query and slice of the centroid
// range the largest scaled product <q, c> / |c|.  Slices hold different rows, so the k-th largest of
// those maxima is reached by at least k rows: a lower bound on the k-th best.  Pass 2 forms all products
// again and lists, per query, the rows that reach its bound - the k best are among them, and with many
// more slices than k there are rarely more than a few k of them.  The cosines of the listed rows are then
// recomputed (as the finalize step of a lookup does) and ranked: larger cosine first, lower index among
// equal cosines.  For an 8-bit cache the batch is quantised first, as in a lookup, and everything here sees codes
// and the inverse lengths of code rows.
// General path: every centroid row by row, one workgroup per query, each wave keeping its k best in its
// lanes.  It serves the other caches and, behind the fast path, the queries with more listed rows than the
// list holds (many exact duplicates at the bound, a query without length).
#include "siso_internal.h"

namespace {

// (value, index): larger value first, then the lower index; index -1 = no entry (worse than any entry)
__device__ __forceinline__ bool ranks_before(float va, int ia, float vb, int ib) {
    if (ia < 0) return false;
    if (ib < 0) return true;
    return va > vb || (va == vb && ia < ib);
}

// Pass 1 -> bound: tau[q] = value of the k-th largest key of query q (-inf with fewer than k keys: every
// row is wanted then).  One 256-thread block per query; the keys sit in LDS, k rounds of "largest left".
__global__ __launch_bounds__(256) void k_topk_bound(const u64 *__restrict__ keys, int slices, int k, float *tau, int *cnt,
                                                     int *scan) {
    extern __shared__ u64 sk[];  // [slices]
    __shared__ u64 wmax[4];
    __shared__ int wpos[4];
    const long q = blockIdx.x;
    const int t = threadIdx.x;
    for (int s = t; s < slices; s += 256) sk[s] = keys[(size_t)q * slices + s];
    __syncthreads();
    u64 kth = 0;
    for (int r = 0; r < k; ++r) {
        u64 best = 0;
        int pos = -1;
        for (int s = t; s < slices; s += 256)
            if (sk[s] > best) {
                best = sk[s];
                pos = s;
            }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const u64 ob = __shfl_xor(best, off);
            const int op = __shfl_xor(pos, off);
            if (ob > best) {  // keys of different slices differ (they name different rows)
                best = ob;
                pos = op;
            }
        }
        if ((t & 63) == 0) {
            wmax[t >> 6] = best;
            wpos[t >> 6] = pos;
        }
        __syncthreads();
        best = wmax[0];
        pos = wpos[0];
        for (int w = 1; w < 4; ++w)
            if (wmax[w] > best) {
                best = wmax[w];
                pos = wpos[w];
            }
        kth = best;
        __syncthreads();
        if (best == 0) break;  // fewer than k keys
        if (t == 0) sk[pos] = 0;
        __syncthreads();
    }
    if (t == 0) {
        tau[q] = kth == 0 ? -INFINITY : unordered_bits((unsigned)(kth >> 32));
        cnt[q] = 0;
        scan[q] = 0;
    }
}

// Listed rows -> result: exact cosines of the listed rows of query q (one wave per row), ranked; queries
// whose list overflowed are marked for the scan instead.  One 256-thread block per query.
template <typename T>
__global__ __launch_bounds__(256) void k_topk_select(const T *__restrict__ Q, const T *__restrict__ cent,
                                                      const float *__restrict__ invn, long K, int d, int k,
                                                      const int *__restrict__ cand, const int *__restrict__ cnt, int cap,
                                                      const float *__restrict__ q_inv, int *scan, int *out_idx,
                                                      float *out_sim) {
    constexpr int EPC = 16 / (int)sizeof(T);
    __shared__ float sh_f[4];
    __shared__ u32x4_t sh_q[SISO_MAX_DIM / EPC];
    __shared__ float val[SISO_TOPK_CAND];
    __shared__ int idx[SISO_TOPK_CAND];
    const long q = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const T *qrow = Q + (size_t)q * d;
    float ss = 0.f;
    for (int e = t * EPC; e < d; e += 256 * EPC) {
        const u32x4_t v = *(const u32x4_t *)(qrow + e);
        sh_q[e / EPC] = v;
        if (!q_inv) ss += chunk_dot(v, v, T());
    }
    ss = wave_sum(ss);
    if (lane == 0) sh_f[wave] = ss;
    __syncthreads();
    // (q_inv: the inverse lengths that came with the quantised batch)
    const float qi = q_inv ? q_inv[q] : inv_length((sh_f[0] + sh_f[1]) + (sh_f[2] + sh_f[3]));
    const int listed = cnt[q];
    if (!(qi == qi)) {  // a query holding a NaN or an infinity
        for (int r = t; r < k; r += 256) {
            out_idx[(size_t)q * k + r] = -1;
            out_sim[(size_t)q * k + r] = __uint_as_float(0x7FC00000u);
        }
        return;
    }
    if (listed > cap) {  // more rows at the bound than the list holds: the scan takes this query
        if (t == 0) scan[q] = 1;
        return;
    }
    for (int i = wave; i < listed; i += 4) {
        const int r = cand[(size_t)q * cap + i];
        const T *crow = cent + (size_t)r * d;
        float acc = 0.f;
        for (int e0 = lane * EPC; e0 < d; e0 += 64 * EPC) acc += chunk_dot(sh_q[e0 / EPC], *(const u32x4_t *)(crow + e0), T());
        acc = wave_sum(acc);
        const float sv = acc * qi * invn[r];
        if (lane == 0) {
            val[i] = sv;
            idx[i] = sv == sv ? r : -1;  // a NaN is never chosen
        }
    }
    __syncthreads();
    // rank by counting the entries that come before (all differ in their index)
    if (t < listed && idx[t] >= 0) {
        int before = 0;
        for (int j = 0; j < listed; ++j) before += ranks_before(val[j], idx[j], val[t], idx[t]) ? 1 : 0;
        if (before < k) {
            out_idx[(size_t)q * k + before] = idx[t];
            out_sim[(size_t)q * k + before] = val[t];
        }
    }
    // fewer usable rows than k: the rest is empty
    int usable = 0;
    for (int j = 0; j < listed; ++j) usable += idx[j] >= 0 ? 1 : 0;
    for (int r = usable + t; r < k; r += 256) {
        out_idx[(size_t)q * k + r] = -1;
        out_sim[(size_t)q * k + r] = -INFINITY;
    }
}

// Row by row: one 256-thread block per query (only the queries with scan[q] != 0 if scan is given).  Wave w
// takes rows w, w + 4, ...; lane j of a wave holds the wave's j-th best so far, a better row is inserted by
// shifting the lanes behind its place.  The four lists are merged by counting.
template <typename T>
__global__ __launch_bounds__(256) void k_topk_scan(const T *__restrict__ Q, const T *__restrict__ cent,
                                                    const float *__restrict__ invn, long K, int d, int k, int vec,
                                                    const float *__restrict__ q_inv, const int *__restrict__ scan,
                                                    int *out_idx, float *out_sim) {
    constexpr int EPC = 16 / (int)sizeof(T);
    __shared__ float sh_f[4];
    __shared__ u32x4_t sh_q[SISO_MAX_DIM / EPC];
    __shared__ float val[4 * SISO_TOPK_MAX];
    __shared__ int idx[4 * SISO_TOPK_MAX];
    const long q = blockIdx.x;
    if (scan && !scan[q]) return;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const T *qrow = Q + (size_t)q * d;
    float ss = 0.f;
    if (vec) {
        for (int e = t * EPC; e < d; e += 256 * EPC) {
            const u32x4_t v = *(const u32x4_t *)(qrow + e);
            sh_q[e / EPC] = v;
            ss += chunk_dot(v, v, T());
        }
    } else {
        for (int e = t; e < d; e += 256) ss += widen(qrow[e]) * widen(qrow[e]);
    }
    ss = wave_sum(ss);
    if (lane == 0) sh_f[wave] = ss;
    __syncthreads();
    const float qi = q_inv ? q_inv[q] : inv_length((sh_f[0] + sh_f[1]) + (sh_f[2] + sh_f[3]));
    if (!(qi == qi)) {
        for (int r = t; r < k; r += 256) {
            out_idx[(size_t)q * k + r] = -1;
            out_sim[(size_t)q * k + r] = __uint_as_float(0x7FC00000u);
        }
        return;
    }
    float mv = -INFINITY;  // this lane's entry of the wave's list
    int mi = -1;
    for (long r = wave; r < K; r += 4) {
        const T *crow = cent + (size_t)r * d;
        float acc = 0.f;
        if (vec) {
            for (int e0 = lane * EPC; e0 < d; e0 += 64 * EPC)
                acc += chunk_dot(sh_q[e0 / EPC], *(const u32x4_t *)(crow + e0), T());
        } else {
            for (int e = lane; e < d; e += 64) acc += widen(qrow[e]) * widen(crow[e]);
        }
        acc = wave_sum(acc);
        const float sv = acc * qi * invn[r];
        if (!(sv == sv)) continue;  // uniform over the wave
        // place = number of entries that stay before the new one (rows ascend, so an equal value stays before)
        const u64 stay = __ballot(lane < k && ranks_before(mv, mi, sv, (int)r));
        const int place = __popcll(stay);
        if (place >= k) continue;
        const float uv = __shfl_up(mv, 1);
        const int ui = __shfl_up(mi, 1);
        if (lane > place) {
            mv = uv;
            mi = ui;
        } else if (lane == place) {
            mv = sv;
            mi = (int)r;
        }
    }
    if (lane < k) {
        val[wave * SISO_TOPK_MAX + lane] = mv;
        idx[wave * SISO_TOPK_MAX + lane] = mi;
    }
    __syncthreads();
    int usable = 0;
    for (int w = 0; w < 4; ++w)
        for (int j = 0; j < k; ++j) usable += idx[w * SISO_TOPK_MAX + j] >= 0 ? 1 : 0;
    if (t < 4 * SISO_TOPK_MAX && (t % SISO_TOPK_MAX) < k && idx[t] >= 0) {
        int before = 0;
        for (int w = 0; w < 4; ++w)
            for (int j = 0; j < k; ++j) {
                const int o = w * SISO_TOPK_MAX + j;
                before += ranks_before(val[o], idx[o], val[t], idx[t]) ? 1 : 0;
            }
        if (before < k) {
            out_idx[(size_t)q * k + before] = idx[t];
            out_sim[(size_t)q * k + before] = val[t];
        }
    }
    for (int r = usable + t; r < k; r += 256) {
        out_idx[(size_t)q * k + r] = -1;
        out_sim[(size_t)q * k + r] = -INFINITY;
    }
}

int ensure_topk_workspace(siso_cache *c, long n) {
    if (n <= c->topk_cap) return SISO_OK;
    if (c->topk_tau) {
        const int rc = siso_check_hip(c, hipStreamSynchronize(c->stream), "siso_lookup_topk: synchronize");
        if (rc != SISO_OK) return rc;
        (void)hipFree(c->topk_tau);
        (void)hipFree(c->topk_cnt);
        (void)hipFree(c->topk_cand);
        c->topk_tau = nullptr;
        c->topk_cnt = nullptr;
        c->topk_cand = nullptr;
        c->topk_cap = 0;
    }
    bool ok = hipMalloc((void **)&c->topk_tau, (size_t)n * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->topk_cnt, (size_t)n * 2 * sizeof(int)) == hipSuccess;  // counts, then scan flags
    ok = ok && hipMalloc((void **)&c->topk_cand, (size_t)n * SISO_TOPK_CAND * sizeof(int)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        if (c->topk_tau) (void)hipFree(c->topk_tau);
        if (c->topk_cnt) (void)hipFree(c->topk_cnt);
        c->topk_tau = nullptr;
        c->topk_cnt = nullptr;
        c->topk_cand = nullptr;
        return siso_fail(c, SISO_ENOMEM, "siso_lookup_topk: workspace for %ld queries", n);
    }
    c->topk_cap = n;
    return SISO_OK;
}

template <typename T>
int topk_launch(siso_cache *c, const void *queries, long n, int k, int slices, const float *q_inv, int *out_idx,
                float *out_sim) {
    const T *Q = (const T *)queries;
    const T *cent = (const T *)c->cent;
    const int vec = ((c->dim * sizeof(T)) % 16 == 0 && ((uintptr_t)queries & 15) == 0) ? 1 : 0;
    const int *scan = nullptr;
    if (slices > 0) {
        int *cnt = c->topk_cnt, *flags = c->topk_cnt + c->topk_cap;
        hipLaunchKernelGGL(k_topk_bound, dim3((unsigned)n), dim3(256), (size_t)slices * sizeof(u64), c->stream, c->keys, slices,
                           k, c->topk_tau, cnt, flags);
        int rc = siso_check_hip(c, hipGetLastError(), "k_topk_bound");
        if (rc == SISO_OK)
            rc = siso_topk_mfma_collect(c, queries, n, slices, c->topk_tau, c->topk_cand, cnt, SISO_TOPK_CAND);
        if (rc != SISO_OK) return rc;
        hipLaunchKernelGGL(k_topk_select<T>, dim3((unsigned)n), dim3(256), 0, c->stream, Q, cent, c->invn, c->count, c->dim, k,
                           c->topk_cand, cnt, SISO_TOPK_CAND, q_inv, flags, out_idx, out_sim);
        rc = siso_check_hip(c, hipGetLastError(), "k_topk_select");
        if (rc != SISO_OK) return rc;
        scan = flags;
    }
    hipLaunchKernelGGL(k_topk_scan<T>, dim3((unsigned)n), dim3(256), 0, c->stream, Q, cent, c->invn, c->count, c->dim, k, vec,
                       q_inv, scan, out_idx, out_sim);
    return siso_check_hip(c, hipGetLastError(), "k_topk_scan");
}

}  // namespace

// siso_reserve's part for top-k lookups is not needed: the call says that it may allocate.
extern "C" int siso_lookup_topk(siso_cache *c, const void *queries, long n, int k, int *out_idx, float *out_sim) {
    if (!c) return SISO_EINVAL;
    if (n < 0 || k < 1 || k > SISO_TOPK_MAX || (n > 0 && (!queries || !out_idx || !out_sim)))
        return siso_fail(c, SISO_EINVAL, "siso_lookup_topk: bad arguments (1 <= k <= %d)", SISO_TOPK_MAX);
    if (n == 0) return SISO_OK;
    if (n > 2147483647L / 4) return siso_fail(c, SISO_EINVAL, "siso_lookup_topk: batch of %ld is too large", n);
    const bool fp8 = c->dtype == SISO_FP8;
    int rc = SISO_OK;
    const void *rows = queries;  // what the kernels read: the batch, or its codes
    if (fp8) {
        rc = siso_fp8_ensure_batch(c, n);
        if (rc == SISO_OK) rc = siso_fp8_quantize_batch(c, queries, n);
        if (rc != SISO_OK) return rc;
        rows = c->fp8_q;
    }
    // the two-pass path needs many more slices than k, and rows that are whole 16-byte chunks; for codes
    // it exists on the 64-deep kernels only
    int slices = 0;
    const bool mfma_ok = c->dtype == SISO_BF16 || (fp8 && (c->opt_mfma_config == 0 || (c->opt_mfma_config >= 6 && c->opt_mfma_config <= 8)));
    if (c->count >= 512L * k && mfma_ok && ((uintptr_t)rows & 15) == 0) {
        c->plan_min_slices = 8 * k;
        slices = siso_topk_mfma_slices(c, n);
        if (slices < 2 * k || slices > 4096) slices = 0;  // (the bound kernel keeps a query's keys in LDS)
    }
    if (slices > 0) {
        rc = ensure_topk_workspace(c, n);
        if (rc == SISO_OK) rc = siso_ensure_keys(c, n * (long)slices);
        int row_keys = 0;
        if (rc == SISO_OK) rc = siso_topk_mfma_pass1(c, rows, n, slices, c->keys, &row_keys);
    }
    if (rc == SISO_OK)
        rc = c->dtype == SISO_F32 ? topk_launch<float>(c, rows, n, k, slices, nullptr, out_idx, out_sim)
             : fp8              ? topk_launch<fp8_t>(c, rows, n, k, slices, c->fp8_qinv, out_idx, out_sim)
                                : topk_launch<bf16_t>(c, rows, n, k, slices, nullptr, out_idx, out_sim);
    c->plan_min_slices = 0;
    return rc;
}

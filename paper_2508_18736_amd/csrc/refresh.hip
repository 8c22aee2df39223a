// Cache replacement: Algorithm 1 (SISO-CacheManager) of section 4.2 — MergeCentroids,
// FilteringCentroids, UpdateCentroids.
//
// The merge step takes the repository centroids one after the other and compares each with
// C_new as it stands then, so its decisions form a chain.  What is heavy in it is data
// parallel and runs in the library's kernels:
//   * every repository row against every cached centroid: one batched lookup;
//   * every repository row against every other one: the pair search, which lists the pairs above
//     the clustering threshold (only those can change a decision: a row joins C_new when nothing
//     in it is closer than the threshold, whatever is closest then);
//   * the cosines of the listed pairs (to tell which candidate is the closest).
// The chain itself (who joined, who took whose cluster size) and the choice of the survivors
// (the smallest (cluster_size, access_count) go first) are bookkeeping over a few numbers per
// row and are done on the host, in the order the algorithm states; then the new centroid set is
// gathered on the GPU and becomes the cache between two lookups of the stream (a lookup sees
// the old set or the new one, never a mixture; nothing is locked, so nothing needs to be
// replaced piecemeal).
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "siso_internal.h"

namespace {

typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__global__ void k_clear(u64 *p) { *p = 0; }

__global__ void k_nan_tail(float *p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = __uint_as_float(0x7FC00000u);
}

// Copy the repository rows into a buffer with readable rows behind them, with 1 / |row|; count the
// rows that hold a NaN or an infinity and the cluster sizes that are not positive finite numbers.
template <typename T>
__global__ __launch_bounds__(256) void k_stage_repo(const T *__restrict__ src, const float *__restrict__ sizes, T *dst,
                                                     float *invn, int d, u64 *bad) {
    __shared__ float sh[4];
    const long k = blockIdx.x;
    float ss = 0.f;
    for (int e = threadIdx.x; e < d; e += 256) {
        const T x = src[(size_t)k * d + e];
        dst[(size_t)k * d + e] = x;
        const float f = widen(x);
        ss += f * f;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float inv = inv_length((sh[0] + sh[1]) + (sh[2] + sh[3]));
        invn[k] = inv;
        const float s = sizes[k];
        if (!(inv == inv) || !(s > 0.f) || s > 3.0e38f) atomicAdd(bad, 1ull);
    }
}

// cosine of the two rows of every listed pair, one wave per pair (the arithmetic of the lookup's
// last step: fp32 products summed per lane, then over the lanes, then scaled by both inverse lengths)
template <typename T>
__global__ __launch_bounds__(256) void k_pair_cosines(const T *__restrict__ rows, const float *__restrict__ invn,
                                                       const int *__restrict__ pairs, long n_pairs, int d, float *out) {
    const long p = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= n_pairs) return;
    const int lane = threadIdx.x & 63;
    const long a = pairs[2 * p], b = pairs[2 * p + 1];
    float acc = 0.f;
    for (int e = lane; e < d; e += 64) acc += widen(rows[(size_t)a * d + e]) * widen(rows[(size_t)b * d + e]);
    acc = wave_sum(acc);
    if (lane == 0) out[p] = acc * invn[a] * invn[b];
}

// New row j <- source src[j]: a cached row (src < K0) with all it carries, or repository row
// src - K0, which starts a cluster of its own: stored as it is, mean = its direction, weight of
// the mean = its cluster size rounded to a whole number of members (at least 1).
template <typename T>
__global__ __launch_bounds__(256) void k_refresh_gather(const int *__restrict__ src, long K0, const T *__restrict__ cent,
                                                         const float *__restrict__ mean, const int *__restrict__ size,
                                                         const float *__restrict__ invn, const T *__restrict__ repo,
                                                         const float *__restrict__ repo_invn,
                                                         const float *__restrict__ repo_size, T *cent2, float *mean2,
                                                         int *size2, float *invn2, int d) {
    const long j = blockIdx.x;
    const long s = src[j];
    if (s < K0) {
        for (int e = threadIdx.x; e < d; e += 256) {
            cent2[(size_t)j * d + e] = cent[(size_t)s * d + e];
            mean2[(size_t)j * d + e] = mean[(size_t)s * d + e];
        }
        if (threadIdx.x == 0) {
            size2[j] = size[s];
            invn2[j] = invn[s];
        }
    } else {
        const long r = s - K0;
        const float inv = repo_invn[r];
        for (int e = threadIdx.x; e < d; e += 256) {
            const T x = repo[(size_t)r * d + e];
            cent2[(size_t)j * d + e] = x;
            mean2[(size_t)j * d + e] = widen(x) * inv;  // inv = 0 for a zero row
        }
        if (threadIdx.x == 0) {
            const float w = rintf(repo_size[r]);
            size2[j] = w < 1.f ? 1 : (w > 2147483647.f ? 2147483647 : (int)w);
            invn2[j] = inv;
        }
    }
}

struct DeviceBuf {  // frees on every way out
    void *p = nullptr;
    ~DeviceBuf() {
        if (p) (void)hipFree(p);
    }
    bool alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 1) == hipSuccess; }
    template <class U>
    U *as() const {
        return (U *)p;
    }
};

struct Candidate {  // an earlier repository row above the threshold
    int row;
    float cosine;
};

// The decisions of Algorithm 1 from what the kernels found.  Per repository row i: h_idx / h_sim = its closest
// cached centroid and the cosine; h_pairs / h_cos = the pairs (a, b), a < b, of repository rows above the
// threshold with their cosines.  loc / acc = cluster_size and access_count of the cached centroids (they grow
// by the rows that join).  keep = source of every surviving row in order (cached row, or K0 + repository row),
// loc2 = its cluster_size after the decay.
void plan_refresh(long K0, long r, const int *h_idx, const float *h_sim, const float *h_rsize, const int *h_pairs,
                  const float *h_cos, long n_pairs, std::vector<float> loc, std::vector<unsigned> acc, float theta_c,
                  long max_centroids, std::vector<int> &keep, std::vector<float> &loc2, long &merged, long &added,
                  long &evicted) {
    // ---- the chain of the merge step, in the order of the repository ---------------------
    // candidates of row b: the earlier rows a < b with cosine above the threshold (pairs come as a < b)
    std::vector<long> first((size_t)r + 1, 0);
    for (long p = 0; p < n_pairs; ++p) first[(size_t)h_pairs[2 * p + 1] + 1] += 1;
    for (long i = 0; i < r; ++i) first[(size_t)i + 1] += first[(size_t)i];
    std::vector<Candidate> cand((size_t)n_pairs);
    {
        std::vector<long> fill(first.begin(), first.end() - 1);
        for (long p = 0; p < n_pairs; ++p) {
            const int b = h_pairs[2 * p + 1];
            cand[(size_t)fill[(size_t)b]++] = Candidate{h_pairs[2 * p], h_cos[(size_t)p]};
        }
    }
    std::vector<long> place((size_t)r, -1);  // position in C_new of a repository row that joined
    std::vector<int> src;                    // C_new: source of every row (cached row, or K0 + repository row)
    src.reserve((size_t)(K0 + r));
    for (long j = 0; j < K0; ++j) src.push_back((int)j);
    merged = added = 0;
    for (long i = 0; i < r; ++i) {
        long best = h_idx[(size_t)i];
        float bsim = h_sim[(size_t)i];
        if (best < 0 || !(bsim == bsim)) {
            best = -1;
            bsim = -INFINITY;
        }
        for (long q = first[(size_t)i]; q < first[(size_t)i + 1]; ++q) {
            const long pos = place[(size_t)cand[(size_t)q].row];
            if (pos < 0) continue;  // that row did not join: it is not in C_new
            const float s = cand[(size_t)q].cosine;
            if (s > bsim || (s == bsim && pos < best)) {
                bsim = s;
                best = pos;
            }
        }
        if (best >= 0 && bsim > theta_c) {
            loc[(size_t)best] = loc[(size_t)best] + h_rsize[(size_t)i];
            ++merged;
        } else {
            place[(size_t)i] = (long)src.size();
            src.push_back((int)(K0 + i));
            loc.push_back(h_rsize[(size_t)i]);
            acc.push_back(SISO_ACCESS_INF);
            ++added;
        }
    }

    // ---- filtering step: the smallest (cluster_size, access_count) go, the first such first ----
    const long n_new = (long)src.size();
    evicted = 0;
    std::vector<unsigned char> gone((size_t)n_new, 0);
    if (n_new > max_centroids) {
        evicted = n_new - max_centroids;
        std::vector<int> order((size_t)n_new);
        for (long j = 0; j < n_new; ++j) order[(size_t)j] = (int)j;
        auto before = [&](int x, int y) {
            if (loc[(size_t)x] != loc[(size_t)y]) return loc[(size_t)x] < loc[(size_t)y];
            if (acc[(size_t)x] != acc[(size_t)y]) return acc[(size_t)x] < acc[(size_t)y];
            return x < y;
        };
        std::nth_element(order.begin(), order.begin() + evicted, order.end(), before);
        for (long v = 0; v < evicted; ++v) gone[(size_t)order[(size_t)v]] = 1;
    }
    keep.reserve((size_t)(n_new - evicted));
    loc2.reserve((size_t)(n_new - evicted));
    for (long j = 0; j < n_new; ++j) {
        if (gone[(size_t)j]) continue;
        keep.push_back(src[(size_t)j]);
        loc2.push_back(loc[(size_t)j] / 1.1f);
    }
}

}  // namespace

static int refresh_impl(siso_cache *c, const void *repo, const float *repo_size, long r, float theta_c,
                        long max_centroids, long *out_stats) {
    if (!c) return SISO_EINVAL;
    if (c->dtype == SISO_FP8) return siso_fail(c, SISO_EINVAL, "siso_refresh: not available with the 8-bit storage");
    if (out_stats) out_stats[0] = out_stats[1] = out_stats[2] = 0;
    if (r < 0 || max_centroids < 1 || max_centroids > c->capacity || (r > 0 && (!repo || !repo_size)))
        return siso_fail(c, SISO_EINVAL, "siso_refresh: bad arguments (1 <= max_centroids <= capacity %ld)", c->capacity);
    if (r > 2147483647L / 4 || c->count + r > 2147483647L)
        return siso_fail(c, SISO_EINVAL, "siso_refresh: %ld repository rows are too many", r);
    if (((uintptr_t)repo & 15) != 0) return siso_fail(c, SISO_EINVAL, "siso_refresh: repository rows must be 16-byte aligned");
    const long K0 = c->count;
    const int d = c->dim;
    const size_t eb = c->dtype == SISO_F32 ? 4 : 2;
    hipStream_t st = c->stream;
#define REFRESH_TRY(expr, what)                                   \
    do {                                                          \
        const int rc_ = siso_check_hip(c, (expr), what);          \
        if (rc_ != SISO_OK) return rc_;                           \
    } while (0)

    // ---- device side of the merge step -------------------------------------------------
    DeviceBuf d_rows, d_rinv, d_idx, d_sim, d_pairs, d_cos;
    std::vector<int> h_idx((size_t)r);
    std::vector<float> h_sim((size_t)r), h_rsize((size_t)r), h_cos;
    std::vector<int> h_pairs;
    long n_pairs = 0;
    if (r > 0) {
        if (!d_rows.alloc((size_t)(r + SISO_PAD_ROWS) * d * eb) || !d_rinv.alloc((size_t)(r + SISO_PAD_ROWS) * sizeof(float)) ||
            !d_idx.alloc((size_t)r * sizeof(int)) || !d_sim.alloc((size_t)r * sizeof(float))) {
            (void)hipGetLastError();
            return siso_fail(c, SISO_ENOMEM, "siso_refresh: staging for %ld repository rows", r);
        }
        REFRESH_TRY(hipMemsetAsync((char *)d_rows.p + (size_t)r * d * eb, 0, (size_t)SISO_PAD_ROWS * d * eb, st), "clear pad rows");
        hipLaunchKernelGGL(k_clear, dim3(1), dim3(1), 0, st, c->counters + 2);
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_stage_repo<float>, dim3((unsigned)r), dim3(256), 0, st, (const float *)repo, repo_size,
                               d_rows.as<float>(), d_rinv.as<float>(), d, c->counters + 2);
        else
            hipLaunchKernelGGL(k_stage_repo<bf16_t>, dim3((unsigned)r), dim3(256), 0, st, (const bf16_t *)repo, repo_size,
                               d_rows.as<bf16_t>(), d_rinv.as<float>(), d, c->counters + 2);
        hipLaunchKernelGGL(k_nan_tail, dim3(1), dim3(SISO_PAD_ROWS), 0, st, d_rinv.as<float>() + r, SISO_PAD_ROWS);
        REFRESH_TRY(hipGetLastError(), "stage repository rows");
        u64 bad = 0;
        int rc = siso_read_counter(c, 2, &bad);
        if (rc != SISO_OK) return rc;
        if (bad != 0)
            return siso_fail(c, SISO_EINVAL, "siso_refresh: %llu repository rows are not finite or have no positive cluster size", bad);

        // every repository row against the cache (test lookups: no references are counted)
        rc = siso_lookup_impl(c, d_rows.p, r, &theta_c, 1, -1, d_idx.as<int>(), d_sim.as<float>(), nullptr);
        if (rc != SISO_OK) return rc;

        // repository rows among themselves: the pairs above the threshold, then their cosines
        long cap = r * 4 > (1L << 20) ? r * 4 : (1L << 20);
        for (int attempt = 0; attempt < 2 && r >= 2; ++attempt) {
            if (d_pairs.p) {
                (void)hipFree(d_pairs.p);
                d_pairs.p = nullptr;
            }
            if (!d_pairs.alloc((size_t)cap * 2 * sizeof(int))) {
                (void)hipGetLastError();
                return siso_fail(c, SISO_ENOMEM, "siso_refresh: room for %ld pairs", cap);
            }
            hipLaunchKernelGGL(k_clear, dim3(1), dim3(1), 0, st, c->counters + 1);
            REFRESH_TRY(hipGetLastError(), "k_clear");
            if (siso_pairs_mfma_supported(c, r))
                rc = siso_pairs_mfma_launch(c, d_rows.p, d_rinv.as<float>(), r, theta_c, d_pairs.as<int>(), cap, c->counters + 1);
            else
                rc = siso_pairs_scalar_launch(c, d_rows.p, d_rinv.as<float>(), r, theta_c, d_pairs.as<int>(), cap, c->counters + 1);
            if (rc != SISO_OK) return rc;
            u64 total = 0;
            rc = siso_read_counter(c, 1, &total);
            if (rc != SISO_OK) return rc;
            n_pairs = (long)total;
            if (n_pairs <= cap) break;
            if (attempt == 1) return siso_fail(c, SISO_ENOMEM, "siso_refresh: %ld pairs above the threshold", n_pairs);
            cap = n_pairs;  // once more with room for all of them
        }
        if (n_pairs > 0) {
            if (!d_cos.alloc((size_t)n_pairs * sizeof(float))) {
                (void)hipGetLastError();
                return siso_fail(c, SISO_ENOMEM, "siso_refresh: cosines of %ld pairs", n_pairs);
            }
            const unsigned blocks = (unsigned)((n_pairs + 3) / 4);
            if (c->dtype == SISO_F32)
                hipLaunchKernelGGL(k_pair_cosines<float>, dim3(blocks), dim3(256), 0, st, d_rows.as<float>(), d_rinv.as<float>(),
                                   d_pairs.as<int>(), n_pairs, d, d_cos.as<float>());
            else
                hipLaunchKernelGGL(k_pair_cosines<bf16_t>, dim3(blocks), dim3(256), 0, st, d_rows.as<bf16_t>(), d_rinv.as<float>(),
                                   d_pairs.as<int>(), n_pairs, d, d_cos.as<float>());
            REFRESH_TRY(hipGetLastError(), "k_pair_cosines");
            h_pairs.resize((size_t)n_pairs * 2);
            h_cos.resize((size_t)n_pairs);
            REFRESH_TRY(hipMemcpyAsync(h_pairs.data(), d_pairs.p, (size_t)n_pairs * 2 * sizeof(int), hipMemcpyDeviceToHost, st), "pairs to host");
            REFRESH_TRY(hipMemcpyAsync(h_cos.data(), d_cos.p, (size_t)n_pairs * sizeof(float), hipMemcpyDeviceToHost, st), "cosines to host");
        }
        REFRESH_TRY(hipMemcpyAsync(h_idx.data(), d_idx.p, (size_t)r * sizeof(int), hipMemcpyDeviceToHost, st), "idx to host");
        REFRESH_TRY(hipMemcpyAsync(h_sim.data(), d_sim.p, (size_t)r * sizeof(float), hipMemcpyDeviceToHost, st), "sim to host");
        REFRESH_TRY(hipMemcpyAsync(h_rsize.data(), repo_size, (size_t)r * sizeof(float), hipMemcpyDeviceToHost, st), "sizes to host");
    }
    std::vector<float> loc((size_t)K0);
    std::vector<unsigned> acc((size_t)K0);
    if (K0 > 0) {
        REFRESH_TRY(hipMemcpyAsync(loc.data(), c->locality, (size_t)K0 * sizeof(float), hipMemcpyDeviceToHost, st), "cluster sizes to host");
        REFRESH_TRY(hipMemcpyAsync(acc.data(), c->access, (size_t)K0 * sizeof(unsigned), hipMemcpyDeviceToHost, st), "access counts to host");
    }
    REFRESH_TRY(hipStreamSynchronize(st), "siso_refresh: synchronize");

    // ---- merge step and filtering step: bookkeeping on the host ----------------------------------
    std::vector<int> keep;
    std::vector<float> loc2;
    long merged = 0, added = 0, evicted = 0;
    plan_refresh(K0, r, h_idx.data(), h_sim.data(), h_rsize.data(), h_pairs.data(), h_cos.data(), n_pairs, loc, acc, theta_c,
                 max_centroids, keep, loc2, merged, added, evicted);
    const long live = (long)keep.size();

    // ---- update step: gather the new set, then it becomes the cache ---------------------------
    DeviceBuf d_src;
    if (live > 0) {
        const int rc2 = siso_second_set(c);
        if (rc2 != SISO_OK) return rc2;
        if (!d_src.alloc((size_t)live * sizeof(int))) {
            (void)hipGetLastError();
            return siso_fail(c, SISO_ENOMEM, "siso_refresh: sources of %ld centroids", live);
        }
        REFRESH_TRY(hipMemcpyAsync(d_src.p, keep.data(), (size_t)live * sizeof(int), hipMemcpyHostToDevice, st), "sources to device");
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_refresh_gather<float>, dim3((unsigned)live), dim3(256), 0, st, d_src.as<int>(), K0,
                               (const float *)c->cent, c->mean, c->size, c->invn, d_rows.as<float>(), d_rinv.as<float>(),
                               repo_size, (float *)c->cent_b, c->mean_b, c->size_b, c->invn_b, d);
        else
            hipLaunchKernelGGL(k_refresh_gather<bf16_t>, dim3((unsigned)live), dim3(256), 0, st, d_src.as<int>(), K0,
                               (const bf16_t *)c->cent, c->mean, c->size, c->invn, d_rows.as<bf16_t>(), d_rinv.as<float>(),
                               repo_size, (bf16_t *)c->cent_b, c->mean_b, c->size_b, c->invn_b, d);
        REFRESH_TRY(hipGetLastError(), "k_refresh_gather");
        REFRESH_TRY(hipMemcpyAsync(c->locality_b, loc2.data(), (size_t)live * sizeof(float), hipMemcpyHostToDevice, st), "new cluster sizes");
        REFRESH_TRY(hipMemsetAsync(c->access_b, 0, (size_t)live * sizeof(unsigned), st), "reset access counts");
        siso_swap_sets(c);  // lookups enqueued from here on see the new set
    }
    hipLaunchKernelGGL(k_nan_tail, dim3(1), dim3(SISO_PAD_ROWS), 0, st, c->invn + live, SISO_PAD_ROWS);
    REFRESH_TRY(hipGetLastError(), "k_nan_tail");
    REFRESH_TRY(hipStreamSynchronize(st), "siso_refresh: synchronize");
    c->count = live;
    if (out_stats) {
        out_stats[0] = merged;
        out_stats[1] = added;
        out_stats[2] = evicted;
    }
#undef REFRESH_TRY
    return SISO_OK;
}

extern "C" int siso_refresh(siso_cache *c, const void *repo, const float *repo_size, long r, float theta_c,
                            long max_centroids, long *out_stats) {
    if (!c) return SISO_EINVAL;
    try {
        return refresh_impl(c, repo, repo_size, r, theta_c, max_centroids, out_stats);
    } catch (const std::bad_alloc &) {  // the host lists; they are all built before the update step
        return siso_fail(c, SISO_ENOMEM, "siso_refresh: host memory for the bookkeeping");
    }
}

// The host part of siso_refresh alone (all pointers are HOST pointers).
extern "C" long siso_refresh_plan(long k0, const float *cluster_size, const unsigned *access_count, long r,
                                  const float *repo_size, const int *best_idx, const float *best_sim, const int *pairs,
                                  const float *pair_cosine, long n_pairs, float theta_c, long max_centroids,
                                  int *out_source, float *out_cluster_size, long *out_stats) {
    if (k0 < 0 || r < 0 || n_pairs < 0 || max_centroids < 1 || !out_source || !out_cluster_size) return SISO_EINVAL;
    if ((k0 > 0 && (!cluster_size || !access_count)) || (r > 0 && (!repo_size || !best_idx || !best_sim)) ||
        (n_pairs > 0 && (!pairs || !pair_cosine)))
        return SISO_EINVAL;
    for (long p = 0; p < n_pairs; ++p)
        if (pairs[2 * p] < 0 || pairs[2 * p] >= pairs[2 * p + 1] || pairs[2 * p + 1] >= r) return SISO_EINVAL;
    for (long i = 0; i < r; ++i)
        if (best_idx[i] >= k0 || !(repo_size[i] > 0.f)) return SISO_EINVAL;
    try {
        std::vector<float> loc(cluster_size, cluster_size + k0), loc2;
        std::vector<unsigned> acc(access_count, access_count + k0);
        std::vector<int> keep;
        long merged = 0, added = 0, evicted = 0;
        plan_refresh(k0, r, best_idx, best_sim, repo_size, pairs, pair_cosine, n_pairs, loc, acc, theta_c, max_centroids,
                     keep, loc2, merged, added, evicted);
        for (size_t j = 0; j < keep.size(); ++j) {
            out_source[j] = keep[j];
            out_cluster_size[j] = loc2[j];
        }
        if (out_stats) {
            out_stats[0] = merged;
            out_stats[1] = added;
            out_stats[2] = evicted;
        }
        return (long)keep.size();
    } catch (const std::bad_alloc &) {
        return SISO_ENOMEM;
    }
}

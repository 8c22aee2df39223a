// Clustering of a query log into the centroid repository (section 4.1): community detection at the
// clustering threshold ("Selecting a clustering algorithm"), then one repository row per cluster
// ("Keeping centroids in a repository": id, centroid = the average of the members (section 3.1),
// cluster_size = their number).
//
// The heavy part is the all-pairs similarity of the n vectors, n * n * dim / 2 products: that is the
// pair search of the merge (the pairs above the threshold are the edges of the neighbour graph), and
// the member averages; both run in kernels.  Between them sits the greedy choice of the communities
// (largest candidate first; a candidate keeps the vectors no earlier community took), which is a walk
// over the edge list in a fixed order: bookkeeping on the host, linear in vectors + edges.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "siso_internal.h"

namespace {

__global__ void k_clear_counter(u64 *p) { *p = 0; }

__global__ void k_nan_fill(float *p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = __uint_as_float(0x7FC00000u);
}

// Copy the vectors into a buffer with readable rows behind them, with 1 / |row|; count the rows that
// hold a NaN or an infinity or have no length.
template <typename T>
__global__ __launch_bounds__(256) void k_stage_vectors(const T *__restrict__ src, T *dst, float *invn, int d, u64 *bad) {
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
        if (!(inv == inv) || inv == 0.f) atomicAdd(bad, 1ull);
    }
}

__device__ __forceinline__ float block_total(float v, float *sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// One block per cluster k: members member[first[k] .. first[k+1]) in ascending order.
// mean = average of the unit-length members; stored centroid = mean / |mean| rounded to the element
// type (a zero row when the mean has no length); size = cluster_size = number of members; no references yet.
// rep (nullable): the member with the largest cosine to the mean, the lowest index among equals.
template <typename T>
__global__ __launch_bounds__(256) void k_cluster_rows(const T *__restrict__ vec, const float *__restrict__ vinv,
                                                       const long *__restrict__ first, const int *__restrict__ member,
                                                       T *cent, float *mean, int *size, float *invn, float *locality,
                                                       unsigned *access, int *rep, int d) {
    __shared__ float sh[4];
    __shared__ float sh_mean[SISO_MAX_DIM];
    __shared__ float sh_best[4];
    __shared__ int sh_who[4];
    const long k = blockIdx.x;
    const int t = threadIdx.x;
    const long lo = first[k], hi = first[k + 1];
    const float count = (float)(hi - lo);
    float ss = 0.f;
    for (int col = t; col < d; col += 256) {
        float acc = 0.f;
        for (long p = lo; p < hi; ++p) {
            const long j = member[p];
            acc += widen(vec[(size_t)j * d + col]) * vinv[j];
        }
        const float m = acc / count;
        mean[(size_t)k * d + col] = m;
        sh_mean[col] = m;
        ss += m * m;
    }
    const float n2 = block_total(ss, sh);
    const bool has_length = n2 > 0.f && n2 <= 3.0e38f;
    const float nrm = has_length ? sqrtf(n2) : 1.f;
    float cs = 0.f;
    for (int col = t; col < d; col += 256) {
        T v;
        narrow(has_length ? mean[(size_t)k * d + col] / nrm : 0.f, &v);  // this thread wrote that element itself
        cent[(size_t)k * d + col] = v;
        const float back = widen(v);
        cs += back * back;
    }
    const float c2 = block_total(cs, sh);  // (its barriers also make the whole mean in LDS visible)
    if (t == 0) {
        size[k] = hi - lo > 2147483647L ? 2147483647 : (int)(hi - lo);
        invn[k] = inv_length(c2);
        locality[k] = count;
        access[k] = 0u;
    }
    if (!rep) return;
    // the member closest to the centroid: cosine(x_j, m) = <x_j, m> / (|x_j| |m|), and |m| is the same for
    // all of them.  One wave per member, members in ascending order within a wave.
    const int lane = t & 63, wave = t >> 6;
    float best = -INFINITY;
    int who = 0x7FFFFFFF;
    for (long p = lo + wave; p < hi; p += 4) {
        const long j = member[p];
        float dot = 0.f;
        for (int col = lane; col < d; col += 64) dot += widen(vec[(size_t)j * d + col]) * sh_mean[col];
        dot = wave_sum(dot) * vinv[j];
        if (dot > best) {
            best = dot;
            who = (int)j;
        }
    }
    if (lane == 0) {
        sh_best[wave] = best;
        sh_who[wave] = who;
    }
    __syncthreads();
    if (t == 0) {
        for (int w = 1; w < 4; ++w)
            if (sh_best[w] > best || (sh_best[w] == best && sh_who[w] < who)) {
                best = sh_best[w];
                who = sh_who[w];
            }
        rep[k] = who;
    }
}

struct DeviceMem {  // frees on every way out
    void *p = nullptr;
    ~DeviceMem() { release(); }
    void release() {
        if (p) (void)hipFree(p);
        p = nullptr;
    }
    bool alloc(size_t bytes) {
        release();
        return hipMalloc(&p, bytes ? bytes : 1) == hipSuccess;
    }
    template <class U>
    U *as() const {
        return (U *)p;
    }
};

// The greedy choice of the communities from the list of neighbour pairs (host memory, each pair once, in any
// order): candidates = every vector with its neighbours, largest first, equal sizes by index; a candidate
// keeps the vectors no earlier cluster took and becomes a cluster if at least min_size remain.
// label[i] = cluster of vector i or -1; the members of cluster k, in ascending order, are
// member[first[k] .. first[k+1]).  Linear in vectors + pairs (counting sort, one pass over the lists).
void choose_communities(const int *h_pairs, long n_pairs, long n, int min_size, std::vector<int> &label,
                        std::vector<long> &first, std::vector<int> &member) {
    // ---- neighbour lists -----------------------------------------------------------------------
    std::vector<long> start((size_t)n + 1, 0);
    for (long p = 0; p < 2 * n_pairs; ++p) start[(size_t)h_pairs[(size_t)p] + 1] += 1;
    long largest = 0;
    for (long i = 0; i < n; ++i) {
        if (start[(size_t)i + 1] > largest) largest = start[(size_t)i + 1];
        start[(size_t)i + 1] += start[(size_t)i];
    }
    std::vector<int> nbr((size_t)(2 * n_pairs));
    {
        std::vector<long> fill(start.begin(), start.end() - 1);
        for (long p = 0; p < n_pairs; ++p) {
            const int a = h_pairs[(size_t)(2 * p)], b = h_pairs[(size_t)(2 * p + 1)];
            nbr[(size_t)fill[(size_t)a]++] = b;
            nbr[(size_t)fill[(size_t)b]++] = a;
        }
    }
    // ---- candidates by size (itself + neighbours), largest first, equal sizes by index ------------
    // a counting sort over the sizes 1 .. largest + 1
    std::vector<long> bucket((size_t)largest + 3, 0);
    for (long i = 0; i < n; ++i) bucket[(size_t)(largest + 1 - (start[(size_t)i + 1] - start[(size_t)i])) + 1] += 1;
    for (long s = 0; s <= largest + 1; ++s) bucket[(size_t)s + 1] += bucket[(size_t)s];
    std::vector<int> order((size_t)n);
    for (long i = 0; i < n; ++i) order[(size_t)bucket[(size_t)(largest + 1 - (start[(size_t)i + 1] - start[(size_t)i]))]++] = (int)i;

    // ---- greedy choice ----------------------------------------------------------------------------
    label.assign((size_t)n, -1);
    first.assign(1, 0);
    member.clear();
    member.reserve((size_t)n);
    for (long q = 0; q < n; ++q) {
        const long i = order[(size_t)q];
        const long lo = start[(size_t)i], hi = start[(size_t)i + 1];
        if (hi - lo + 1 < (long)min_size) break;   // every later candidate is smaller still
        long left = label[(size_t)i] < 0 ? 1 : 0;
        for (long p = lo; p < hi; ++p) left += label[(size_t)nbr[(size_t)p]] < 0 ? 1 : 0;
        if (left < (long)min_size) continue;
        const int id = (int)(first.size() - 1);
        if (label[(size_t)i] < 0) {
            label[(size_t)i] = id;
            member.push_back((int)i);
        }
        for (long p = lo; p < hi; ++p) {
            const int j = nbr[(size_t)p];
            if (label[(size_t)j] < 0) {
                label[(size_t)j] = id;
                member.push_back(j);
            }
        }
        std::sort(member.begin() + first.back(), member.end());   // averages take the members in ascending order
        first.push_back((long)member.size());
    }
}

}  // namespace

static long cluster_impl(siso_cache *c, const void *vectors, long n, float theta_c, int min_size, int *out_label,
                         int *out_representative, long *out_stats) {
    if (!c) return SISO_EINVAL;
    if (out_stats) out_stats[0] = out_stats[1] = 0;
    if (n < 0 || min_size < 1 || (n > 0 && !vectors))
        return siso_fail(c, SISO_EINVAL, "siso_cluster: bad arguments (n >= 0, min_size >= 1)");
    if (n > 2147483647L / 4) return siso_fail(c, SISO_EINVAL, "siso_cluster: %ld vectors are too many", n);
    if (((uintptr_t)vectors & 15) != 0) return siso_fail(c, SISO_EINVAL, "siso_cluster: vectors must be 16-byte aligned");
    const int d = c->dim;
    const size_t eb = c->dtype == SISO_F32 ? 4 : 2;
    hipStream_t st = c->stream;
#define CLUSTER_TRY(expr, what)                                   \
    do {                                                          \
        const int rc_ = siso_check_hip(c, (expr), what);          \
        if (rc_ != SISO_OK) return rc_;                           \
    } while (0)

    // ---- the neighbour graph: every pair of vectors above the threshold -----------------------
    DeviceMem d_rows, d_inv, d_pairs;
    std::vector<int> h_pairs;
    long n_pairs = 0;
    if (n > 0) {
        if (!d_rows.alloc((size_t)(n + SISO_PAD_ROWS) * d * eb) || !d_inv.alloc((size_t)(n + SISO_PAD_ROWS) * sizeof(float))) {
            (void)hipGetLastError();
            return siso_fail(c, SISO_ENOMEM, "siso_cluster: staging for %ld vectors", n);
        }
        CLUSTER_TRY(hipMemsetAsync((char *)d_rows.p + (size_t)n * d * eb, 0, (size_t)SISO_PAD_ROWS * d * eb, st), "clear pad rows");
        hipLaunchKernelGGL(k_clear_counter, dim3(1), dim3(1), 0, st, c->counters + 2);
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_stage_vectors<float>, dim3((unsigned)n), dim3(256), 0, st, (const float *)vectors,
                               d_rows.as<float>(), d_inv.as<float>(), d, c->counters + 2);
        else
            hipLaunchKernelGGL(k_stage_vectors<bf16_t>, dim3((unsigned)n), dim3(256), 0, st, (const bf16_t *)vectors,
                               d_rows.as<bf16_t>(), d_inv.as<float>(), d, c->counters + 2);
        hipLaunchKernelGGL(k_nan_fill, dim3(1), dim3(SISO_PAD_ROWS), 0, st, d_inv.as<float>() + n, SISO_PAD_ROWS);
        CLUSTER_TRY(hipGetLastError(), "stage vectors");
        u64 bad = 0;
        int rc = siso_read_counter(c, 2, &bad);
        if (rc != SISO_OK) return rc;
        if (bad != 0) return siso_fail(c, SISO_EINVAL, "siso_cluster: %llu vectors are not finite or have no length", bad);

        // room for 32 pairs per vector at first (256 bytes each); a log with more gets a second pass with the exact room
        long cap = n * 32 > (1L << 20) ? n * 32 : (1L << 20);
        for (int attempt = 0; attempt < 2 && n >= 2; ++attempt) {
            if (!d_pairs.alloc((size_t)cap * 2 * sizeof(int))) {
                (void)hipGetLastError();
                return siso_fail(c, SISO_ENOMEM, "siso_cluster: room for %ld pairs", cap);
            }
            hipLaunchKernelGGL(k_clear_counter, dim3(1), dim3(1), 0, st, c->counters + 1);
            CLUSTER_TRY(hipGetLastError(), "k_clear_counter");
            if (siso_pairs_mfma_supported(c, n))
                rc = siso_pairs_mfma_launch(c, d_rows.p, d_inv.as<float>(), n, theta_c, d_pairs.as<int>(), cap, c->counters + 1);
            else
                rc = siso_pairs_scalar_launch(c, d_rows.p, d_inv.as<float>(), n, theta_c, d_pairs.as<int>(), cap, c->counters + 1);
            if (rc != SISO_OK) return rc;
            u64 total = 0;
            rc = siso_read_counter(c, 1, &total);
            if (rc != SISO_OK) return rc;
            n_pairs = (long)total;
            if (n_pairs <= cap) break;
            if (attempt == 1) return siso_fail(c, SISO_ENOMEM, "siso_cluster: %ld pairs above the threshold", n_pairs);
            cap = n_pairs;  // once more with room for all of them
        }
        if (n_pairs > 0) {
            h_pairs.resize((size_t)n_pairs * 2);
            CLUSTER_TRY(hipMemcpyAsync(h_pairs.data(), d_pairs.p, (size_t)n_pairs * 2 * sizeof(int), hipMemcpyDeviceToHost, st), "pairs to host");
            CLUSTER_TRY(hipStreamSynchronize(st), "siso_cluster: synchronize");
        }
        d_pairs.release();
    }

    // ---- the communities: a walk over the pairs on the host ------------------------------------------
    std::vector<int> label;
    std::vector<long> first;   // members of cluster k: member[first[k] .. first[k+1])
    std::vector<int> member;
    choose_communities(h_pairs.data(), n_pairs, n, min_size, label, first, member);
    std::vector<int>().swap(h_pairs);
    const long clusters = (long)first.size() - 1;
    if (clusters > c->capacity)
        return siso_fail(c, SISO_ECAPACITY, "siso_cluster: %ld clusters, capacity %ld", clusters, c->capacity);

    // ---- the repository: one row per cluster -----------------------------------------------------
    DeviceMem d_first, d_member;
    if (clusters > 0) {
        if (!d_first.alloc(first.size() * sizeof(long)) || !d_member.alloc(member.size() * sizeof(int))) {
            (void)hipGetLastError();
            return siso_fail(c, SISO_ENOMEM, "siso_cluster: member lists of %ld clusters", clusters);
        }
        CLUSTER_TRY(hipMemcpyAsync(d_first.p, first.data(), first.size() * sizeof(long), hipMemcpyHostToDevice, st), "member offsets");
        CLUSTER_TRY(hipMemcpyAsync(d_member.p, member.data(), member.size() * sizeof(int), hipMemcpyHostToDevice, st), "members");
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_cluster_rows<float>, dim3((unsigned)clusters), dim3(256), 0, st, d_rows.as<float>(),
                               d_inv.as<float>(), d_first.as<long>(), d_member.as<int>(), (float *)c->cent, c->mean, c->size,
                               c->invn, c->locality, c->access, out_representative, d);
        else
            hipLaunchKernelGGL(k_cluster_rows<bf16_t>, dim3((unsigned)clusters), dim3(256), 0, st, d_rows.as<bf16_t>(),
                               d_inv.as<float>(), d_first.as<long>(), d_member.as<int>(), (bf16_t *)c->cent, c->mean, c->size,
                               c->invn, c->locality, c->access, out_representative, d);
        CLUSTER_TRY(hipGetLastError(), "k_cluster_rows");
    }
    hipLaunchKernelGGL(k_nan_fill, dim3(1), dim3(SISO_PAD_ROWS), 0, st, c->invn + clusters, SISO_PAD_ROWS);
    CLUSTER_TRY(hipGetLastError(), "k_nan_fill");
    if (out_label && n > 0)
        CLUSTER_TRY(hipMemcpyAsync(out_label, label.data(), (size_t)n * sizeof(int), hipMemcpyHostToDevice, st), "labels");
    CLUSTER_TRY(hipStreamSynchronize(st), "siso_cluster: synchronize");
    c->count = clusters;
    if (out_stats) {
        out_stats[0] = n_pairs;
        out_stats[1] = (long)member.size();
    }
#undef CLUSTER_TRY
    return clusters;
}

extern "C" long siso_cluster(siso_cache *c, const void *vectors, long n, float theta_c, int min_size, int *out_label,
                             int *out_representative, long *out_stats) {
    if (!c) return SISO_EINVAL;
    if (c->dtype == SISO_FP8) return siso_fail(c, SISO_EINVAL, "siso_cluster: not available with the 8-bit storage");
    try {
        return cluster_impl(c, vectors, n, theta_c, min_size, out_label, out_representative, out_stats);
    } catch (const std::bad_alloc &) {  // the host lists; nothing has been changed yet when they are built
        return siso_fail(c, SISO_ENOMEM, "siso_cluster: host memory for the neighbour lists");
    }
}

// The host part of siso_cluster alone: pairs and labels are HOST arrays.
extern "C" long siso_choose_communities(const int *pairs, long n_pairs, long n, int min_size, int *out_label) {
    if (n < 0 || n_pairs < 0 || min_size < 1 || (n_pairs > 0 && !pairs) || (n > 0 && !out_label)) return SISO_EINVAL;
    for (long p = 0; p < 2 * n_pairs; ++p)
        if (pairs[p] < 0 || pairs[p] >= n) return SISO_EINVAL;
    for (long p = 0; p < n_pairs; ++p)
        if (pairs[2 * p] == pairs[2 * p + 1]) return SISO_EINVAL;
    try {
        std::vector<int> label, member;
        std::vector<long> first;
        choose_communities(pairs, n_pairs, n, min_size, label, first, member);
        for (long i = 0; i < n; ++i) out_label[i] = label[(size_t)i];
        return (long)first.size() - 1;
    } catch (const std::bad_alloc &) {
        return SISO_ENOMEM;
    }
}

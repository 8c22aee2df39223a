// The 8-bit storage variant of the cache (SISO_FP8): bf16 rows come in, every row is kept as one OCP E4M3 code
// per element and one scale per row (blocked scaling, the row being the block), lookups quantise the batch the
// same way and run the fused MFMA kernel over the codes.  The similarity is the cosine of the two stored
// vectors; the scales cancel in it, so the kernels only ever see codes and the inverse lengths of code rows.
//
// Quantisation of a row x, in single precision throughout (the outcome is a code, a decision both this library
// and anything that checks it must take alike):
//     amax = max |x_t|;  scale = amax / 448;  code_t = nearest E4M3 value of x_t / scale, ties to the even
//     mantissa, saturating at +-448 (E4M3: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals
//     m/8 * 2^-6, no infinities).
// A row without length: scale 0, all codes 0; a row holding a NaN or an infinity: scale NaN, inverse length NaN.
#include "siso_internal.h"

namespace {

// One 256-thread block per row: codes [row][d], scale [row] (may be NULL), inv [row] = 1 / |code row| (0 for
// a row without length, NaN for a non-finite one).  With `load`, the row is a centroid being loaded: its unit
// direction goes to nothing (the 8-bit cache keeps no running mean), its bookkeeping is set as siso_load does.
// With `rows` (siso_fp8_follow), block b handles row rows[b] of both sides, if `pick` is NULL or pick[b] != 0 and
// the row lies below `limit`; `counts` are then the sizes of all rows, not of the blocks, and only the size is kept.
__global__ __launch_bounds__(256) void k_fp8_quantize(const bf16_t *__restrict__ src, int d, unsigned char *codes, float *scale,
                                                       float *inv, const int *__restrict__ counts, int *size,
                                                       float *locality, unsigned *access,
                                                       const int *__restrict__ rows, const unsigned char *__restrict__ pick,
                                                       long limit) {
    __shared__ float sh[4];
    constexpr int E = SISO_MAX_DIM / 256;
    long r = blockIdx.x;
    if (rows) {
        if (pick && !pick[blockIdx.x]) return;
        r = rows[blockIdx.x];
        if (r < 0 || r >= limit) return;
    }
    const int t = threadIdx.x;
    float x[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int col = t + e * 256;
        x[e] = col < d ? bf16_to_f32(src[(size_t)r * d + col]) : 0.f;
    }
    fp8_store_row<E>(x, d, codes + (size_t)r * d, scale ? scale + r : nullptr, inv + r, sh);
    if (t == 0) {
        if (size) {
            const int s = counts ? counts[r] : 1;
            size[r] = s < 1 ? 1 : s;
            if (!rows) {
                locality[r] = (float)(s < 1 ? 1 : s);
                access[r] = 0;
            }
        }
    }
}

// the inverse lengths behind the last live row: NaN, so that no row of a partial tile can win
__global__ void k_pad_nan(float *p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = __uint_as_float(0x7FC00000u);
}

// to[k] += from[k], saturating at "infinity" (which stays); from[k] = 0
__global__ void k_hand_counts(unsigned *from, unsigned *to, long k) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= k) return;
    const unsigned a = from[i], b = to[i];
    from[i] = 0;
    if (a == 0 || b == SISO_ACCESS_INF) return;
    const u64 sum = (u64)a + (u64)b;
    to[i] = sum >= (u64)SISO_ACCESS_INF ? SISO_ACCESS_INF : (unsigned)sum;
}

}  // namespace

int siso_fp8_load(siso_cache *c, const void *centroids, const int *counts, long k) {
    if (k > 0) {
        hipLaunchKernelGGL(k_fp8_quantize, dim3((unsigned)k), dim3(256), 0, c->stream, (const bf16_t *)centroids, c->dim,
                           (unsigned char *)c->cent, c->scale, c->invn, counts, c->size, c->locality, c->access,
                           (const int *)nullptr, (const unsigned char *)nullptr, 0L);
        return siso_check_hip(c, hipGetLastError(), "k_fp8_quantize (load)");
    }
    return SISO_OK;
}

// Room for the codes and inverse lengths of a batch of n queries (grown on demand: synchronises and allocates then).
int siso_fp8_ensure_batch(siso_cache *c, long n) {
    if (n <= c->fp8_q_cap) return SISO_OK;
    if (c->fp8_q) {
        const int rc = siso_check_hip(c, hipStreamSynchronize(c->stream), "fp8 lookup: synchronize");
        if (rc != SISO_OK) return rc;
        (void)hipFree(c->fp8_q);
        (void)hipFree(c->fp8_qinv);
        c->fp8_q = nullptr;
        c->fp8_qinv = nullptr;
        c->fp8_q_cap = 0;
    }
    // whole tiles of 256 rows stay readable behind the batch (the kernels clamp their rows, this is slack)
    bool ok = hipMalloc((void **)&c->fp8_q, ((size_t)n + SISO_PAD_ROWS) * c->dim) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->fp8_qinv, (size_t)n * sizeof(float)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        if (c->fp8_q) (void)hipFree(c->fp8_q);
        c->fp8_q = nullptr;
        c->fp8_qinv = nullptr;
        return siso_fail(c, SISO_ENOMEM, "fp8 lookup: codes of %ld queries", n);
    }
    c->fp8_q_cap = n;
    return SISO_OK;
}

int siso_fp8_quantize_batch(siso_cache *c, const void *queries, long n) {
    hipLaunchKernelGGL(k_fp8_quantize, dim3((unsigned)n), dim3(256), 0, c->stream, (const bf16_t *)queries, c->dim,
                       (unsigned char *)c->fp8_q, (float *)nullptr, c->fp8_qinv, (const int *)nullptr, (int *)nullptr,
                       (float *)nullptr, (unsigned *)nullptr, (const int *)nullptr, (const unsigned char *)nullptr, 0L);
    return siso_check_hip(c, hipGetLastError(), "k_fp8_quantize (batch)");
}

extern "C" int siso_export_scales(siso_cache *c, float *scales) {
    if (!c) return SISO_EINVAL;
    if (c->dtype != SISO_FP8) return siso_fail(c, SISO_EINVAL, "siso_export_scales: the cache does not use the 8-bit storage");
    if (c->count == 0 || !scales) return SISO_OK;
    return siso_check_hip(c, hipMemcpyAsync(scales, c->scale, (size_t)c->count * sizeof(float), hipMemcpyDeviceToDevice, c->stream),
                          "siso_export_scales");
}

// An 8-bit cache as the serving copy of a bf16 cache that is updated online: the rows idx[i] (where hit is NULL
// or hit[i] != 0) are quantised again from the master's stored centroids, as siso_load would quantise them, and
// take the master's weights over.  Enqueued on the copy's stream.
extern "C" int siso_fp8_follow(siso_cache *copy, const siso_cache *master, const int *idx, const unsigned char *hit, long n) {
    if (!copy) return SISO_EINVAL;
    if (!master || n < 0 || (n > 0 && !idx)) return siso_fail(copy, SISO_EINVAL, "siso_fp8_follow: bad arguments");
    if (copy->dtype != SISO_FP8 || master->dtype != SISO_BF16 || copy->dim != master->dim)
        return siso_fail(copy, SISO_EINVAL, "siso_fp8_follow: an 8-bit cache follows a bf16 cache of the same dimension");
    if (copy->count != master->count)
        return siso_fail(copy, SISO_EINVAL, "siso_fp8_follow: the copy holds %ld centroids, the master %ld (load the copy again)",
                         copy->count, master->count);
    if (n == 0) return SISO_OK;
    if (n > 2147483647L) return siso_fail(copy, SISO_EINVAL, "siso_fp8_follow: batch of %ld is too large", n);
    hipLaunchKernelGGL(k_fp8_quantize, dim3((unsigned)n), dim3(256), 0, copy->stream, (const bf16_t *)master->cent, copy->dim,
                       (unsigned char *)copy->cent, copy->scale, copy->invn, (const int *)master->size, copy->size,
                       copy->locality, copy->access, idx, hit, copy->count);
    return siso_check_hip(copy, hipGetLastError(), "k_fp8_quantize (follow)");
}

static int fp8_pair_check(siso_cache *copy, const siso_cache *master, const char *who) {
    if (!master) return siso_fail(copy, SISO_EINVAL, "%s: bad arguments", who);
    if (copy->dtype != SISO_FP8 || master->dtype != SISO_BF16 || copy->dim != master->dim)
        return siso_fail(copy, SISO_EINVAL, "%s: an 8-bit cache follows a bf16 cache of the same dimension", who);
    return SISO_OK;
}

// The copy becomes the 8-bit image of the master as it stands (after a merge or a refresh, which renumber the rows):
// every live row quantised as siso_load would, sizes and cluster sizes taken over, reference counts started at zero.
extern "C" int siso_fp8_resync(siso_cache *copy, const siso_cache *master) {
    if (!copy) return SISO_EINVAL;
    int rc = fp8_pair_check(copy, master, "siso_fp8_resync");
    if (rc != SISO_OK) return rc;
    const long k = master->count;
    if (k > copy->capacity)
        return siso_fail(copy, SISO_ECAPACITY, "siso_fp8_resync: the master holds %ld centroids, the copy has room for %ld", k, copy->capacity);
    rc = siso_fp8_load(copy, master->cent, master->size, k);   // sizes, cluster size = size, references = 0
    if (rc != SISO_OK) return rc;
    if (k > 0) {
        rc = siso_check_hip(copy, hipMemcpyAsync(copy->locality, master->locality, (size_t)k * sizeof(float), hipMemcpyDeviceToDevice,
                                                 copy->stream), "siso_fp8_resync: cluster sizes");
        if (rc != SISO_OK) return rc;
    }
    hipLaunchKernelGGL(k_pad_nan, dim3(1), dim3(SISO_PAD_ROWS), 0, copy->stream, copy->invn + k, SISO_PAD_ROWS);
    rc = siso_check_hip(copy, hipGetLastError(), "k_pad_nan");
    if (rc != SISO_OK) return rc;
    copy->count = k;
    return SISO_OK;
}

// The references the copy's lookups have counted go to the master (Algorithm 1 filters by them), saturating at
// infinity; the copy starts counting at zero again.
extern "C" int siso_fp8_hand_counts(siso_cache *copy, siso_cache *master) {
    if (!copy) return SISO_EINVAL;
    const int rc = fp8_pair_check(copy, master, "siso_fp8_hand_counts");
    if (rc != SISO_OK) return rc;
    if (copy->count != master->count)
        return siso_fail(copy, SISO_EINVAL, "siso_fp8_hand_counts: the copy holds %ld centroids, the master %ld", copy->count,
                         master->count);
    const long k = copy->count;
    if (k == 0) return SISO_OK;
    hipLaunchKernelGGL(k_hand_counts, dim3((unsigned)((k + 255) / 256)), dim3(256), 0, copy->stream, copy->access, master->access, k);
    return siso_check_hip(copy, hipGetLastError(), "k_hand_counts");
}

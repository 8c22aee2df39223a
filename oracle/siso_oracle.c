/*
 * TEST INFRASTRUCTURE - NOT PART OF THE PRODUCT PATH.
 *
 * Brute-force, double-precision CPU oracle for the centroid-cache hot path:
 * batched exact lookup, centroid update, all-pairs self-similarity and group
 * merge.  It is written to be checked against the paper by eye: plain loops, no
 * blocking, no fusion, no reordering.  The only concession to run time is an
 * OpenMP "parallel for" over independent outer iterations (queries, rows),
 * which does not change any arithmetic.
 *
 * It shares no code with the GPU library, and only tests, the smoke check and
 * the benchmark's CPU-baseline leg may call it.
 *
 * What is computed, and where the paper defines it:
 *   - CosineSimilarity(a, b) = <a,b> / (|a| |b|): the similarity measure used
 *     throughout (section 3.1; Algorithm 1, MergeCentroids).
 *   - FindClosestCentroid(q, C) = the centroid of C with the largest cosine
 *     similarity to q (Algorithm 1, MergeCentroids; section 4.3 for the batched
 *     online search).  Ties go to the lowest index.
 *   - hit test: similarity strictly greater than the threshold (Algorithm 1
 *     uses ">"; section 3.1 "the similarity threshold for retrieval ... judges
 *     a cache hit").
 *   - a centroid is the average point of its group of vectors (section 3.1):
 *     the update keeps, per centroid, the exact mean m of its unit-length
 *     members and their number n, and stores normalize(m) rounded to the
 *     storage type.
 *   - merge: all pairs i<j of cached centroids whose cosine exceeds the
 *     clustering threshold (the comparison inside MergeCentroids, taken over
 *     all pairs); connected groups are replaced by their count-weighted mean,
 *     the cluster sizes add up (Algorithm 1, MergeCentroids, cluster_size).
 *
 *   - variants of the lookup: one lookup judged against several retrieval
 *     thresholds (the threshold is dynamic, section 3.3; the similarity does not
 *     depend on it), and the k closest centroids instead of the closest one.
 *
 * Readings where the paper is silent:
 *   - vectors are taken at storage precision (bf16 or fp32 widened exactly to
 *     double); similarities are true cosines of the stored values;
 *   - a zero-length vector has similarity 0 to everything; a query holding a
 *     NaN or infinity gets idx -1, sim NaN, no hit; an empty cache gives idx
 *     -1, sim -inf, no hit; a similarity that is NaN never wins;
 *   - the update is batch-synchronous and order-free: every centroid k receives
 *     the sum of the unit-normalised queries assigned to it in this call;
 *   - if an updated mean has zero length the stored centroid is left as it is.
 *
 * parity pins: see tests/test_oracle_*.py (hand-computed cosines, closed forms
 * for means, brute force through an independent numpy/float64 route, planted
 * duplicates and neighbours, threshold invariants, closed-form pair counts).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

typedef struct oracle_cache {
    int dim;
    long capacity;
    int dtype;
    long count;
    void *cent;     /* [capacity][dim] storage type, as loaded / as last rounded */
    double *mean;   /* [capacity][dim] mean of the unit-length members           */
    int *size;      /* [capacity] number of members: the weight of the mean      */
    float *locality;    /* [capacity] cluster_size of Algorithm 1 (decays by 1.1 per refresh: a float) */
    uint32_t *access;   /* [capacity] access_count of Algorithm 1; ORACLE_ACCESS_INF = infinity        */
} oracle_cache;

#define ORACLE_ACCESS_INF 0xFFFFFFFFu

/* ------------------------------------------------------------------ storage */
static size_t elem_size(int dtype) { return dtype == ORACLE_F32 ? 4 : 2; }

/* element e of a storage array, widened exactly */
static double widen(const void *base, int dtype, size_t e) {
    if (dtype == ORACLE_F32) return (double)((const float *)base)[e];
    uint32_t bits = (uint32_t)((const uint16_t *)base)[e] << 16;
    float f;
    memcpy(&f, &bits, 4);
    return (double)f;
}

/* double -> bf16 bit pattern with one round-to-nearest-even step */
static uint16_t round_bf16(double x) {
    if (isnan(x)) return 0x7FC0;
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (isinf(a)) return sign | 0x7F80;
    double r;
    if (a < ldexp(1.0, -126)) {
        /* subnormal range of bf16: spacing 2^-133 */
        r = ldexp(rint(ldexp(a, 133)), -133);
    } else {
        int e;
        double m = frexp(a, &e);            /* a = m * 2^e, m in [0.5, 1) */
        r = ldexp(rint(ldexp(m, 8)), e - 8); /* keep 8 significant bits    */
    }
    if (r >= ldexp(1.0, 128)) return sign | 0x7F80;
    float f = (float)r; /* exact: r has at most 8 significant bits */
    uint32_t bits;
    memcpy(&bits, &f, 4);
    return sign | (uint16_t)(bits >> 16);
}

static void store(void *base, int dtype, size_t e, double x) {
    if (dtype == ORACLE_F32) ((float *)base)[e] = (float)x; /* round-to-nearest-even */
    else ((uint16_t *)base)[e] = round_bf16(x);
}

/* ------------------------------------------------------------- fp8 storage */
/*
 * The 8-bit floating-point storage variant.  Format: OCP 8-bit floating point, E4M3
 * (1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits; exponent field 0 holds
 * the subnormals m/8 * 2^-6; no infinities; S.1111.111 is NaN; largest finite value
 * 448 = 0x7E).  A row is stored as one code per element plus one scale per row
 * (blocked scaling with the row as the block); its value is scale * decode(code).
 *
 * Quantisation of a row x (taken at its input precision), all in single precision
 * because the outcome is a code (an integer decision both sides must take alike):
 *     amax  = max_t |x_t|                   (exact)
 *     scale = amax / 448                    (one correctly rounded division)
 *     y_t   = x_t / scale                   (one correctly rounded division)
 *     code_t = y_t rounded to the nearest E4M3 value, ties to the even mantissa,
 *              values beyond 448 saturate to +-448
 * A row without length gets scale 0 and all codes 0; a row holding a NaN or an
 * infinity gets scale NaN (it can never be chosen).
 */
static double e4m3_decode(uint8_t code) {
    const int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7) return NAN;
    if (e == 0) v = ldexp((double)m / 8.0, -6);
    else v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* nearest E4M3 value of y (finite), ties to even, saturating */
static uint8_t e4m3_encode(float y) {
    const uint8_t sign = signbit(y) ? 0x80 : 0;
    const double a = fabs((double)y);
    if (a >= 448.0) return sign | 0x7E;
    /* spacing of the E4M3 values around a: 2^(e-3) for a in [2^e, 2^(e+1)), e >= -6; 2^-9 below 2^-6 */
    int e;
    (void)frexp(a, &e); /* a = f * 2^e, f in [0.5, 1): a in [2^(e-1), 2^e) */
    int step_exp = (a < ldexp(1.0, -6)) ? -9 : (e - 1) - 3;
    const double steps = rint(ldexp(a, -step_exp)); /* rint: round half to even; a / spacing is exact */
    const double r = ldexp(steps, step_exp);        /* the rounded value, <= 448 */
    if (r == 0.0) return sign;
    /* find its code: the values are ordered like their codes */
    for (int code = 1; code <= 0x7E; ++code)
        if (e4m3_decode((uint8_t)code) == r) return sign | (uint8_t)code;
    return sign | 0x7E; /* not reached */
}

/*
 * Quantise n rows of the input type (f32 or bf16) to codes [n][dim] and scales [n].
 */
int oracle_fp8_quantize(const void *rows, int dtype, long n, int dim, uint8_t *codes, float *scales) {
    if (n < 0 || dim <= 0 || (n > 0 && (!rows || !codes || !scales))) return -1;
    for (long i = 0; i < n; ++i) {
        float amax = 0.0f;
        int finite = 1;
        for (int t = 0; t < dim; ++t) {
            const float x = (float)widen(rows, dtype, (size_t)i * dim + t); /* exact: the inputs are f32 or bf16 */
            if (!isfinite(x)) finite = 0;
            if (fabsf(x) > amax) amax = fabsf(x);
        }
        if (!finite || amax == 0.0f) {
            scales[i] = finite ? 0.0f : NAN;
            memset(codes + (size_t)i * dim, 0, (size_t)dim);
            continue;
        }
        const float scale = amax / 448.0f;
        scales[i] = scale;
        for (int t = 0; t < dim; ++t) {
            const float x = (float)widen(rows, dtype, (size_t)i * dim + t);
            codes[(size_t)i * dim + t] = e4m3_encode(x / scale);
        }
    }
    return 0;
}

/*
 * Lookup over rows stored in the 8-bit format: the queries are quantised the same
 * way, row by row, and the similarity is the cosine of the two stored vectors,
 *     <scale_q decode(q8), scale_c decode(c8)> / (|.| |.|) = <decode(q8), decode(c8)> / (|decode(q8)| |decode(c8)|),
 * in double; top-1, lowest index on ties, strict threshold: as oracle_lookup_rows.
 * cent_codes [k][dim], cent_scales [k] (a NaN scale: the row is never chosen; scale 0: a
 * row without length, similarity 0); queries in their input type.
 */
int oracle_fp8_lookup_rows(const uint8_t *cent_codes, const float *cent_scales, long k, int dim, const void *queries,
                           int qdtype, long n, float threshold, int *out_idx, double *out_sim, unsigned char *out_hit,
                           double *out_second) {
    if (dim <= 0 || k < 0 || n < 0 || (n > 0 && (!queries || !out_idx || !out_sim)) || (k > 0 && (!cent_codes || !cent_scales)))
        return -1;
    uint8_t *q8 = (uint8_t *)malloc((size_t)(n > 0 ? n : 1) * dim);
    float *qs = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    double *cn = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    if (!q8 || !qs || !cn) { free(q8); free(qs); free(cn); return -2; }
    int rc = oracle_fp8_quantize(queries, qdtype, n, dim, q8, qs);
    for (long j = 0; j < k; ++j) {
        double s = 0.0;
        for (int t = 0; t < dim; ++t) {
            const double v = e4m3_decode(cent_codes[(size_t)j * dim + t]);
            s += v * v;
        }
        cn[j] = isnan(cent_scales[j]) ? NAN : sqrt(s);
    }
    const double theta = (double)threshold;
#pragma omp parallel for schedule(dynamic, 1)
    for (long i = 0; i < n; ++i) {
        if (rc != 0) continue;
        int best = -1;
        double best_s = -INFINITY, second = -INFINITY;
        if (isnan(qs[i])) {
            out_idx[i] = -1;
            out_sim[i] = NAN;
            if (out_hit) out_hit[i] = 0;
            if (out_second) out_second[i] = NAN;
            continue;
        }
        double qn = 0.0;
        for (int t = 0; t < dim; ++t) {
            const double v = e4m3_decode(q8[(size_t)i * dim + t]);
            qn += v * v;
        }
        qn = sqrt(qn);
        for (long j = 0; j < k; ++j) {
            double s = 0.0;
            if (isnan(cn[j])) continue;
            if (qn != 0.0 && cn[j] != 0.0) {
                for (int t = 0; t < dim; ++t)
                    s += e4m3_decode(q8[(size_t)i * dim + t]) * e4m3_decode(cent_codes[(size_t)j * dim + t]);
                s /= qn * cn[j];
            }
            if (s > best_s) { second = best_s; best_s = s; best = (int)j; }
            else if (s > second) second = s;
        }
        out_idx[i] = best;
        out_sim[i] = best_s;
        if (out_hit) out_hit[i] = (best >= 0 && best_s > theta) ? 1 : 0;
        if (out_second) out_second[i] = second;
    }
    free(q8); free(qs); free(cn);
    return rc;
}

/*
 * The k closest rows of an 8-bit store instead of the single closest one: the similarities of
 * oracle_fp8_lookup_rows (queries quantised like the rows, cosine of the two code vectors, in
 * double), ranked as oracle_lookup_topk ranks: larger similarity first, the lower index among
 * equal ones; a row with a NaN scale is never chosen; (-1, -inf) where fewer than k rows can be
 * chosen; (-1, NaN) throughout for a query holding a NaN or an infinity.
 */
int oracle_fp8_lookup_topk_rows(const uint8_t *cent_codes, const float *cent_scales, long k, int dim, const void *queries,
                                int qdtype, long n, int kk, int *out_idx, double *out_sim) {
    if (dim <= 0 || k < 0 || n < 0 || kk < 1 || (n > 0 && (!queries || !out_idx || !out_sim)) ||
        (k > 0 && (!cent_codes || !cent_scales)))
        return -1;
    uint8_t *q8 = (uint8_t *)malloc((size_t)(n > 0 ? n : 1) * dim);
    float *qs = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    double *cn = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    if (!q8 || !qs || !cn) { free(q8); free(qs); free(cn); return -2; }
    int rc = oracle_fp8_quantize(queries, qdtype, n, dim, q8, qs);
    for (long j = 0; j < k; ++j) {
        double s = 0.0;
        for (int t = 0; t < dim; ++t) {
            const double v = e4m3_decode(cent_codes[(size_t)j * dim + t]);
            s += v * v;
        }
        cn[j] = isnan(cent_scales[j]) ? NAN : sqrt(s);
    }
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long i = 0; i < n; ++i) {
        int *oi = out_idx + (size_t)i * kk;
        double *os = out_sim + (size_t)i * kk;
        if (rc != 0) continue;
        if (isnan(qs[i])) {
            for (int r = 0; r < kk; ++r) { oi[r] = -1; os[r] = NAN; }
            continue;
        }
        double *sim = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
        char *taken = (char *)calloc((size_t)(k > 0 ? k : 1), 1);
        if (!sim || !taken) { free(sim); free(taken); failed = 1; continue; }
        double qn = 0.0;
        for (int t = 0; t < dim; ++t) {
            const double v = e4m3_decode(q8[(size_t)i * dim + t]);
            qn += v * v;
        }
        qn = sqrt(qn);
        for (long j = 0; j < k; ++j) {
            double s = 0.0;
            if (isnan(cn[j])) { sim[j] = NAN; continue; }
            if (qn != 0.0 && cn[j] != 0.0) {
                for (int t = 0; t < dim; ++t)
                    s += e4m3_decode(q8[(size_t)i * dim + t]) * e4m3_decode(cent_codes[(size_t)j * dim + t]);
                s /= qn * cn[j];
            }
            sim[j] = s;
        }
        for (int r = 0; r < kk; ++r) {
            long best = -1;
            for (long j = 0; j < k; ++j) {
                if (taken[j] || isnan(sim[j])) continue;
                if (best < 0 || sim[j] > sim[best]) best = j; /* strict: the lowest index keeps a tie */
            }
            if (best < 0) { oi[r] = -1; os[r] = -INFINITY; continue; }
            taken[best] = 1;
            oi[r] = (int)best;
            os[r] = sim[best];
        }
        free(sim);
        free(taken);
    }
    free(q8); free(qs); free(cn);
    return failed ? -2 : rc;
}

/* ---------------------------------------------------------------- arithmetic */
static double row_norm(const void *base, int dtype, long row, int dim) {
    double s = 0.0;
    for (int t = 0; t < dim; ++t) {
        double v = widen(base, dtype, (size_t)row * dim + t);
        s += v * v;
    }
    return sqrt(s);
}

static int row_finite(const void *base, int dtype, long row, int dim) {
    for (int t = 0; t < dim; ++t)
        if (!isfinite(widen(base, dtype, (size_t)row * dim + t))) return 0;
    return 1;
}

/* CosineSimilarity of row ra of A and row rb of B, given their lengths */
static double cosine(const void *A, long ra, double na, const void *B, long rb, double nb,
                     int dtype, int dim) {
    if (na == 0.0 || nb == 0.0) return 0.0;
    double s = 0.0;
    for (int t = 0; t < dim; ++t)
        s += widen(A, dtype, (size_t)ra * dim + t) * widen(B, dtype, (size_t)rb * dim + t);
    return s / (na * nb);
}

/* ------------------------------------------------------------------- lookup */
/*
 * For every query: FindClosestCentroid over rows [0,k) of `centroids`, then the
 * strict threshold test.  out_second (nullable) receives the largest similarity
 * among the other centroids (-inf if there is none); tests use it for the top-2
 * gap.  All pointers are host pointers.
 */
int oracle_lookup_rows(const void *centroids, long k, int dim, int dtype, const void *queries, long n,
                       float threshold, int *out_idx, double *out_sim, unsigned char *out_hit,
                       double *out_second) {
    if (dim <= 0 || k < 0 || n < 0) return -1;
    if (n > 0 && (!queries || !out_idx || !out_sim)) return -1;
    if (k > 0 && !centroids) return -1;
    double *cn = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    if (!cn) return -2;
#pragma omp parallel for schedule(static)
    for (long j = 0; j < k; ++j) cn[j] = row_norm(centroids, dtype, j, dim);

    const double theta = (double)threshold;
#pragma omp parallel for schedule(dynamic, 1)
    for (long i = 0; i < n; ++i) {
        int best = -1;
        double best_s = -INFINITY, second = -INFINITY;
        if (!row_finite(queries, dtype, i, dim)) {
            out_idx[i] = -1;
            out_sim[i] = NAN;
            if (out_hit) out_hit[i] = 0;
            if (out_second) out_second[i] = NAN;
            continue;
        }
        double qn = row_norm(queries, dtype, i, dim);
        for (long j = 0; j < k; ++j) {
            double s = cosine(queries, i, qn, centroids, j, cn[j], dtype, dim);
            if (isnan(s)) continue;
            if (s > best_s) { /* strict: the lowest index keeps a tie */
                second = best_s;
                best_s = s;
                best = (int)j;
            } else if (s > second) {
                second = s;
            }
        }
        out_idx[i] = best;
        out_sim[i] = best_s;
        if (out_hit) out_hit[i] = (best >= 0 && best_s > theta) ? 1 : 0;
        if (out_second) out_second[i] = second;
    }
    free(cn);
    return 0;
}

/* -------------------------------------------------------------- cache object */
int oracle_create(int dim, long capacity, int dtype, oracle_cache **out) {
    if (!out || dim <= 0 || capacity <= 0 || (dtype != ORACLE_F32 && dtype != ORACLE_BF16)) return -1;
    oracle_cache *c = (oracle_cache *)calloc(1, sizeof(*c));
    if (!c) return -2;
    c->dim = dim;
    c->capacity = capacity;
    c->dtype = dtype;
    c->cent = calloc((size_t)capacity * dim, elem_size(dtype));
    c->mean = (double *)calloc((size_t)capacity * dim, sizeof(double));
    c->size = (int *)calloc((size_t)capacity, sizeof(int));
    c->locality = (float *)calloc((size_t)capacity, sizeof(float));
    c->access = (uint32_t *)calloc((size_t)capacity, sizeof(uint32_t));
    if (!c->cent || !c->mean || !c->size || !c->locality || !c->access) {
        free(c->cent); free(c->mean); free(c->size); free(c->locality); free(c->access); free(c);
        return -2;
    }
    *out = c;
    return 0;
}

void oracle_destroy(oracle_cache *c) {
    if (!c) return;
    free(c->cent); free(c->mean); free(c->size); free(c->locality); free(c->access); free(c);
}

long oracle_count(const oracle_cache *c) { return c ? c->count : -1; }

/*
 * Replace the cache contents by k rows.  The rows are stored as given (no
 * re-rounding); the running mean starts at the row scaled to unit length and
 * stands for counts[j] members (1 when counts is NULL).
 */
int oracle_load(oracle_cache *c, const void *centroids, const int *counts, long k) {
    if (!c || k < 0 || k > c->capacity || (k > 0 && !centroids)) return -1;
    if (counts)
        for (long j = 0; j < k; ++j)
            if (counts[j] < 1) return -1;
    memcpy(c->cent, centroids, (size_t)k * c->dim * elem_size(c->dtype));
    for (long j = 0; j < k; ++j) {
        double nrm = row_norm(c->cent, c->dtype, j, c->dim);
        for (int t = 0; t < c->dim; ++t) {
            double v = widen(c->cent, c->dtype, (size_t)j * c->dim + t);
            c->mean[(size_t)j * c->dim + t] = (nrm > 0.0 && isfinite(nrm)) ? v / nrm : 0.0;
        }
        c->size[j] = counts ? counts[j] : 1;
        c->locality[j] = (float)c->size[j];
        c->access[j] = 0;
    }
    c->count = k;
    return 0;
}

/*
 * Lookup in the cache.  Every hit is a reference to its centroid: access_count of
 * that centroid goes up by one (section 4.2, "Merge step"); infinity stays infinity.
 */
int oracle_lookup(oracle_cache *c, const void *queries, long n, float threshold, int *out_idx,
                  double *out_sim, unsigned char *out_hit, double *out_second) {
    if (!c) return -1;
    int rc = oracle_lookup_rows(c->cent, c->count, c->dim, c->dtype, queries, n, threshold, out_idx, out_sim,
                                out_hit, out_second);
    if (rc != 0) return rc;
    for (long i = 0; i < n; ++i)
        if (out_idx[i] >= 0 && out_sim[i] > (double)threshold && c->access[out_idx[i]] != ORACLE_ACCESS_INF)
            c->access[out_idx[i]] += 1;
    return 0;
}

/*
 * One lookup judged against m retrieval thresholds at once (the threshold is dynamic,
 * section 3.3; the similarity does not depend on it): out_hit[i * m + j] = 1 where the
 * top-1 similarity of query i exceeds thetas[j], strictly.  count_index = the position of
 * the threshold whose hits are references to their centroids (access_count goes up as in
 * oracle_lookup), or -1 if these are test lookups that count nothing.
 */
int oracle_lookup_multi(oracle_cache *c, const void *queries, long n, const float *thetas, int m, int count_index,
                        int *out_idx, double *out_sim, unsigned char *out_hit, double *out_second) {
    if (!c || m < 0 || count_index >= m || count_index < -1 || (m > 0 && (!thetas || !out_hit))) return -1;
    int rc = oracle_lookup_rows(c->cent, c->count, c->dim, c->dtype, queries, n, 0.0f, out_idx, out_sim, NULL,
                                out_second);
    if (rc != 0) return rc;
    for (long i = 0; i < n; ++i)
        for (int j = 0; j < m; ++j) {
            const int hit = out_idx[i] >= 0 && out_sim[i] > (double)thetas[j];
            out_hit[(size_t)i * m + j] = (unsigned char)hit;
            if (hit && j == count_index && c->access[out_idx[i]] != ORACLE_ACCESS_INF) c->access[out_idx[i]] += 1;
        }
    return 0;
}

/*
 * The k closest centroids of every query instead of the single closest one
 * (FindClosestCentroid of Algorithm 1 taken k times): out_idx[i * k + r], out_sim[i * k + r],
 * r = 0 .. k-1, hold the centroid with the (r+1)-th largest cosine similarity to query i and
 * that similarity; among equal similarities the lower index comes first.  A similarity that
 * is NaN is never chosen; when fewer than k centroids can be chosen the remaining entries
 * are (-1, -inf); a query holding a NaN or an infinity gets (-1, NaN) throughout.
 */
int oracle_lookup_topk(const oracle_cache *c, const void *queries, long n, int k, int *out_idx, double *out_sim) {
    if (!c || n < 0 || k < 1 || (n > 0 && (!queries || !out_idx || !out_sim))) return -1;
    const long K = c->count;
    const int d = c->dim, dt = c->dtype;
    double *cn = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
    if (!cn) return -2;
    for (long j = 0; j < K; ++j) cn[j] = row_norm(c->cent, dt, j, d);
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (long i = 0; i < n; ++i) {
        int *oi = out_idx + (size_t)i * k;
        double *os = out_sim + (size_t)i * k;
        if (!row_finite(queries, dt, i, d)) {
            for (int r = 0; r < k; ++r) { oi[r] = -1; os[r] = NAN; }
            continue;
        }
        double *sim = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
        char *taken = (char *)calloc((size_t)(K > 0 ? K : 1), 1);
        if (!sim || !taken) { free(sim); free(taken); failed = 1; continue; }
        const double qn = row_norm(queries, dt, i, d);
        for (long j = 0; j < K; ++j) sim[j] = cosine(queries, i, qn, c->cent, j, cn[j], dt, d);
        for (int r = 0; r < k; ++r) {
            long best = -1;
            for (long j = 0; j < K; ++j) {
                if (taken[j] || isnan(sim[j])) continue;
                if (best < 0 || sim[j] > sim[best]) best = j; /* strict: the lowest index keeps a tie */
            }
            if (best < 0) { oi[r] = -1; os[r] = -INFINITY; continue; }
            taken[best] = 1;
            oi[r] = (int)best;
            os[r] = sim[best];
        }
        free(sim);
        free(taken);
    }
    free(cn);
    return failed ? -2 : 0;
}

/*
 * Fold query i into centroid idx[i] (idx[i] < 0: skip).  Members are the
 * unit-normalised queries; zero-length and non-finite queries are skipped.
 *   m_k <- (n_k m_k + sum of members) / (n_k + #members),  n_k += #members,
 *   c_k <- round_storage(m_k / |m_k|)        (left alone when |m_k| = 0)
 * Every centroid sees all of its members of this call at once, so the result
 * does not depend on the order of the queries.
 */
int oracle_update(oracle_cache *c, const void *queries, const int *idx, long n) {
    if (!c || n < 0 || (n > 0 && (!queries || !idx))) return -1;
    for (long i = 0; i < n; ++i)
        if (idx[i] >= c->count) return -1;
    const int d = c->dim;
    double *sum = (double *)malloc(sizeof(double) * d);
    char *done = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    if (!sum || !done) { free(sum); free(done); return -2; }
    for (long i = 0; i < n; ++i) {
        if (idx[i] < 0 || done[i]) continue;
        const long k = idx[i];
        long members = 0;
        for (int t = 0; t < d; ++t) sum[t] = 0.0;
        for (long j = i; j < n; ++j) {
            if (idx[j] != k) continue;
            done[j] = 1;
            if (!row_finite(queries, c->dtype, j, d)) continue;
            double qn = row_norm(queries, c->dtype, j, d);
            if (qn == 0.0) continue;
            for (int t = 0; t < d; ++t) sum[t] += widen(queries, c->dtype, (size_t)j * d + t) / qn;
            ++members;
        }
        if (members == 0) continue;
        double *m = c->mean + (size_t)k * d;
        const double n_old = (double)c->size[k], n_new = n_old + (double)members;
        double sq = 0.0;
        for (int t = 0; t < d; ++t) {
            m[t] = (n_old * m[t] + sum[t]) / n_new;
            sq += m[t] * m[t];
        }
        c->size[k] += (int)members;
        double nrm = sqrt(sq);
        if (nrm > 0.0)
            for (int t = 0; t < d; ++t) store(c->cent, c->dtype, (size_t)k * d + t, m[t] / nrm);
    }
    free(sum);
    free(done);
    return 0;
}

/* ------------------------------------------------------------------- merge */
/*
 * All pairs i<j of cached centroids with CosineSimilarity > threshold, written
 * in lexicographic order as (i,j) int pairs.  Returns the total number of such
 * pairs; only the first `cap` are written.
 */
long oracle_merge(const oracle_cache *c, float threshold, int *out_pairs, long cap) {
    if (!c || cap < 0 || (cap > 0 && !out_pairs)) return -1;
    const long k = c->count;
    const double theta = (double)threshold;
    double *cn = (double *)malloc(sizeof(double) * (size_t)(k > 0 ? k : 1));
    int **rows = (int **)calloc((size_t)(k > 0 ? k : 1), sizeof(int *));
    long *cnt = (long *)calloc((size_t)(k > 0 ? k : 1), sizeof(long));
    if (!cn || !rows || !cnt) { free(cn); free(rows); free(cnt); return -2; }
    for (long i = 0; i < k; ++i) cn[i] = row_norm(c->cent, c->dtype, i, c->dim);
#pragma omp parallel for schedule(dynamic, 8)
    for (long i = 0; i < k; ++i) {
        long have = 0, room = 0;
        int *list = NULL;
        for (long j = i + 1; j < k; ++j) {
            double s = cosine(c->cent, i, cn[i], c->cent, j, cn[j], c->dtype, c->dim);
            if (s > theta) {
                if (have == room) {
                    room = room ? 2 * room : 8;
                    list = (int *)realloc(list, sizeof(int) * (size_t)room);
                }
                list[have++] = (int)j;
            }
        }
        rows[i] = list;
        cnt[i] = have;
    }
    long total = 0;
    for (long i = 0; i < k; ++i) {
        for (long h = 0; h < cnt[i]; ++h, ++total) {
            if (total < cap) {
                out_pairs[2 * total] = (int)i;
                out_pairs[2 * total + 1] = rows[i][h];
            }
        }
        free(rows[i]);
    }
    free(cn); free(rows); free(cnt);
    return total;
}

static long uf_find(long *parent, long x) {
    while (parent[x] != x) x = parent[x];
    return x;
}

/*
 * Merge the connected groups of the pair graph.  The survivor of a group is its
 * lowest index; it receives
 *   m_g = sum_i n_i m_i / sum_i n_i,  n_g = sum_i n_i,  c_g = round_storage(m_g/|m_g|)
 * (c_g keeps the survivor's stored row when |m_g| = 0); rows outside any pair
 * are untouched.  Survivors are then packed to the front in their old order.
 * out_survivor (nullable, [old count]) gets the new index of each old row's
 * group.
 */
int oracle_merge_apply(oracle_cache *c, const int *pairs, long n_pairs, int *out_survivor) {
    if (!c || n_pairs < 0 || (n_pairs > 0 && !pairs)) return -1;
    const long k = c->count;
    const int d = c->dim;
    for (long p = 0; p < n_pairs; ++p) {
        int a = pairs[2 * p], b = pairs[2 * p + 1];
        if (a < 0 || b < 0 || a >= k || b >= k || a == b) return -1;
    }
    long *parent = (long *)malloc(sizeof(long) * (size_t)(k > 0 ? k : 1));
    long *newpos = (long *)malloc(sizeof(long) * (size_t)(k > 0 ? k : 1));
    double *acc = (double *)malloc(sizeof(double) * d);
    if (!parent || !newpos || !acc) { free(parent); free(newpos); free(acc); return -2; }
    for (long i = 0; i < k; ++i) parent[i] = i;
    for (long p = 0; p < n_pairs; ++p) {
        long ra = uf_find(parent, pairs[2 * p]), rb = uf_find(parent, pairs[2 * p + 1]);
        if (ra < rb) parent[rb] = ra;       /* the lower index becomes the root */
        else if (rb < ra) parent[ra] = rb;
    }
    for (long r = 0; r < k; ++r) {
        if (uf_find(parent, r) != r) continue;
        long members = 0;
        double wsum = 0.0;
        float loc = 0.0f;      /* cluster sizes add up, in ascending order of the members */
        uint64_t refs = 0;     /* so do the access counts, saturating at infinity          */
        for (int t = 0; t < d; ++t) acc[t] = 0.0;
        for (long i = r; i < k; ++i) {
            if (uf_find(parent, i) != r) continue;
            ++members;
            loc = loc + c->locality[i];
            refs += c->access[i];
            wsum += (double)c->size[i];
            for (int t = 0; t < d; ++t) acc[t] += (double)c->size[i] * c->mean[(size_t)i * d + t];
        }
        if (members == 1) continue;
        c->locality[r] = loc;
        c->access[r] = refs >= ORACLE_ACCESS_INF ? ORACLE_ACCESS_INF : (uint32_t)refs;
        double sq = 0.0;
        for (int t = 0; t < d; ++t) {
            c->mean[(size_t)r * d + t] = acc[t] / wsum;
            sq += c->mean[(size_t)r * d + t] * c->mean[(size_t)r * d + t];
        }
        c->size[r] = (int)wsum;
        double nrm = sqrt(sq);
        if (nrm > 0.0)
            for (int t = 0; t < d; ++t) store(c->cent, c->dtype, (size_t)r * d + t, c->mean[(size_t)r * d + t] / nrm);
    }
    long live = 0;
    const size_t rowb = (size_t)d * elem_size(c->dtype);
    for (long i = 0; i < k; ++i) {
        if (uf_find(parent, i) != i) continue;
        newpos[i] = live;
        if (live != i) {
            memmove((char *)c->cent + (size_t)live * rowb, (char *)c->cent + (size_t)i * rowb, rowb);
            memmove(c->mean + (size_t)live * d, c->mean + (size_t)i * d, sizeof(double) * d);
            c->size[live] = c->size[i];
            c->locality[live] = c->locality[i];
            c->access[live] = c->access[i];
        }
        ++live;
    }
    if (out_survivor)
        for (long i = 0; i < k; ++i) out_survivor[i] = (int)newpos[uf_find(parent, i)];
    c->count = live;
    free(parent); free(newpos); free(acc);
    return 0;
}

/* Copy out the live rows: stored centroids, means (double), sizes.  Any pointer may be NULL. */
int oracle_export(const oracle_cache *c, void *centroids, double *means, int *sizes) {
    if (!c) return -1;
    const size_t cells = (size_t)c->count * c->dim;
    if (centroids) memcpy(centroids, c->cent, cells * elem_size(c->dtype));
    if (means) memcpy(means, c->mean, cells * sizeof(double));
    if (sizes) memcpy(sizes, c->size, (size_t)c->count * sizeof(int));
    return 0;
}

/*
 * Take over a snapshot of k rows as it is (the counterpart of oracle_export and
 * oracle_export_meta; no arithmetic): stored centroids in the storage type, means,
 * sizes (>= 1), cluster_size and access_count (each of the last two may be NULL:
 * cluster_size = size, access_count = 0).
 */
int oracle_import(oracle_cache *c, const void *centroids, const double *means, const int *sizes,
                  const float *locality, const uint32_t *access, long k) {
    if (!c || k < 0 || k > c->capacity || (k > 0 && (!centroids || !means || !sizes))) return -1;
    for (long j = 0; j < k; ++j)
        if (sizes[j] < 1) return -1;
    const size_t cells = (size_t)k * c->dim;
    memcpy(c->cent, centroids, cells * elem_size(c->dtype));
    memcpy(c->mean, means, cells * sizeof(double));
    memcpy(c->size, sizes, (size_t)k * sizeof(int));
    for (long j = 0; j < k; ++j) {
        c->locality[j] = locality ? locality[j] : (float)sizes[j];
        c->access[j] = access ? access[j] : 0;
    }
    c->count = k;
    return 0;
}

/* Copy out cluster_size (float) and access_count (infinity = 0xFFFFFFFF) of the live rows. */
int oracle_export_meta(const oracle_cache *c, float *locality, uint32_t *access) {
    if (!c) return -1;
    if (locality) memcpy(locality, c->locality, (size_t)c->count * sizeof(float));
    if (access) memcpy(access, c->access, (size_t)c->count * sizeof(uint32_t));
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Cache replacement: Algorithm 1 (SISO-CacheManager), section 4.2            */
/* ------------------------------------------------------------------------ */

/*
 * Refresh the cache from r repository centroids (rows `repo`, cluster sizes
 * `repo_size`), clustering threshold theta_c, at most max_centroids survivors.
 *
 * MergeCentroids: C_new starts as the cache; the repository centroids are taken
 * in order; each looks for its closest centroid in C_new as it stands then (lowest
 * index among equals; the cache rows come first, added rows follow in the order
 * they were added).  If the cosine exceeds theta_c its cluster size is added to
 * that centroid's; otherwise it joins C_new with access_count = infinity.
 * FilteringCentroids: while C_new has more than max_centroids rows, the row with
 * the smallest (cluster_size, access_count) goes, the first such row in the order
 * of C_new; then every cluster size is divided by 1.1 and every access count reset.
 * UpdateCentroids: C_new becomes the cache (survivors keep their order).
 *
 * cluster_size is single precision here as on the GPU (additions in the order of
 * the repository, one division by 1.1f), because it decides who is evicted.
 * A row that joins starts a mean at its own direction with weight
 * max(1, round(repo_size)).  stats (nullable) = {merged, added, evicted};
 * min_margin (nullable) = the smallest |cosine - theta_c| met in a decision.
 */
int oracle_refresh_gap(oracle_cache *c, const void *repo, const float *repo_size, long r, float theta_c,
                       long max_centroids, long *stats, double *min_margin, double *min_gap);

int oracle_refresh(oracle_cache *c, const void *repo, const float *repo_size, long r, float theta_c,
                   long max_centroids, long *stats, double *min_margin) {
    return oracle_refresh_gap(c, repo, repo_size, r, theta_c, max_centroids, stats, min_margin, NULL);
}

/*
 * The same, and (min_gap, nullable) how close FindClosestCentroid came to a different answer: the smallest
 * difference between the closest and the second-closest cosine over the repository rows that were merged
 * (a row that is not merged joins C_new whichever centroid was closest).  Exactly equal cosines (equal rows:
 * the lowest index wins on both sides) do not count.  A diagnostic for the parity tests; nothing else changes.
 */
int oracle_refresh_gap(oracle_cache *c, const void *repo, const float *repo_size, long r, float theta_c,
                       long max_centroids, long *stats, double *min_margin, double *min_gap) {
    if (!c || r < 0 || max_centroids < 1 || max_centroids > c->capacity || (r > 0 && (!repo || !repo_size))) return -1;
    const int d = c->dim, dt = c->dtype;
    for (long i = 0; i < r; ++i)
        if (!row_finite(repo, dt, i, d) || !(repo_size[i] > 0.0f) || !isfinite(repo_size[i])) return -1;
    const long k0 = c->count, cap = k0 + r;
    const size_t rowb = (size_t)d * elem_size(dt);
    /* C_new, with room for every repository row */
    char *cent = (char *)malloc((size_t)(cap > 0 ? cap : 1) * rowb);
    double *mean = (double *)malloc((size_t)(cap > 0 ? cap : 1) * d * sizeof(double));
    double *norm = (double *)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(double));
    int *size = (int *)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(int));
    float *loc = (float *)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(float));
    uint32_t *acc = (uint32_t *)malloc((size_t)(cap > 0 ? cap : 1) * sizeof(uint32_t));
    if (!cent || !mean || !norm || !size || !loc || !acc) {
        free(cent); free(mean); free(norm); free(size); free(loc); free(acc);
        return -2;
    }
    memcpy(cent, c->cent, (size_t)k0 * rowb);
    memcpy(mean, c->mean, (size_t)k0 * d * sizeof(double));
    memcpy(size, c->size, (size_t)k0 * sizeof(int));
    memcpy(loc, c->locality, (size_t)k0 * sizeof(float));
    memcpy(acc, c->access, (size_t)k0 * sizeof(uint32_t));
    for (long j = 0; j < k0; ++j) norm[j] = row_norm(cent, dt, j, d);
    long cnt = k0, merged = 0, added = 0, evicted = 0;
    double margin = INFINITY, gap = INFINITY;

    /* merge step */
    for (long i = 0; i < r; ++i) {
        const double ni = row_norm(repo, dt, i, d);
        long best = -1;
        double bsim = -INFINITY;
#ifdef _OPENMP
#pragma omp parallel
#endif
        {
            long lbest = -1;
            double lsim = -INFINITY;
#ifdef _OPENMP
#pragma omp for nowait schedule(static)
#endif
            for (long j = 0; j < cnt; ++j) {
                double sj = cosine(repo, i, ni, cent, j, norm[j], dt, d);
                if (sj > lsim) { lsim = sj; lbest = j; }   /* ascending j: the lowest index keeps a tie */
            }
#ifdef _OPENMP
#pragma omp critical
#endif
            if (lbest >= 0 && (lsim > bsim || (lsim == bsim && lbest < best))) { bsim = lsim; best = lbest; }
        }
        if (best >= 0 && fabs(bsim - (double)theta_c) < margin) margin = fabs(bsim - (double)theta_c);
        if (best >= 0 && bsim > (double)theta_c) {
            if (min_gap)
                for (long j = 0; j < cnt; ++j) {
                    if (j == best) continue;
                    const double sj = cosine(repo, i, ni, cent, j, norm[j], dt, d);
                    if (sj != bsim && bsim - sj < gap) gap = bsim - sj;
                }
            loc[best] = loc[best] + repo_size[i];
            ++merged;
        } else {
            memcpy(cent + (size_t)cnt * rowb, (const char *)repo + (size_t)i * rowb, rowb);
            norm[cnt] = ni;
            for (int t = 0; t < d; ++t)
                mean[(size_t)cnt * d + t] = ni > 0.0 ? widen(repo, dt, (size_t)i * d + t) / ni : 0.0;
            long w = lrintf(repo_size[i]);
            size[cnt] = w < 1 ? 1 : (w > 2147483647L ? 2147483647 : (int)w);
            loc[cnt] = repo_size[i];
            acc[cnt] = ORACLE_ACCESS_INF;
            ++cnt;
            ++added;
        }
    }

    /* filtering step */
    while (cnt > max_centroids) {
        long victim = 0;
        for (long j = 1; j < cnt; ++j)
            if (loc[j] < loc[victim] || (loc[j] == loc[victim] && acc[j] < acc[victim])) victim = j;
        memmove(cent + (size_t)victim * rowb, cent + (size_t)(victim + 1) * rowb, (size_t)(cnt - victim - 1) * rowb);
        memmove(mean + (size_t)victim * d, mean + (size_t)(victim + 1) * d, (size_t)(cnt - victim - 1) * d * sizeof(double));
        memmove(size + victim, size + victim + 1, (size_t)(cnt - victim - 1) * sizeof(int));
        memmove(loc + victim, loc + victim + 1, (size_t)(cnt - victim - 1) * sizeof(float));
        memmove(acc + victim, acc + victim + 1, (size_t)(cnt - victim - 1) * sizeof(uint32_t));
        --cnt;
        ++evicted;
    }
    for (long j = 0; j < cnt; ++j) {
        loc[j] = loc[j] / 1.1f;
        acc[j] = 0;
    }

    /* update step */
    memcpy(c->cent, cent, (size_t)cnt * rowb);
    memcpy(c->mean, mean, (size_t)cnt * d * sizeof(double));
    memcpy(c->size, size, (size_t)cnt * sizeof(int));
    memcpy(c->locality, loc, (size_t)cnt * sizeof(float));
    memcpy(c->access, acc, (size_t)cnt * sizeof(uint32_t));
    c->count = cnt;
    if (stats) { stats[0] = merged; stats[1] = added; stats[2] = evicted; }
    if (min_margin) *min_margin = margin;
    if (min_gap) *min_gap = gap;
    free(cent); free(mean); free(norm); free(size); free(loc); free(acc);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Threshold-to-hit-ratio table and SLO-aware threshold choice (section 4.3,  */
/* "Adjusting theta_R to meet SLO", equations 1 and 2)                         */
/* ------------------------------------------------------------------------ */

/*
 * T2H table: out_hits[j] = number of sample queries that hit the cache at the
 * retrieval threshold thetas[j], i.e. whose top-1 cosine similarity exceeds it
 * (strictly; the threshold is a float widened to double, as in oracle_lookup).
 * The hit ratio h(theta_j) is out_hits[j] / n.
 */
int oracle_t2h(const oracle_cache *c, const void *queries, long n, const float *thetas, int m, long *out_hits) {
    if (!c || n < 0 || m < 0 || (m > 0 && (!thetas || !out_hits)) || (n > 0 && !queries)) return -1;
    for (int j = 0; j < m; ++j) out_hits[j] = 0;
    if (n == 0 || m == 0) return 0;
    int *idx = (int *)malloc((size_t)n * sizeof(int));
    double *sim = (double *)malloc((size_t)n * sizeof(double));
    if (!idx || !sim) {
        free(idx);
        free(sim);
        return -4;
    }
    /* test lookups: they are no references to the centroids, access_count stays */
    int rc = oracle_lookup_rows(c->cent, c->count, c->dim, c->dtype, queries, n, 0.0f, idx, sim, NULL, NULL);
    if (rc == 0) {
        for (long i = 0; i < n; ++i)
            for (int j = 0; j < m; ++j)
                if (sim[i] > (double)thetas[j]) out_hits[j] += 1; /* NaN and -inf never hit */
    }
    free(idx);
    free(sim);
    return rc;
}

/*
 * Expected waiting time of the LLM system seen as an M/D/1 queue (equation 2):
 *   E = L (1 - h),  W = E + lambda E^2 / (2 (1 - lambda E)),
 * L = average serving time of the LLM, lambda = arrival rate, h = hit ratio.
 * The queue is unstable for lambda E >= 1: W = +infinity.
 */
double oracle_md1_wait(double L, double lambda, double h) {
    const double E = L * (1.0 - h);
    const double rho = lambda * E;
    if (!(rho < 1.0)) return INFINITY;
    return E + lambda * E * E / (2.0 * (1.0 - rho));
}

/*
 * The highest threshold of the table whose expected waiting time stays below the
 * SLO latency S (S > W, strictly).  Returns its position in thetas, or -1 if no
 * entry satisfies the SLO.  The table may be in any order.
 */
int oracle_pick_threshold(const float *thetas, const double *hit_ratio, int m, double L, double lambda, double slo) {
    int best = -1;
    for (int j = 0; j < m; ++j) {
        const double W = oracle_md1_wait(L, lambda, hit_ratio[j]);
        if (slo > W && (best < 0 || thetas[j] > thetas[best])) best = j;
    }
    return best;
}

/*
 * Correction when the measured waiting time W' is off the estimate W by more
 * than 10 %: if W' is longer, move to the next lower threshold of the table
 * (more hits, less traffic to the LLM); if it is shorter, to the next higher
 * one.  At the end of the table, or within 10 %, the position stays.
 */
int oracle_adjust_threshold(const float *thetas, int m, int index, double w_est, double w_actual) {
    if (index < 0 || index >= m) return index;
    int want_lower;
    if (w_actual > 1.1 * w_est) want_lower = 1;
    else if (w_actual < 0.9 * w_est) want_lower = 0;
    else return index;
    int next = -1;
    for (int j = 0; j < m; ++j) {
        if (want_lower) {
            if (thetas[j] < thetas[index] && (next < 0 || thetas[j] > thetas[next])) next = j;
        } else {
            if (thetas[j] > thetas[index] && (next < 0 || thetas[j] < thetas[next])) next = j;
        }
    }
    return next < 0 ? index : next;
}

/* ------------------------------------------------------------------------ */
/* Clustering of the query log into the centroid repository (section 4.1)    */
/* ------------------------------------------------------------------------ */

/*
 * Community detection at the clustering threshold theta_c ("Selecting a
 * clustering algorithm"), followed by "Keeping centroids in a repository": every
 * cluster gets an id, its centroid (the average of its members, section 3.1)
 * and cluster_size (the number of its members).  The paper names the algorithm
 * and its threshold and cites it; the steps below are that published greedy
 * scheme (a reading: the paper itself prints no steps):
 *   1. two vectors are neighbours when their cosine exceeds theta_c (strictly,
 *      as every threshold test of the paper);
 *   2. the candidate community of vector i is i together with its neighbours;
 *      candidates with fewer than min_size vectors are dropped;
 *   3. the candidates are taken by size, largest first, equal sizes by index;
 *   4. of a candidate the vectors not yet in a cluster remain (i itself may be
 *      gone already); if at least min_size remain they become the next cluster
 *      (ids count up from 0 in this order), otherwise the candidate is dropped;
 *   5. vectors that end in no cluster get label -1.
 * Then the cache `c` is replaced by the clusters: row id = cluster id, mean =
 * average of the unit-length members, size = cluster_size = their number,
 * stored centroid = mean / |mean| rounded to the storage type (a zero row if the
 * mean has no length), access_count 0.
 *
 * The repository also names, per cluster, the input query closest to the centroid
 * (its output text stands for the cluster, "Keeping centroids in a repository"):
 * out_rep [clusters] = the member with the largest cosine to the mean, the lowest
 * index among equals; out_rep_gap [clusters] = that cosine minus the second
 * largest (infinity for a cluster of one).
 *
 * out_label [n], out_seed [number of clusters] (the vector whose candidate
 * formed the cluster; room for n), out_rep, out_rep_gap (room for n each) and
 * min_margin (the smallest |cosine - theta_c| over all pairs) may each be NULL.  Returns the number of clusters;
 * -1 bad arguments or a vector that is not finite or has no length; -2 out of
 * memory; -3 more clusters than the capacity of c (nothing changed then).
 */
long oracle_cluster(oracle_cache *c, const void *vectors, long n, float theta_c, int min_size,
                    int *out_label, int *out_seed, int *out_rep, double *out_rep_gap, double *min_margin) {
    if (!c || n < 0 || min_size < 1 || (n > 0 && !vectors)) return -1;
    const int d = c->dim, dt = c->dtype;
    const long n1 = n > 0 ? n : 1;
    double *norm = (double *)malloc((size_t)n1 * sizeof(double));
    unsigned char *adj = (unsigned char *)calloc((size_t)n1 * (size_t)n1, 1); /* adj[i*n+j] = neighbours */
    long *size = (long *)calloc((size_t)n1, sizeof(long));
    int *label = (int *)malloc((size_t)n1 * sizeof(int));
    int *seed = (int *)malloc((size_t)n1 * sizeof(int));
    if (!norm || !adj || !size || !label || !seed) {
        free(norm); free(adj); free(size); free(label); free(seed);
        return -2;
    }
    long rc = 0;
    for (long i = 0; i < n; ++i) {
        norm[i] = row_finite(vectors, dt, i, d) ? row_norm(vectors, dt, i, d) : 0.0;
        if (!(norm[i] > 0.0) || !isfinite(norm[i])) rc = -1;
    }
    double margin = INFINITY;
    if (rc == 0) {
        /* step 1: the neighbour relation */
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 8) reduction(min : margin)
#endif
        for (long i = 0; i < n; ++i)
            for (long j = i + 1; j < n; ++j) {
                const double s = cosine(vectors, i, norm[i], vectors, j, norm[j], dt, d);
                if (s > (double)theta_c) adj[(size_t)i * n + j] = adj[(size_t)j * n + i] = 1;
                const double g = fabs(s - (double)theta_c);
                if (g < margin) margin = g;
            }
        /* step 2: candidate sizes */
        for (long i = 0; i < n; ++i) {
            size[i] = 1;
            for (long j = 0; j < n; ++j) size[i] += adj[(size_t)i * n + j];
            label[i] = -1;
        }
        /* steps 3 and 4: largest candidate first, equal sizes in index order */
        long clusters = 0;
        for (long s = n; s >= (long)min_size; --s)
            for (long i = 0; i < n; ++i) {
                if (size[i] != s) continue;
                long left = label[i] < 0 ? 1 : 0;
                for (long j = 0; j < n; ++j)
                    if (adj[(size_t)i * n + j] && label[j] < 0) ++left;
                if (left < (long)min_size) continue;
                if (label[i] < 0) label[i] = (int)clusters;
                for (long j = 0; j < n; ++j)
                    if (adj[(size_t)i * n + j] && label[j] < 0) label[j] = (int)clusters;
                seed[clusters++] = (int)i;
            }
        rc = clusters;
        if (clusters > c->capacity) rc = -3;
    }
    if (rc >= 0) {
        /* the repository: centroid = average of the members, cluster_size = their number */
        const long clusters = rc;
        for (long k = 0; k < clusters; ++k) {
            double *m = c->mean + (size_t)k * d;
            long members = 0;
            for (int t = 0; t < d; ++t) m[t] = 0.0;
            for (long i = 0; i < n; ++i) {
                if (label[i] != (int)k) continue;
                for (int t = 0; t < d; ++t) m[t] += widen(vectors, dt, (size_t)i * d + t) / norm[i];
                ++members;
            }
            double sq = 0.0;
            for (int t = 0; t < d; ++t) {
                m[t] /= (double)members;
                sq += m[t] * m[t];
            }
            const double len = sqrt(sq);
            for (int t = 0; t < d; ++t) store(c->cent, dt, (size_t)k * d + t, len > 0.0 ? m[t] / len : 0.0);
            /* the member closest to the centroid: cosine(x_i, m) = <x_i, m> / (|x_i| |m|) */
            long rep = -1;
            double best = -INFINITY, second = -INFINITY;
            for (long i = 0; i < n; ++i) {
                if (label[i] != (int)k) continue;
                double dot = 0.0;
                for (int t = 0; t < d; ++t) dot += widen(vectors, dt, (size_t)i * d + t) * m[t];
                const double cs = len > 0.0 ? dot / (norm[i] * len) : 0.0;
                if (cs > best) { second = best; best = cs; rep = i; }   /* ascending i: the lowest index keeps a tie */
                else if (cs > second) second = cs;
            }
            if (out_rep) out_rep[k] = (int)rep;
            if (out_rep_gap) out_rep_gap[k] = best - second;
            c->size[k] = (int)members;
            c->locality[k] = (float)members;
            c->access[k] = 0;
        }
        c->count = clusters;
        if (out_label) memcpy(out_label, label, (size_t)n * sizeof(int));
        if (out_seed) memcpy(out_seed, seed, (size_t)clusters * sizeof(int));
        if (min_margin) *min_margin = margin;
    }
    free(norm); free(adj); free(size); free(label); free(seed);
    return rc;
}


/* Number of threads the parallel loops use. */
int oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

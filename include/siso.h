/*
 * siso.h - C ABI of the centroid-based semantic cache hot path on one MI355X.
 *
 * The library keeps a bounded set of centroid vectors resident in GPU memory
 * (the semantic cache C_cur of Algorithm 1, bounded by the capacity M) and
 * offers the data-parallel operations on it:
 *
 *   lookup  - batched FindClosestCentroid with CosineSimilarity and the strict
 *             threshold test that judges a cache hit (Algorithm 1,
 *             MergeCentroids; section 3.1; batched online search: section 4.3);
 *   update  - fold queries into their centroid, the centroid being the average
 *             point of its group of vectors (section 3.1); lookup and update
 *             of the hits as one call for the online loop;
 *   merge   - all-pairs centroid self-similarity above the clustering
 *             threshold (the comparison inside MergeCentroids taken over all
 *             pairs), then merging connected groups into their count-weighted
 *             mean while their cluster sizes add up (Algorithm 1,
 *             cluster_size);
 *   refresh - the cache replacement of Algorithm 1 (MergeCentroids,
 *             FilteringCentroids, UpdateCentroids; section 4.2), with the
 *             access counts that lookups keep;
 *   t2h     - the threshold-to-hit-ratio table of a query sample and the choice
 *             of the retrieval threshold from the M/D/1 waiting time
 *             (section 4.3, equations 1 and 2);
 *   cluster - community detection over a query log at the clustering threshold,
 *             one repository row per cluster (section 4.1).
 *
 * Conventions
 *   - "device pointer" = memory of the current HIP device, owned by the caller,
 *     row-major and contiguous, element type fixed when the cache is created
 *     (SISO_BF16: 16-bit bfloat16 bit patterns; SISO_F32: float).
 *     The library never keeps a caller pointer after the call's work has
 *     finished on the stream.
 *   - All GPU work is enqueued on the stream given to siso_set_stream (the
 *     null stream by default).  siso_lookup, siso_update, siso_update_hits and
 *     siso_lookup_update never synchronise with the host; the other calls say
 *     when they do.
 *   - Every call returns SISO_OK (0) or a negative error code; n = 0 is a
 *     successful no-op.  siso_last_error gives a message for the last failure
 *     on that cache.  No C++ exception crosses this boundary.
 *   - The calls on one cache are not thread-safe against each other.
 */
#ifndef SISO_H
#define SISO_H

#ifdef __cplusplus
extern "C" {
#endif

typedef struct siso_cache siso_cache; /* opaque; owns all centroid state on the device */

enum { SISO_F32 = 0, SISO_BF16 = 1, SISO_FP8 = 2 /* 8-bit storage of bf16 inputs: see siso_create_ex */ };

enum {
    SISO_OK = 0,
    SISO_EINVAL = -1,    /* NULL pointer, negative size, unsupported dimension, bad index */
    SISO_ECAPACITY = -2, /* more rows than the cache was created for */
    SISO_EHIP = -3,      /* a HIP runtime call failed */
    SISO_ENOMEM = -4     /* device or host allocation failed */
};

/*
 * Create a cache for `capacity` centroids of `dim` elements (bf16 storage for
 * siso_create).  dim must be in [1, 4096]; capacity in [1, 2^31 - 1].
 * Allocates device memory: per centroid dim * (2 or 4) bytes for the stored
 * vector, 4 * dim bytes for its running mean, 16 bytes for its inverse length,
 * the weight of its mean, cluster_size and access_count.  *out receives the
 * handle.  Synchronises.
 *
 * SISO_FP8 is the 8-bit storage variant: a read-only serving copy for lookups.  Its
 * inputs (siso_load, the lookups, siso_t2h) are bf16 rows; every stored centroid is kept
 * as one 8-bit floating-point code per element (OCP E4M3: 1 sign, 4 exponent, 3 mantissa
 * bits, largest value 448) and one float scale per row, value = scale * code, with
 *     scale = max|x_t| / 448,  code_t = x_t / scale rounded to the nearest E4M3 value
 * (single precision, ties to the even mantissa, saturating); a lookup quantises its
 * batch the same way and returns the cosine of the two stored vectors - close to the
 * cosine of the bf16 rows (each element keeps 4 significant bits; cosines move by about
 * 1e-3), not equal to it.  Half the bytes of bf16 per centroid, no running means (dim
 * bytes + 20 per centroid).  dim must be a multiple of 128, at least 256.  Available:
 * siso_load, siso_lookup, siso_lookup_multi, siso_lookup_topk, siso_lookup_static,
 * siso_t2h, siso_reserve, siso_count, siso_export (codes; means must be NULL),
 * siso_export_scales, siso_export_meta, siso_fp8_follow, siso_fp8_lookup_update,
 * siso_fp8_hand_counts, siso_fp8_resync; the other calls return SISO_EINVAL.
 */
int siso_create(int dim, long capacity, siso_cache **out);
int siso_create_ex(int dim, long capacity, int dtype, siso_cache **out);

/* Waits for the cache's stream, then frees everything the cache owns. */
void siso_destroy(siso_cache *c);

/* hip_stream: a hipStream_t (NULL = the null stream).  Later calls enqueue there. */
int siso_set_stream(siso_cache *c, void *hip_stream);

/*
 * Replace the cache contents by k centroids.
 *   centroids: device pointer, [k][dim] in the cache's element type.  Rows are
 *              stored as given (they need not be exactly unit length: lookups
 *              compute true cosines of the stored values).
 *   counts:    device pointer to k cluster sizes (each >= 1), or NULL for all 1.
 * The running mean of each centroid starts as the row scaled to unit length.
 * Fails with SISO_ECAPACITY if k exceeds the capacity.  Asynchronous.
 */
int siso_load(siso_cache *c, const void *centroids, const int *counts, long k);

/* Number of live centroids (host-side value; no synchronisation). */
long siso_count(const siso_cache *c);

/*
 * Batched lookup (section 4.3; FindClosestCentroid + CosineSimilarity + hit test).
 *   queries:   device pointer, [n][dim]; need not be normalised.
 *   threshold: the retrieval threshold for this call.
 *   out_idx:   device pointer, n ints: index of the centroid with the largest
 *              cosine similarity (the lowest index among equal maxima), whether
 *              or not it is a hit; -1 for an empty cache or a query that holds
 *              a NaN or an infinity.
 *   out_sim:   device pointer, n floats: that similarity (-inf for an empty
 *              cache, NaN for a non-finite query, 0 for a zero-length query).
 *   out_hit:   device pointer, n bytes, or NULL: 1 where out_sim > threshold.
 * The similarity matrix is never written to memory.  Asynchronous, with one
 * exception: the first phase leaves a few keys per query in a workspace of the
 * cache, and a call that needs more room than any before it (a larger batch, more
 * centroids) waits for the stream and allocates.  siso_reserve sizes the workspace
 * ahead of time.
 */
int siso_lookup(siso_cache *c, const void *queries, long n, float threshold, int *out_idx, float *out_sim,
                unsigned char *out_hit);

/*
 * One lookup judged against several retrieval thresholds at once.  The retrieval
 * threshold is dynamic (section 3.3, section 4.3 "Adjusting theta_R to meet SLO") and
 * the similarity does not depend on it, so a sweep costs one similarity pass and m
 * comparisons per query instead of m lookups.
 *   thetas:      HOST pointer, m thresholds, 1 <= m <= 32 (passed on as kernel
 *                arguments: nothing is allocated or copied).
 *   count_index: position of the threshold whose hits are references to their
 *                centroids (access_count, as in siso_lookup), or -1: test lookups
 *                that count nothing.
 *   out_idx, out_sim: as in siso_lookup.
 *   out_hit:     device pointer, [n][m] bytes: out_hit[i * m + j] = 1 where out_sim[i]
 *                exceeds thetas[j], strictly.
 * Asynchronous like siso_lookup (same workspace).
 */
int siso_lookup_multi(siso_cache *c, const void *queries, long n, const float *thetas, int m, int count_index,
                      int *out_idx, float *out_sim, unsigned char *out_hit);

/*
 * The k closest centroids of every query: FindClosestCentroid (Algorithm 1) taken k
 * times, for callers that re-rank or vote among several cached answers.
 *   k:        1 <= k <= 32.
 *   out_idx:  device pointer, [n][k] ints: out_idx[i * k + r] = the centroid with the
 *             (r+1)-th largest cosine similarity to query i; among equal
 *             similarities the lower index comes first.
 *   out_sim:  device pointer, [n][k] floats: those similarities, non-increasing in r.
 * When fewer than k centroids can be chosen (a small cache, centroids holding a NaN)
 * the remaining entries are (-1, -inf); a query holding a NaN or an infinity gets
 * (-1, NaN) throughout; a query without length has similarity 0 to every centroid.
 * No threshold is involved and no access is counted.
 * bf16 caches whose dimension is a multiple of 64, and 8-bit caches (the batch is
 * quantised as in a lookup; similarities are those of the stored code vectors), take
 * two passes of the fused MFMA kernel (the k-th largest of the per-slice maxima of
 * the first pass bounds the k-th best similarity from below; the second pass lists
 * the few rows that reach the bound;
 * their cosines are then recomputed and ranked); other caches, caches of fewer than
 * 512 * k centroids and queries with more than 128 rows at the bound (many exact
 * duplicates) are scanned row by row.  Asynchronous; grows a workspace of the cache
 * (about 530 bytes per query) the first time a larger n is seen, which allocates.
 */
int siso_lookup_topk(siso_cache *c, const void *queries, long n, int k, int *out_idx, float *out_sim);

/*
 * siso_lookup for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results, but the keys of the first phase go to a
 * key array that is part of the library's image (1,048,576 keys = 8 MiB, held by
 * every GPU the library runs on until the process ends) instead of the cache's own
 * workspace: the call never allocates, frees or synchronises, and records no
 * timing events.  A batch whose first phase needs more keys (queries x slices of
 * the centroid range, e.g. the 16,384 x 512 of the largest configuration) is
 * rejected with SISO_ECAPACITY and a message; nothing has been enqueued then.
 * The array holds the last call's keys and every entry a call reads is written by
 * that call first, so nothing is cleared.  All calls on one GPU share the array:
 * calls that overlap on one GPU (two caches on two streams) race; calls on one
 * stream are ordered.  An 8-bit cache quantises the batch into a workspace of the
 * cache that siso_reserve sizes: a larger batch is rejected with SISO_ECAPACITY.
 */
int siso_lookup_static(siso_cache *c, const void *queries, long n, float threshold, int *out_idx, float *out_sim,
                       unsigned char *out_hit);

/*
 * Size the workspaces of siso_lookup, siso_update and siso_update_hits for batches
 * of up to n queries (with the cache as full as it is now, and with a full cache),
 * so that a serving loop whose batches stay within n neither allocates nor
 * synchronises in those calls.  Synchronises and allocates itself if the room
 * grows.  (Forcing another lookup kernel or tiling afterwards, see siso_bench.h,
 * changes the need.)
 */
int siso_reserve(siso_cache *c, long n);

/*
 * Centroid update as a segmented mean keyed by the assigned index.
 * For every centroid k with members I_k = { i : idx[i] == k }:
 *     mean_k  <- (size_k * mean_k + sum_{i in I_k} q_i / |q_i|) / (size_k + |I_k|)
 *     size_k  <- size_k + |I_k|
 *     stored centroid_k <- mean_k / |mean_k| rounded to the element type
 *                          (left alone if |mean_k| = 0)
 *   queries: device pointer, [n][dim];  idx: device pointer, n ints.
 * Entries with idx[i] < 0 are skipped, and so are zero-length and non-finite
 * queries.  An idx[i] >= siso_count() is skipped too and counted: see
 * siso_bad_indices.  All members of a centroid are taken in ascending i, so
 * the result does not depend on scheduling.  Asynchronous; the first batch of
 * more than 256 queries allocates 8 bytes per centroid of capacity for notes
 * (siso_reserve does it ahead of time).
 *
 * siso_update_hits folds only the entries with hit[i] != 0 (device pointer, n
 * bytes): the outputs of siso_lookup can be passed on without touching the host.
 */
int siso_update(siso_cache *c, const void *queries, const int *idx, long n);
int siso_update_hits(siso_cache *c, const void *queries, const int *idx, const unsigned char *hit, long n);

/*
 * One step of the online loop as one call: siso_lookup, then siso_update_hits with the
 * lookup's own outputs - every query that hits is folded into its centroid before the
 * next batch is looked up (the running mean of section 3.1's centroids, applied where
 * FindClosestCentroid of Algorithm 1 found a match).  Arguments as siso_lookup (out_hit
 * may not be NULL); outputs and state are bit for bit those of the two calls.
 * Batches of at most 256 queries whose lookup runs on kernels that name the winning
 * row (bf16 batches of at most 128 on the MFMA kernels, fp32 caches) finish in one
 * kernel that ends the lookup and applies the update: the workgroups of the batch tell
 * each other their (index, hit) through 256 slots of device memory of the cache (emptied
 * by the kernel before, so the call can be captured in a graph and replayed), and each
 * waits, a bounded time, until all slots of the batch are written; one that gives up
 * (never observed: all workgroups are resident together) leaves its centroid as it was
 * and is counted by siso_bad_indices.  Other batches run the two calls.  Asynchronous;
 * allocates what siso_lookup and siso_update_hits would (siso_reserve avoids that).
 */
int siso_lookup_update(siso_cache *c, const void *queries, long n, float threshold, int *out_idx, float *out_sim,
                       unsigned char *out_hit);

/* Number of queries that updates skipped since the cache was created: out-of-range
 * indices, and hits that a siso_lookup_update gave up on.
 * Synchronises with the stream.  Negative = error code. */
long siso_bad_indices(siso_cache *c);

/*
 * All-pairs self-similarity: every pair i < j of live centroids whose cosine
 * similarity exceeds `threshold` (strictly).
 *   out_pairs: device pointer, [cap][2] ints, in no particular order.
 * Returns the total number of such pairs, which may exceed cap; only the first
 * cap pairs found are written.  Negative = error code.  Synchronises.
 */
long siso_merge(siso_cache *c, float threshold, int *out_pairs, long cap);

/*
 * Merge the connected groups of the pair graph.
 *   pairs: device pointer, [n_pairs][2] ints, each a pair of distinct live
 *          indices in either order (SISO_EINVAL otherwise, nothing changed).
 *   out_survivor: device pointer, [old count] ints, or NULL: new index of the
 *          row that each old row was merged into.
 * The lowest index of a group survives with mean = sum size_i mean_i / sum size_i,
 * size = sum size_i, stored centroid = mean / |mean| rounded to the element
 * type; rows in no pair are untouched.  Survivors are packed to the front in
 * their old order and the count shrinks.  The survivors are gathered into a
 * second set of the cache's arrays, which then changes places with the first:
 * the first call that rebuilds the cache (this one or siso_refresh) allocates
 * that set, as much device memory again as siso_create took (option
 * "second_set" of siso_bench.h does it ahead of time), before anything is
 * changed: if that fails the cache is as it was.  Allocates small temporaries per call.
 * Synchronises.
 */
int siso_merge_apply(siso_cache *c, const int *pairs, long n_pairs, int *out_survivor);

/* Copy out the live rows (device pointers, any may be NULL): stored centroids
 * [count][dim] in the element type (one code byte per element for SISO_FP8), running
 * means [count][dim] floats, cluster sizes [count] ints.  Asynchronous. */
int siso_export(siso_cache *c, void *centroids, float *means, int *counts);

/* SISO_FP8 caches: the scale of every live row ([count] floats, device pointer; NaN for
 * a row that held a NaN or an infinity).  Asynchronous. */
int siso_export_scales(siso_cache *c, float *scales);

/*
 * An 8-bit cache as the serving copy of a bf16 cache that is updated online (the
 * running mean of section 3.1 is kept by the bf16 cache, the lookups of section 4.3
 * run on the copy): after siso_update / siso_update_hits on `master`, the same idx
 * (and hit, nullable: then every entry counts) bring the copy up to date - each of
 * those centroids is quantised again from the master's stored row, exactly as siso_load
 * would quantise it, and takes the weight of its mean over.  Entries below 0 or beyond
 * the live rows are skipped.  Both caches must hold the same number of centroids of the
 * same dimension (after a merge or a refresh of the master: siso_fp8_resync).
 *   idx, hit: device pointers, n entries.
 * Asynchronous on the copy's stream; the caller orders it behind the master's update
 * (same stream, or an event).
 */
int siso_fp8_follow(siso_cache *copy, const siso_cache *master, const int *idx, const unsigned char *hit, long n);

/*
 * One step of the online loop with an 8-bit serving copy, as one call: siso_lookup on
 * `copy`, siso_update_hits of its hits on `master`, siso_fp8_follow of the copy; outputs
 * and the state of both caches are bit for bit those of the three calls.  Arguments as
 * siso_lookup_update; both caches on the same stream, with the same centroids (as for
 * siso_fp8_follow).  Batches of at most 256 queries end in the one kernel that
 * siso_lookup_update describes, which also quantises the rewritten centroids into the
 * copy; others run the three calls.  A hit given up on is counted by siso_bad_indices
 * of the copy.  Asynchronous.
 */
int siso_fp8_lookup_update(siso_cache *copy, siso_cache *master, const void *queries, long n, float threshold, int *out_idx,
                           float *out_sim, unsigned char *out_hit);

/*
 * The 8-bit copy around a merge or a refresh of its master (Algorithm 1, section 4.2,
 * filters by the references that the lookups count, and those run on the copy; both calls
 * renumber the master's rows):
 *   siso_fp8_hand_counts  adds the references the copy's lookups have counted since the
 *       last hand-over to the master's access counts (saturating at infinity, which
 *       stays) and starts the copy's at zero again; same number of centroids on both.
 *   siso_fp8_resync  makes the copy the 8-bit image of the master as it stands: every live
 *       row quantised as siso_load would quantise it, weights and cluster sizes taken
 *       over, reference counts zero, siso_count(copy) = siso_count(master).
 *       SISO_ECAPACITY if the master holds more rows than the copy has room for.
 * The usual order: hand_counts, siso_refresh (or siso_merge + siso_merge_apply) on the
 * master, resync.  Both asynchronous on the copy's stream; the caller orders them against
 * the master's work (same stream, or an event).
 */
int siso_fp8_hand_counts(siso_cache *copy, siso_cache *master);
int siso_fp8_resync(siso_cache *copy, const siso_cache *master);

/*
 * Cache replacement: Algorithm 1 (SISO-CacheManager), section 4.2.
 *
 * Besides its vector every centroid carries the two numbers of that algorithm:
 * cluster_size (a float: siso_load sets it to counts[k] or 1, a refresh adds the
 * cluster sizes of merged repository centroids and then divides by 1.1) and
 * access_count (the number of hits siso_lookup has reported for it since the
 * last refresh; 0xFFFFFFFF stands for infinity, the value a centroid has while
 * it is new).  siso_merge_apply adds both up per group.
 *
 *   repo:          device pointer, [r][dim] repository centroids, element type
 *                  of the cache, 16-byte aligned, every value finite.
 *   repo_size:     device pointer, r cluster sizes (> 0).
 *   theta_c:       clustering threshold.
 *   max_centroids: M, the number of centroids the cache may hold afterwards,
 *                  1 <= M <= capacity.
 *   out_stats:     HOST pointer to 3 longs or NULL: merged, added, evicted.
 * MergeCentroids: C_new starts as the cache; the repository centroids are taken
 * in order; each looks for its closest centroid in C_new as it stands then
 * (lowest index among equals; cached centroids first, then the added ones in
 * the order they were added); if the cosine exceeds theta_c (strictly) its
 * cluster size is added to that centroid's, otherwise it joins C_new, stored as
 * given, with access_count = infinity.  FilteringCentroids: while C_new has more
 * than M rows the row with the smallest (cluster_size, access_count) goes, the
 * first such row in the order of C_new; then every cluster_size is divided by
 * 1.1 (in single precision) and every access_count reset to 0.  UpdateCentroids:
 * C_new becomes the cache, survivors keep their order; a lookup enqueued before
 * the call sees the old set, one enqueued after it the new one.
 * The similarity work (repository against cache, repository against itself)
 * runs on the GPU; the chain of decisions and the choice of the survivors are
 * bookkeeping on the host.  Nothing changes if an error is returned before the
 * update step (bad arguments, a non-finite row, a cluster size <= 0).
 * The new set is gathered into the second set of the cache's arrays (see
 * siso_merge_apply), which then becomes the cache: nothing is copied back.
 * Allocates temporary device memory for the repository.  Synchronises.
 *
 * siso_export_meta: copy out cluster_size [count] floats and access_count
 * [count] unsigned ints (device pointers, either may be NULL).  Asynchronous.
 */
int siso_refresh(siso_cache *c, const void *repo, const float *repo_size, long r, float theta_c, long max_centroids,
                 long *out_stats);
int siso_export_meta(siso_cache *c, float *cluster_size, unsigned *access_count);

/*
 * Replace the cache contents by a snapshot of k centroids, taken over as it is:
 * what siso_export and siso_export_meta copied out (the centroid repository is the
 * persistent store of section 4.1; the paper gives no format, the arrays are it).
 *   centroids [k][dim] element type, means [k][dim] floats, counts [k] ints (>= 1):
 *   device pointers, required;  cluster_size [k] floats, access_count [k] unsigned
 *   ints (0xFFFFFFFF = infinity): device pointers or NULL (cluster_size = counts,
 *   access_count = 0).
 * Nothing is normalised or rounded; only the inverse length of each stored row is
 * computed.  SISO_ECAPACITY if k exceeds the capacity.  Asynchronous.
 */
int siso_import(siso_cache *c, const void *centroids, const float *means, const int *counts,
                const float *cluster_size, const unsigned *access_count, long k);

/*
 * The host part of siso_refresh by itself: the decisions of Algorithm 1 from
 * the similarities that the kernels supply.  Needs no GPU; all pointers are
 * HOST pointers.
 *   cluster_size, access_count: [k0] of the cached centroids.
 *   repo_size:  [r] cluster sizes of the repository rows (> 0).
 *   best_idx, best_sim: [r] per repository row its closest cached centroid
 *               (-1 if the cache is empty) and the cosine.
 *   pairs, pair_cosine: [n_pairs] pairs (a, b), a < b < r, of repository rows
 *               whose cosine exceeds theta_c, and that cosine.
 *   out_source: room for k0 + r ints: per surviving row, in order, the cached
 *               row it is (< k0) or k0 + the repository row that joined.
 *   out_cluster_size: room for k0 + r floats: its cluster_size afterwards.
 *   out_stats:  3 longs or NULL: merged, added, evicted.
 * Returns the number of surviving rows, or a negative error code.
 */
long siso_refresh_plan(long k0, const float *cluster_size, const unsigned *access_count, long r,
                       const float *repo_size, const int *best_idx, const float *best_sim, const int *pairs,
                       const float *pair_cosine, long n_pairs, float theta_c, long max_centroids,
                       int *out_source, float *out_cluster_size, long *out_stats);

/*
 * Clustering of a query log into the centroid repository: section 4.1
 * ("Selecting a clustering algorithm": community detection at the clustering
 * threshold; "Keeping centroids in a repository": id, centroid, cluster_size)
 * with the centroid of section 3.1, the average of the group.
 *
 *   vectors:   device pointer, [n][dim] query vectors, element type of the
 *              cache, 16-byte aligned, every one finite and of non-zero length
 *              (SISO_EINVAL otherwise, nothing changed).
 *   theta_c:   clustering threshold;  min_size: smallest cluster kept (>= 1).
 *   out_label: device pointer, n ints, or NULL: cluster id of every vector,
 *              -1 for a vector that ends in no cluster.
 *   out_representative: device pointer, room for min(n, capacity) ints, or
 *              NULL: per cluster the member with the largest cosine to the
 *              centroid (the lowest index among equals): the query whose
 *              output text stands for the cluster in the repository.
 *   out_stats: HOST pointer to 2 longs or NULL: pairs above the threshold,
 *              vectors that ended in a cluster.
 * Two vectors are neighbours when their cosine exceeds theta_c (strictly).  The
 * candidate community of a vector is itself with its neighbours; candidates
 * are taken by size, largest first, equal sizes by index; of a candidate the
 * vectors that no earlier cluster holds remain (the vector it was built around
 * may be gone), and if at least min_size remain they become the next cluster;
 * ids count up from 0 in that order.
 * Afterwards the cache `c` IS the repository: row id holds cluster id, mean =
 * average of the unit-length members (summed in ascending index), size =
 * cluster_size = their number, stored centroid = mean / |mean| rounded to the
 * element type (a zero row if the mean has no length), access_count 0; what
 * the cache held before is gone.  siso_export / siso_export_meta hand the rows
 * and sizes on, e.g. to siso_refresh of the serving cache.
 * Returns the number of clusters; SISO_ECAPACITY (nothing changed) if that
 * exceeds the capacity of `c`; other negative values are error codes.
 * The all-pairs similarity and the averages run on the GPU; the choice of the
 * communities walks the list of pairs on the host.  Allocates temporary device
 * memory (the vectors once more, 8 bytes per pair).  Synchronises.
 */
long siso_cluster(siso_cache *c, const void *vectors, long n, float theta_c, int min_size, int *out_label,
                  int *out_representative, long *out_stats);

/*
 * The host part of siso_cluster by itself: the choice of the communities from a
 * list of neighbour pairs (same section, same rules).  Needs no GPU.
 *   pairs:     HOST pointer, [n_pairs][2] ints: every pair of neighbours once,
 *              in either order, indices in [0, n), the two of a pair distinct
 *              (SISO_EINVAL otherwise).
 *   out_label: HOST pointer, n ints: cluster id of every vector or -1.
 * Returns the number of clusters, or a negative error code.
 */
long siso_choose_communities(const int *pairs, long n_pairs, long n, int min_size, int *out_label);

/*
 * Threshold-to-hit-ratio (T2H) table (section 4.3, "Adjusting theta_R to meet
 * SLO"): test lookups of a sample of queries, counted against a sweep of
 * retrieval thresholds (the paper sweeps 0.98 down to 0.6).
 *   queries:  device pointer, [n][dim] sample queries.
 *   thetas:   HOST pointer, m thresholds in any order, m <= 1024.
 *   out_hits: HOST pointer, m counts: out_hits[j] = number of sample queries
 *             whose top-1 similarity exceeds thetas[j] (strictly, compared as
 *             floats like the hit test of siso_lookup); h(theta_j) = out_hits[j] / n.
 * One lookup serves all thresholds (the similarity does not depend on them).
 * Allocates temporary device memory.  Synchronises.
 */
int siso_t2h(siso_cache *c, const void *queries, long n, const float *thetas, int m, long *out_hits);

/*
 * Host-side arithmetic of the same section; no GPU work, no cache needed.
 *
 * siso_md1_wait: expected waiting time W of the LLM system modelled as an M/D/1
 * queue (equation 2): E = llm_time * (1 - hit_ratio),
 * W = E + arrival_rate * E^2 / (2 * (1 - arrival_rate * E)); +infinity when the
 * queue is unstable (arrival_rate * E >= 1).
 *
 * siso_pick_threshold: the highest threshold of a T2H table (thetas[j],
 * hit_ratio[j], j < m, any order, host pointers) whose W stays below the SLO
 * latency (slo > W, strictly).  *out_index = its position, -1 if no entry meets
 * the SLO.  Returns SISO_OK or SISO_EINVAL.
 *
 * siso_adjust_threshold: the correction applied when the measured waiting time
 * is more than 10 % off the estimate: longer -> the next lower threshold of the
 * table, shorter -> the next higher one; otherwise, or at the end of the table,
 * or for an index outside [0, m), the position is returned unchanged.
 */
double siso_md1_wait(double llm_time, double arrival_rate, double hit_ratio);
int siso_pick_threshold(const float *thetas, const double *hit_ratio, int m, double llm_time, double arrival_rate,
                        double slo, int *out_index);
int siso_adjust_threshold(const float *thetas, int m, int index, double wait_estimated, double wait_measured);

/* Message for the last error on this cache ("" if none).  Owned by the cache. */
const char *siso_last_error(const siso_cache *c);

#ifdef __cplusplus
}
#endif
#endif /* SISO_H */

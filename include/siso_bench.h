/*
 * siso_bench.h - tuning and measurement entry points of libsiso.so, for benchmarks,
 * profiling runs and tests that force one kernel.  Nothing here is needed to use the
 * cache (include/siso.h); the defaults are chosen by the library.
 */
#ifndef SISO_BENCH_H
#define SISO_BENCH_H

#include "siso.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Lookup kernel selection for siso_set_lookup_path. */
enum {
    SISO_PATH_AUTO = 0,   /* choose by element type, dimension and batch size       */
    SISO_PATH_SCALAR = 1, /* LDS-tiled fp32 FMA kernel; any type and dimension       */
    SISO_PATH_MFMA = 2,   /* fused bf16 MFMA GEMM + running arg-max (large batches)  */
    SISO_PATH_SKINNY = 3  /* bandwidth-bound bf16 path for batches of at most 64     */
};

/* Force one lookup kernel (SISO_PATH_*); a path that cannot handle the cache's
 * type or dimension, or the batch size of a later call, makes that call fail
 * with SISO_EINVAL. */
int siso_set_lookup_path(siso_cache *c, int path);

/*
 * Tuning knobs, for benchmarking; the defaults are chosen by the library.
 *   "mfma_config"     0 = default; 1 = 256x256 tile, 2 = 256x128, 3 = 256x64, 4 = 256x256 with half-width slabs,
 *                     5 = 256x256 with four waves of 128x128; 8-bit caches: 6, 7, 8 = the tiles of 1, 2, 3 on the
 *                     64-deep fp8 MFMA (their default), 1, 2, 3 = the same on the 16-deep one
 *   "tiles_per_slice" 0 = default; >0 = centroid tiles one workgroup walks through
 *   "merge_config"    0 = default (bf16: the eight-wave MFMA pair search); 1 = use the scalar pair search;
 *                     2 = the four-wave MFMA pair search (128x128 per wave)
 *   "mfma_qblock"     0 = default; 1, 2, 4, 8, 16, 32 = query tiles that share an XCD's centroid tiles
 *   "fold_spin_limit" -1 = default; >= 0: how often a workgroup of siso_lookup_update's one-kernel end looks at the
 *                     board before it gives up (0: at once - for tests of that path)
 *   "stream_hint"     0 = default (the centroid loads of a lookup are marked non-temporal when the batch is one
 *                     tile of queries and the centroids exceed 288 MiB, or, four-wave kernel, when they exceed
 *                     288 MiB); 1 = always, 2 = never
 *   "second_set"      1 = allocate now the second set of arrays that siso_merge_apply and siso_refresh
 *                     gather the rebuilt cache into (otherwise their first call does); synchronises
 * Unknown names or values out of range give SISO_EINVAL.
 */
int siso_set_option(siso_cache *c, const char *name, long value);

/*
 * Kernel timing for benchmarks.  While enabled (on = N > 0), every N-th
 * siso_lookup / siso_merge brackets its dominant kernel (the similarity kernel,
 * without the finalize kernel) with a pair of HIP events on the cache's stream
 * (an event costs a few microseconds on the stream, so short steps sample).
 * A pair of events with nothing between them already reads about 4 us;
 * siso_profile_enable measures that on the stream (it synchronises) and every
 * bracket is reduced by it.
 * siso_profile_read synchronises with the stream, returns the sum of the
 * bracketed durations in milliseconds and the number of brackets since the
 * last read (host pointers, either may be NULL), and releases the events.
 * At most 8192 brackets are kept between reads; later ones are not recorded.
 */
int siso_profile_enable(siso_cache *c, int on);
int siso_profile_read(siso_cache *c, double *total_ms, long *launches);

/*
 * What this chip delivers, for the roofline lines of a benchmark (no cache
 * needed; runs on the null stream of the current device, allocates and frees
 * its own memory, synchronises; takes a fraction of a second):
 *   which = 0: a register-resident bf16 MFMA loop on random operands, TFLOP/s
 *              (the clock the chip sustains depends on how much operands toggle);
 *   which = 1: the same on constant operands, TFLOP/s;
 *   which = 2: a plain streaming read of 2 GiB from HBM, GB/s.
 * *out_value (host pointer) receives the rate.  SISO_OK, SISO_EINVAL or SISO_EHIP.
 */
int siso_probe(int which, double *out_value);

#ifdef __cplusplus
}
#endif
#endif /* SISO_BENCH_H */

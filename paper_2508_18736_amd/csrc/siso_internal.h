// Internal declarations shared by the translation units of libsiso.so.
// Nothing here is visible through the C ABI (include/siso.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "siso.h"
#include "siso_bench.h"

typedef unsigned long long u64;
typedef unsigned short bf16_t;  // bfloat16 bit pattern

// A phase-1 lookup kernel reduces, for every query q and every slice s of the
// centroid range, the scaled dot products <q, c_k> / |c_k| to one 64-bit key
//     key = ordered(value) << 32 | (0xFFFFFFFF - id)
// so that an unsigned max over keys picks the largest value and, among equal
// values, the lowest id.  Key 0 means "no candidate".  The id is either the row
// itself (kernels that can afford the exact arg-max in their epilogue: the value
// then is the similarity but for the factor 1 / |q|), or the number k / 4 of a
// group of four consecutive rows that holds the best one (what a lane of a
// 32 x 32 MFMA accumulator holds in four consecutive registers: rows 8*g + 4*h
// + j of an aligned run of 32, j = 0..3); the finalize kernel then recomputes
// the four cosines exactly and picks the lowest index among their maxima.  Ids
// ascend with the rows, so "the lowest id among equal values" always holds the
// lowest index among equal maxima.
enum { SISO_KEY_ROWS = 1, SISO_KEY_GROUPS4 = 3 };
#define SISO_ACCESS_INF 0xFFFFFFFFu
#define SISO_MAX_DIM 4096
#define SISO_FOLD_BOARD 256  // queries of a siso_lookup_update that ends in one kernel: one slot each
#define SISO_MULTI_MAX 32  // thresholds one lookup can be judged against
#define SISO_PAD_ROWS 256  // readable rows past the capacity of the stored-centroid array

struct siso_cache {
    int dim;
    long capacity;
    int dtype;
    long count;
    int device;
    int path;
    hipStream_t stream;

    void *cent;   // [capacity][dim] stored centroids (bf16 bits or float)
    float *mean;  // [capacity][dim] mean of the unit-length members
    int *size;    // [capacity] cluster_size
    float *invn;  // [capacity] 1 / |stored centroid| (0 for a zero row, NaN for a non-finite row)
    float *locality;   // [capacity] cluster_size of Algorithm 1: grows by merges, decays by 1.1 per refresh
    unsigned *access;  // [capacity] access_count of Algorithm 1: hits since the last refresh; SISO_ACCESS_INF = infinity
    // A second set of the six arrays, allocated the first time a call rebuilds the cache (group merge, refresh):
    // the new set is gathered there and the two sets change places, so nothing is copied back and such calls
    // allocate nothing afterwards.
    void *cent_b;
    float *mean_b;
    int *size_b;
    float *invn_b;
    float *locality_b;
    unsigned *access_b;

    // large update batches: first member and number of members per centroid, [capacity] each, allocated at
    // the first such batch; between calls every entry is back at (INT_MAX, 0)
    int *upd_owner;
    int *upd_members;

    // workspace, grown on demand
    u64 *keys;     // [keys_cap] phase-1 keys, n * slices
    long keys_cap;

    u64 *static_keys;  // this device's copy of the library's static key array (siso_lookup_static)

    u64 *counters;  // device: [0] bad update indices, [1] merge pair count, [2] scratch, [3] scratch; behind them the
                    // board of siso_lookup_update (SISO_FOLD_BOARD slots)
    u64 *host_pin;  // pinned host mirror for counter read-back (4 entries)

    // 8-bit storage (SISO_FP8): cent holds one E4M3 code per element, scale [capacity] the scale of every row
    // (NaN for a non-finite row), invn the inverse lengths of the code rows; there is no running mean.
    // fp8_q / fp8_qinv: codes and inverse code lengths of the batch being looked up, [fp8_q_cap] rows, grown on demand
    float *scale;
    void *fp8_q;
    float *fp8_qinv;
    long fp8_q_cap;

    // top-k lookups: per query the bound, the number of listed rows, a flag "scan this query row by row" and
    // the listed rows ([topk_cap] floats / ints / ints, [topk_cap][SISO_TOPK_CAND] ints), grown on demand
    float *topk_tau;
    int *topk_cnt;
    int *topk_cand;
    long topk_cap;
    int plan_min_slices;  // > 0 while a top-k lookup plans its passes: at least this many slices (if the tiles allow)
    const siso_cache *fold_master;  // not NULL while siso_fp8_lookup_update runs its lookup on this 8-bit copy
    int mark_in_finalize;  // siso_lookup_update on a large batch: 1 = the finalize step shall take the update's notes
                           // (first member and number of members per centroid), 2 = it has; 0 otherwise
    u64 *board_to_clear;  // not NULL while siso_lookup_update launches its first phase: a kernel that empties these
                          // slots sets it back to NULL

    // tuning knobs (siso_set_option); 0 = library default
    int opt_mfma_config;
    int opt_tiles_per_slice;
    int opt_merge_config;
    int opt_mfma_qblock;
    int opt_fold_spin_limit;  // -1 = default
    int opt_stream_hint;      // 0 = default; 1 = mark the centroid loads of the eight-wave lookups as streaming, 2 = never

    // kernel timing (siso_profile_enable / siso_profile_read)
    int profile_on;       // 0 = off, N = bracket every N-th call
    long prof_calls;      // calls seen since profiling was enabled
    int prof_open;        // a bracket was opened by the current call
    hipEvent_t *prof_ev;  // pairs: [2*i] start, [2*i+1] stop
    int prof_count;       // recorded pairs
    double prof_empty_ms; // what a pair of events with nothing between them measures on this stream

    char err[256];
};

// ----------------------------------------------------------------------------
// device helpers
// ----------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }

// round-to-nearest-even float -> bf16 bit pattern (NaN stays NaN)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)0x7FC0;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(bf16_t v) { return bf16_to_f32(v); }

// One OCP E4M3 code of the 8-bit storage (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals
// m/8 * 2^-6); a type of its own so that templates can tell a code from a byte.
struct fp8_t {
    unsigned char v;
};
__device__ __forceinline__ float e4m3_to_f32(unsigned code) {
    const unsigned e = (code >> 3) & 15u, m = code & 7u;
    const float v = e == 0 ? (float)m * 0.001953125f : __uint_as_float(((e + 120u) << 23) | (m << 20));
    return (code & 0x80u) ? -v : v;
}
__device__ __forceinline__ float widen(fp8_t c) { return e4m3_to_f32(c.v); }

__device__ __forceinline__ void narrow(float v, float *out) { *out = v; }
__device__ __forceinline__ void narrow(float v, bf16_t *out) { *out = f32_to_bf16(v); }

// monotone map float -> unsigned (larger float <=> larger unsigned; NaN excluded by callers)
__device__ __forceinline__ unsigned ordered_bits(float f) {
    unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float unordered_bits(unsigned o) {
    unsigned u = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(u);
}
__device__ __forceinline__ u64 pack_key(float value, unsigned block) {
    return ((u64)ordered_bits(value) << 32) | (u64)(0xFFFFFFFFu - block);
}

// 1/|x| from the sum of squares: 0 for a zero vector, NaN if the sum is not finite
__device__ __forceinline__ float inv_length(float sumsq) {
    if (!(sumsq == sumsq) || sumsq > 3.0e38f) return __uint_as_float(0x7FC00000u);
    if (sumsq == 0.0f) return 0.0f;
    return 1.0f / sqrtf(sumsq);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// 16-byte chunk dot products (finalize, top-k re-ranking)
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float chunk_dot(const float *a, const float *b) {
    const float4 x = *(const float4 *)a, y = *(const float4 *)b;
    return x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
}
__device__ __forceinline__ float chunk_dot(const bf16_t *a, const bf16_t *b) {
    const u32x4_t x = *(const u32x4_t *)a, y = *(const u32x4_t *)b;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s += __uint_as_float(x[i] << 16) * __uint_as_float(y[i] << 16);
        s += __uint_as_float(x[i] & 0xFFFF0000u) * __uint_as_float(y[i] & 0xFFFF0000u);
    }
    return s;
}

// the same sums from chunks that are already in registers
__device__ __forceinline__ float chunk_dot(u32x4_t x, u32x4_t y, float) {
    return __uint_as_float(x[0]) * __uint_as_float(y[0]) + __uint_as_float(x[1]) * __uint_as_float(y[1]) +
           __uint_as_float(x[2]) * __uint_as_float(y[2]) + __uint_as_float(x[3]) * __uint_as_float(y[3]);
}
__device__ __forceinline__ float chunk_dot(u32x4_t x, u32x4_t y, bf16_t) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s += __uint_as_float(x[i] << 16) * __uint_as_float(y[i] << 16);
        s += __uint_as_float(x[i] & 0xFFFF0000u) * __uint_as_float(y[i] & 0xFFFF0000u);
    }
    return s;
}

__device__ __forceinline__ float chunk_dot(u32x4_t x, u32x4_t y, fp8_t) {  // sixteen codes
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int b = 0; b < 32; b += 8) s += e4m3_to_f32((x[i] >> b) & 0xFFu) * e4m3_to_f32((y[i] >> b) & 0xFFu);
    }
    return s;
}

// ---- the quantiser of the 8-bit storage (k_fp8_quantize, and the end of siso_fp8_lookup_update)
__device__ __forceinline__ unsigned f32_to_e4m3(float y) {
    const unsigned sign = (__float_as_uint(y) >> 24) & 0x80u;
    const float a = fabsf(y);
    if (a >= 448.f) return sign | 0x7Eu;
    if (a < 0.015625f) return sign | (unsigned)(int)rintf(a * 512.f);  // multiples of 2^-9; 8 of them is 2^-6 = code 0x08
    unsigned v = __float_as_uint(a);
    v += 0x7FFFFu + ((v >> 20) & 1u);  // to three mantissa bits, ties to even (may carry into the exponent)
    return sign | ((((v >> 23) - 120u) << 3) | ((v >> 20) & 7u));
}
__device__ __forceinline__ float block_max256(float v, float *sh) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}
__device__ __forceinline__ float block_sum256f(float v, float *sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}
// One row by a 256-thread block: x = this thread's elements (columns t + 256 e; 0 beyond d).  Writes the codes,
// the scale (if asked for) and 1 / |code row| (0 for a row without length, NaN for a non-finite one).
template <int E>
__device__ __forceinline__ void fp8_store_row(const float (&x)[E], int d, unsigned char *codes_row, float *scale_out,
                                              float *inv_out, float *sh) {
    const int t = threadIdx.x;
    float amax = 0.f;
    bool finite = true;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        finite = finite && fabsf(x[e]) <= 3.4e38f;  // false for NaN and infinity
        amax = fmaxf(amax, fabsf(x[e]));
    }
    const float bad = block_max256(finite ? 0.f : 1.f, sh);
    amax = block_max256(amax, sh);
    const float sc = amax / 448.0f;
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int col = t + e * 256;
        if (col < d) {
            const unsigned code = (bad > 0.f || amax == 0.f) ? 0u : f32_to_e4m3(__fdiv_rn(x[e], sc));
            codes_row[col] = (unsigned char)code;
            const float back = e4m3_to_f32(code);
            ss = __fmaf_rn(back, back, ss);
        }
    }
    ss = block_sum256f(ss, sh);
    if (t == 0) {
        const float nanv = __uint_as_float(0x7FC00000u);
        if (scale_out) *scale_out = bad > 0.f ? nanv : sc;
        *inv_out = bad > 0.f ? nanv : inv_length(ss);
    }
}

// Wave-ballot compaction of (i, j) pairs into out[cap][2]; every lane of the wave
// must call it.  counter accumulates the total number of pairs, also beyond cap.
__device__ __forceinline__ void emit_pair(bool pred, int i, int j, int *out, long cap, u64 *counter) {
    const u64 mask = __ballot(pred);
    if (mask == 0) return;
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((long long)mask) - 1;
    u64 base = 0;
    if (lane == leader) base = atomicAdd(counter, (u64)__popcll(mask));
    base = __shfl(base, leader);
    if (pred) {
        const u64 pos = base + (u64)__popcll(mask & ((1ull << lane) - 1ull));
        if (pos < (u64)cap) {
            out[2 * pos] = i;
            out[2 * pos + 1] = j;
        }
    }
}

// The same for up to 32 candidates per lane at once: bit I of `mask` says that this lane has the
// pair (i, j0 + row_of(I)); the wave takes one slot range with a single atomic and every lane
// writes its pairs behind those of the lanes before it.  Every lane of the wave must call it.
template <class RowOf>
__device__ __forceinline__ void emit_pairs(unsigned mask, int i, RowOf row_of, int *out, long cap, u64 *counter) {
    const int lane = threadIdx.x & 63;
    const int cnt = __popc(mask);
    int incl = cnt;  // inclusive prefix sum over the wave
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
    }
    const int total = __shfl(incl, 63);
    if (total == 0) return;
    u64 base = 0;
    if (lane == 63) base = atomicAdd(counter, (u64)total);
    base = __shfl(base, 63);
    u64 pos = base + (u64)(incl - cnt);
    while (mask != 0) {
        const int I = __ffs((int)mask) - 1;
        mask &= mask - 1;
        if (pos < (u64)cap) {
            out[2 * pos] = i;
            out[2 * pos + 1] = row_of(I);
        }
        ++pos;
    }
}

// The same with a staging buffer of the workgroup in LDS (stage[room][2], *staged = entries taken):
// the lanes take their slots with LDS atomics, which cost a fraction of the round trip of a global
// one; what does not fit any more goes straight to the global list.  Every lane must call it.
template <class RowOf>
__device__ __forceinline__ void emit_pairs_staged(unsigned mask, int i, RowOf row_of, int *stage, int *staged, int room,
                                                  int *out, long cap, u64 *counter) {
    // few lanes hold pairs (a block of 32 x 32 products with one group of near-duplicates in it): each of them
    // takes its slots with an LDS atomic of its own, which is cheaper than a prefix sum over the wave
    const int cnt = __popc(mask);
    if (__ballot(cnt != 0) == 0) return;
    int pos = cnt != 0 ? atomicAdd(staged, cnt) : 0;
    unsigned rest = 0;  // pairs of this lane that found no room
    while (mask != 0) {
        const int I = __ffs((int)mask) - 1;
        mask &= mask - 1;
        if (pos < room) {
            stage[2 * pos] = i;
            stage[2 * pos + 1] = row_of(I);
        } else {
            rest |= 1u << I;
        }
        ++pos;
    }
    if (__ballot(rest != 0) != 0) emit_pairs(rest, i, row_of, out, cap, counter);  // uniform over the wave
}

// Move the staged pairs of the workgroup to the global list and empty the buffer.  Every thread of
// the workgroup must call it (it synchronises); `slot` = one u64 of LDS for the broadcast.
__device__ __forceinline__ void flush_staged_pairs(const int *stage, int *staged, int room, u64 *slot, int *out, long cap,
                                                   u64 *counter) {
    __syncthreads();
    const int n = *staged < room ? *staged : room;
    if (threadIdx.x == 0 && n > 0) *slot = atomicAdd(counter, (u64)n);
    __syncthreads();
    if (n > 0) {
        const u64 base = *slot;
        for (int p = threadIdx.x; p < n; p += blockDim.x) {
            if (base + (u64)p < (u64)cap) {
                out[2 * (base + p)] = stage[2 * p];
                out[2 * (base + p) + 1] = stage[2 * p + 1];
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) *staged = 0;
    __syncthreads();
}

// ----------------------------------------------------------------------------
// host-side plumbing shared by the translation units
// ----------------------------------------------------------------------------
int siso_fail(siso_cache *c, int code, const char *fmt, ...);
void siso_prof_begin(siso_cache *c);  // bracket the dominant kernel of a call (no-ops unless enabled)
void siso_prof_end(siso_cache *c);
int siso_check_hip(siso_cache *c, hipError_t e, const char *what);

// Phase-1 launchers.  Each fills keys[q * slices + s] for all q < n, s < slices (every entry is written,
// nothing has to be cleared beforehand).
// *_slices returns the number of slices the launcher will use (0 = path cannot
// handle this cache / batch).
int siso_scalar_slices(const siso_cache *c, long n);
int siso_scalar_launch(siso_cache *c, const void *queries, long n, int slices, u64 *keys);
int siso_mfma_slices(const siso_cache *c, long n);
int siso_mfma_launch(siso_cache *c, const void *queries, long n, int slices, u64 *keys, int *row_keys);
int siso_skinny_slices(const siso_cache *c, long n);
int siso_skinny_launch(siso_cache *c, const void *queries, long n, int slices, u64 *keys, int *row_keys);

// Top-k lookups on the MFMA kernels: pass 1 = the phase-1 keys of a lookup planned with c->plan_min_slices;
// pass 2 lists, per query q, the rows whose scaled product <q, c> / |c| reaches tau[q] (cand[q * cap + i],
// i < min(cnt[q], cap); cnt counts all of them; cnt must be zero before).  Both passes sum every product in
// the same order, so a row that set a key in pass 1 compares equal to it in pass 2.
#define SISO_TOPK_MAX 32
#define SISO_TOPK_CAND 128
int siso_topk_mfma_slices(const siso_cache *c, long n);  // slices of the plan (0 = these kernels cannot serve the cache)
int siso_topk_mfma_pass1(siso_cache *c, const void *queries, long n, int slices, u64 *keys, int *row_keys);
int siso_topk_mfma_collect(siso_cache *c, const void *queries, long n, int slices, const float *tau, int *cand,
                           int *cnt, int cap);

// Self-similarity pair search over `count` rows of the cache's element type and dimension with
// their inverse lengths (counter already zeroed).  The MFMA kernel reads whole tiles: rows and invn
// must be readable for SISO_PAD_ROWS entries past count, the invn entries there holding NaN.
int siso_pairs_scalar_launch(siso_cache *c, const void *rows, const float *invn, long count, float threshold,
                             int *out_pairs, long cap, u64 *counter);
int siso_pairs_mfma_supported(const siso_cache *c, long count);
int siso_pairs_mfma_launch(siso_cache *c, const void *rows, const float *invn, long count, float threshold,
                           int *out_pairs, long cap, u64 *counter);

// siso_lookup without the argument checks of the ABI, against m thresholds (host pointer, 1 <= m <=
// SISO_MULTI_MAX; out_hit is [n][m] or NULL); the hits at thetas[count_index] are references to their
// centroids (access_count goes up), as in serving; count_index = -1 for test lookups.  static_keys: NULL = the phase-1
// keys go to the cache's own workspace (grown on demand); otherwise they go there (room for static_cap keys:
// a larger need is an error), and the call allocates nothing and records no timing events.
// folded: NULL = a lookup and nothing else; otherwise the caller is about to fold the hits into their centroids
// and *folded tells whether the lookup has already done it (small batches: one kernel ends the lookup and
// applies the update).
int siso_lookup_impl(siso_cache *c, const void *queries, long n, const float *thetas, int m, int count_index,
                     int *out_idx, float *out_sim, unsigned char *out_hit, u64 *static_keys = nullptr,
                     long static_cap = 0, int *folded = nullptr);
int siso_fp8_load(siso_cache *c, const void *centroids, const int *counts, long k);  // siso_load of an 8-bit cache
int siso_fp8_ensure_batch(siso_cache *c, long n);
int siso_fp8_quantize_batch(siso_cache *c, const void *queries, long n);  // bf16 queries -> c->fp8_q, c->fp8_qinv
int siso_read_counter(siso_cache *c, int which, u64 *value);
int siso_ensure_keys(siso_cache *c, long need);  // room for `need` phase-1 keys in c->keys (may synchronise and allocate)
int siso_second_set(siso_cache *c);    // make sure the second set of arrays exists (allocates once; synchronises then)
void siso_swap_sets(siso_cache *c);    // the second set becomes the cache, the old arrays the second set  // synchronises

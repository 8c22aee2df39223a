// C ABI of the centroid cache (include/siso.h): state management, the kernels
// that are not matrix-shaped (row norms, finalize, update, group merge) and the
// LDS-tiled fp32 kernels that serve any element type and dimension.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>
#include <utility>

#include "siso_internal.h"

// ============================================================================
// error plumbing
// ============================================================================
int siso_fail(siso_cache *c, int code, const char *fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

int siso_check_hip(siso_cache *c, hipError_t e, const char *what) {
    if (e == hipSuccess) return SISO_OK;
    return siso_fail(c, SISO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(c, call)                                          \
    do {                                                          \
        int rc_ = siso_check_hip((c), (call), #call);             \
        if (rc_ != SISO_OK) return rc_;                           \
    } while (0)

#define SISO_PROF_MAX 8192

void siso_prof_begin(siso_cache *c) {
    c->prof_open = 0;
    if (!c->profile_on || c->prof_count >= SISO_PROF_MAX) return;
    if (c->prof_calls++ % c->profile_on != 0) return;
    if (!c->prof_ev) {
        c->prof_ev = (hipEvent_t *)calloc(2 * SISO_PROF_MAX, sizeof(hipEvent_t));
        if (!c->prof_ev) return;
    }
    hipEvent_t *e = c->prof_ev + 2 * c->prof_count;
    if (hipEventCreate(&e[0]) != hipSuccess || hipEventCreate(&e[1]) != hipSuccess) return;
    (void)hipEventRecord(e[0], c->stream);
    c->prof_open = 1;
}

void siso_prof_end(siso_cache *c) {
    if (!c->prof_open) return;
    hipEvent_t *e = c->prof_ev + 2 * c->prof_count;
    if (!e[0] || !e[1]) return;
    (void)hipEventRecord(e[1], c->stream);
    c->prof_count++;
}

static inline size_t elem_bytes(int dtype) { return dtype == SISO_F32 ? 4 : dtype == SISO_FP8 ? 1 : 2; }

// the calls an 8-bit cache does not offer (it is a read-only serving copy: lookups, and siso_load to rebuild it)
#define SISO_NOT_FP8(c, what)                                                                                        \
    do {                                                                                                             \
        if ((c)->dtype == SISO_FP8) return siso_fail((c), SISO_EINVAL, what ": not available with the 8-bit storage"); \
    } while (0)

// ============================================================================
// small kernels
// ============================================================================
// Block-wide sum for 256-thread blocks; every thread gets the result.
__device__ __forceinline__ float block_sum256(float v, float *sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// siso_load: store rows verbatim, mean = row / |row|, size = counts or 1, invn = 1/|row|.
template <typename T>
__global__ __launch_bounds__(256) void k_load_rows(const T *__restrict__ src, const int *__restrict__ counts, T *cent,
                                                    float *mean, int *size, float *invn, float *locality,
                                                    unsigned *access, int d) {
    __shared__ float sh[4];
    const long k = blockIdx.x;
    const T *row = src + (size_t)k * d;
    float ss = 0.f;
    for (int e = threadIdx.x; e < d; e += 256) {
        float x = widen(row[e]);
        ss += x * x;
    }
    const float n2 = block_sum256(ss, sh);
    const float inv = inv_length(n2);
    const bool ok = (inv == inv) && inv > 0.f;
    const float nrm = sqrtf(n2);
    for (int e = threadIdx.x; e < d; e += 256) {
        T x = row[e];
        cent[(size_t)k * d + e] = x;
        mean[(size_t)k * d + e] = ok ? widen(x) / nrm : 0.f;
    }
    if (threadIdx.x == 0) {
        int s = counts ? counts[k] : 1;
        size[k] = s < 1 ? 1 : s;
        invn[k] = inv;
        locality[k] = (float)(s < 1 ? 1 : s);
        access[k] = 0;
    }
}

// siso_import: take over a snapshot as it is; only the inverse length of the stored row is computed.
template <typename T>
__global__ __launch_bounds__(256) void k_import_rows(const T *__restrict__ src, const float *__restrict__ src_mean,
                                                      const int *__restrict__ src_size, const float *__restrict__ src_loc,
                                                      const unsigned *__restrict__ src_acc, T *cent, float *mean, int *size,
                                                      float *invn, float *locality, unsigned *access, int d) {
    __shared__ float sh[4];
    const long k = blockIdx.x;
    float ss = 0.f;
    for (int e = threadIdx.x; e < d; e += 256) {
        const T x = src[(size_t)k * d + e];
        cent[(size_t)k * d + e] = x;
        mean[(size_t)k * d + e] = src_mean[(size_t)k * d + e];
        ss += widen(x) * widen(x);
    }
    const float n2 = block_sum256(ss, sh);
    if (threadIdx.x == 0) {
        const int s = src_size[k] < 1 ? 1 : src_size[k];
        size[k] = s;
        invn[k] = inv_length(n2);
        locality[k] = src_loc ? src_loc[k] : (float)s;
        access[k] = src_acc ? src_acc[k] : 0u;
    }
}

// Finalize: per query, max over the slice keys; then either the key names the row (nothing to read), or it
// names a group of four consecutive rows: their exact cosines (one wave per row; strict ">" in ascending
// row order, so the lowest index keeps a tie); then the strict threshold test.  One 256-thread block
// per query.  `vec` = rows are 16-byte aligned and a whole number of 16-byte chunks.
// The thresholds of a call travel as kernel arguments (nothing to allocate or copy): out_hit[q * m + j] = 1 where
// the similarity of query q exceeds v[j]; the hits at v[count_at] are the references that access counts.
struct ThetaList {
    float v[SISO_MULTI_MAX];
    int m, count_at;
};

template <typename T>
__global__ __launch_bounds__(256) void k_lookup_finalize(const T *__restrict__ Q, const T *__restrict__ cent,
                                                          const float *__restrict__ invn, const u64 *__restrict__ keys,
                                                          long n, long K, int d, int slices, ThetaList thetas, int vec,
                                                          int key_kind, int *out_idx, float *out_sim,
                                                          unsigned char *out_hit, unsigned *access,
                                                          const float *__restrict__ q_inv, int *upd_owner,
                                                          int *upd_members) {
    constexpr int EPC = 16 / (int)sizeof(T);  // elements per 16-byte chunk
    __shared__ float sh_f[4];
    __shared__ u64 sh_k[4];
    __shared__ float sh_s[16];
    __shared__ long sh_i[16];
    __shared__ u32x4_t sh_q[SISO_MAX_DIM / EPC];  // the query row
    const long q = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6, grp = t >> 4, gl = t & 15;
    const T *qrow = Q + (size_t)q * d;
    // 1/|q|: 0 for a zero-length query, NaN for a non-finite one
    float ss = 0.f;
    if (q_inv) {
        // 1 / |q| is given (the batch was quantised: Q is not read at all; such keys always name rows)
    } else if (vec) {  // the row also goes to LDS: sixteen groups of lanes will read it again
        for (int e = t * EPC; e < d; e += 256 * EPC) {
            const u32x4_t v = *(const u32x4_t *)(qrow + e);
            sh_q[e / EPC] = v;
            ss += chunk_dot(v, v, T());
        }
    } else {
        for (int e = t; e < d; e += 256) ss += widen(qrow[e]) * widen(qrow[e]);
    }
    u64 key = 0;
    for (int s = t; s < slices; s += 256) {
        const u64 k2 = keys[(size_t)q * slices + s];
        key = k2 > key ? k2 : key;
    }
    ss = wave_sum(ss);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const u64 o = __shfl_xor(key, off);
        key = o > key ? o : key;
    }
    if (lane == 0) {
        sh_f[wave] = ss;
        sh_k[wave] = key;
    }
    __syncthreads();
    const float qi = q_inv ? q_inv[q] : inv_length((sh_f[0] + sh_f[1]) + (sh_f[2] + sh_f[3]));
#pragma unroll
    for (int w = 0; w < 4; ++w) key = sh_k[w] > key ? sh_k[w] : key;

    long best_i = -1;
    float best_s = -INFINITY;
    const bool finite_q = qi == qi;
    if (key_kind == SISO_KEY_ROWS) {
        // the key names the row and carries <q, c> / |c| as the kernel summed it: nothing left to read
        if (finite_q && K > 0 && key != 0) {
            best_i = (long)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull));
            best_s = unordered_bits((unsigned)(key >> 32)) * qi;
        }
    } else if (finite_q && K > 0 && key != 0) {
        // the key names a group of four consecutive rows: one wave per row, its lanes share the row's chunks
        const long r = 4L * (long)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull)) + wave;
        float acc = 0.f;
        if (vec) {
            // both chunks of a lane in flight together; a row past the end reads the last row and is discarded
            const T *crow = cent + (size_t)(r < K ? r : K - 1) * d;
            for (int e0 = lane * EPC; e0 < d; e0 += 2 * 64 * EPC) {
                const int e1 = e0 + 64 * EPC;
                const u32x4_t c0v = *(const u32x4_t *)(crow + e0);
                const u32x4_t c1v = *(const u32x4_t *)(crow + (e1 < d ? e1 : 0));
                acc += chunk_dot(sh_q[e0 / EPC], c0v, T());
                const float part = chunk_dot(sh_q[(e1 < d ? e1 : 0) / EPC], c1v, T());
                acc += e1 < d ? part : 0.f;
            }
        } else if (r < K) {
            const T *crow = cent + (size_t)r * d;
            for (int e = lane; e < d; e += 64) acc += widen(qrow[e]) * widen(crow[e]);
        }
        acc = wave_sum(acc);
        const float sv = r < K ? acc * qi * invn[r] : __uint_as_float(0x7FC00000u);
        if (sv == sv) {  // a NaN never wins
            best_s = sv;
            best_i = r;
        }
    }
    if (gl == 0) {
        sh_s[grp] = best_s;
        sh_i[grp] = best_i;
    }
    __syncthreads();
    if (t == 0) {
        // rows ascend with the group number inside a pass, and pass 1 lies above pass 0
        // (with groups of four every wave holds one row, ascending with the wave: the 16 entries repeat them)
        for (int g = 1; g < (key_kind == SISO_KEY_ROWS ? 1 : 16); ++g) {
            const float os = sh_s[g];
            const long oi = sh_i[g];
            if (oi >= 0 && (best_i < 0 || os > best_s || (os == best_s && oi < best_i))) {
                best_s = os;
                best_i = oi;
            }
        }
        if (!finite_q) best_s = __uint_as_float(0x7FC00000u);
        out_idx[q] = (int)best_i;
        out_sim[q] = best_s;
        for (int j = 0; j < thetas.m; ++j) {
            const bool hit = best_i >= 0 && best_s > thetas.v[j];
            if (out_hit) out_hit[(size_t)q * thetas.m + j] = hit ? 1 : 0;
            // a hit is a reference to its centroid (access_count of Algorithm 1); infinity stays infinity
            if (hit && j == thetas.count_at && access && access[best_i] != SISO_ACCESS_INF) atomicAdd(&access[best_i], 1u);
            // siso_lookup_update on a large batch: the notes that k_update_mark would take (first member and
            // number of members of each centroid), taken here, a launch earlier
            if (hit && j == 0 && upd_owner) {
                atomicMin(&upd_owner[best_i], (int)q);
                atomicAdd(&upd_members[best_i], 1);
            }
        }
    }
}

// ============================================================================
// LDS-tiled fp32 GEMM core shared by the scalar lookup and scalar merge kernels:
// a 64 x 64 tile of dot products per 256-thread block, thread (ty, tx) owning
// rows ty*4..+4 of A and rows tx*4..+4 of B.
// ============================================================================
#define ST_M 64
#define ST_K 16

template <typename T>
__device__ __forceinline__ void scalar_tile(const T *__restrict__ A, long a0, long a_end, const T *__restrict__ B,
                                            long b0, long b_end, int d, float (*As)[ST_M + 4],
                                            float (*Bs)[ST_M + 4], float acc[4][4]) {
    const int t = threadIdx.x;
    const int tx = t & 15, ty = t >> 4;
    const int lr = t >> 2, lk = (t & 3) * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < d; k0 += ST_K) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int k = k0 + lk + e;
            const long ar = a0 + lr, br = b0 + lr;
            As[lk + e][lr] = (ar < a_end && k < d) ? widen(A[(size_t)ar * d + k]) : 0.f;
            Bs[lk + e][lr] = (br < b_end && k < d) ? widen(B[(size_t)br * d + k]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < ST_K; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
}

// Phase 1, scalar path: block (x = query tile, y = slice of the centroid range).
template <typename T>
__global__ __launch_bounds__(256) void k_lookup_scalar(const T *__restrict__ Q, const T *__restrict__ cent,
                                                        const float *__restrict__ invn, long n, long K, int d,
                                                        long rows_per_slice, int slices, u64 *keys, u64 *board) {
    __shared__ float As[ST_K][ST_M + 4];
    __shared__ float Bs[ST_K][ST_M + 4];
    // (a step that ends in k_finalize_update: the slots of its board are emptied here, a kernel ahead)
    if (board != nullptr && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < SISO_FOLD_BOARD) board[threadIdx.x] = 0;
    const long q0 = (long)blockIdx.x * ST_M;
    const int s = blockIdx.y;
    const long c_begin = (long)s * rows_per_slice;
    const long c_end = (c_begin + rows_per_slice < K) ? c_begin + rows_per_slice : K;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float best[4];
    long bidx[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        best[i] = -INFINITY;
        bidx[i] = -1;
    }
    for (long c0 = c_begin; c0 < c_end; c0 += ST_M) {
        float acc[4][4];
        scalar_tile(Q, q0, n, cent, c0, c_end, d, As, Bs, acc);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const long cidx = c0 + tx * 4 + j;
            if (cidx < c_end) {
                const float w = invn[cidx];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = acc[i][j] * w;
                    if (v > best[i]) {
                        best[i] = v;
                        bidx[i] = cidx;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            const float ov = __shfl_xor(best[i], off);
            const long oi = __shfl_xor(bidx[i], off);
            if (oi >= 0 && (bidx[i] < 0 || ov > best[i] || (ov == best[i] && oi < bidx[i]))) {
                best[i] = ov;
                bidx[i] = oi;
            }
        }
        const long q = q0 + ty * 4 + i;
        if (tx == 0 && q < n)
            keys[(size_t)q * slices + s] = bidx[i] < 0 ? 0ull : pack_key(best[i], (unsigned)bidx[i]);
    }
}

int siso_scalar_slices(const siso_cache *c, long n) {
    // enough blocks to fill the chip, at least one 64-row tile per slice
    const long qtiles = (n + ST_M - 1) / ST_M;
    const long ctiles = (c->count + ST_M - 1) / ST_M;
    long want = (2048 + qtiles - 1) / qtiles;
    if (want > ctiles) want = ctiles;
    if (want < 1) want = 1;
    if (want > 65535) want = 65535;
    return (int)want;
}

template <typename T>
static int scalar_launch_t(siso_cache *c, const void *queries, long n, int slices, u64 *keys) {
    const long ctiles = (c->count + ST_M - 1) / ST_M;
    const long rows_per_slice = ((ctiles + slices - 1) / slices) * ST_M;
    dim3 grid((unsigned)((n + ST_M - 1) / ST_M), (unsigned)slices);
    hipLaunchKernelGGL(k_lookup_scalar<T>, grid, dim3(256), 0, c->stream, (const T *)queries, (const T *)c->cent,
                       c->invn, n, c->count, c->dim, rows_per_slice, slices, keys, c->board_to_clear);
    c->board_to_clear = nullptr;  // taken
    return siso_check_hip(c, hipGetLastError(), "k_lookup_scalar");
}

int siso_scalar_launch(siso_cache *c, const void *queries, long n, int slices, u64 *keys) {
    return c->dtype == SISO_F32 ? scalar_launch_t<float>(c, queries, n, slices, keys)
                                : scalar_launch_t<bf16_t>(c, queries, n, slices, keys);
}

// Self-similarity, scalar path: block (x, y) = tile pair, upper triangle only.
template <typename T>
__global__ __launch_bounds__(256) void k_merge_scalar(const T *__restrict__ cent, const float *__restrict__ invn, long K,
                                                       int d, float threshold, int *out_pairs, long cap, u64 *counter) {
    if (blockIdx.x > blockIdx.y) return;
    __shared__ float As[ST_K][ST_M + 4];
    __shared__ float Bs[ST_K][ST_M + 4];
    const long i0 = (long)blockIdx.x * ST_M, j0 = (long)blockIdx.y * ST_M;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4];
    scalar_tile(cent, i0, K, cent, j0, K, d, As, Bs, acc);
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const long i = i0 + ty * 4 + a;
        const float wi = i < K ? invn[i] : 0.f;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const long j = j0 + tx * 4 + b;
            const float wj = j < K ? invn[j] : 0.f;
            const float s = acc[a][b] * wi * wj;
            emit_pair(i < j && j < K && s > threshold, (int)i, (int)j, out_pairs, cap, counter);
        }
    }
}

int siso_pairs_scalar_launch(siso_cache *c, const void *rows, const float *invn, long count, float threshold,
                             int *out_pairs, long cap, u64 *counter) {
    const unsigned tiles = (unsigned)((count + ST_M - 1) / ST_M);
    if (tiles > 65535u) return siso_fail(c, SISO_EINVAL, "scalar pair search handles at most %d rows", 65535 * ST_M);
    dim3 grid(tiles, tiles);
    if (c->dtype == SISO_F32)
        hipLaunchKernelGGL(k_merge_scalar<float>, grid, dim3(256), 0, c->stream, (const float *)rows, invn, count, c->dim,
                           threshold, out_pairs, cap, counter);
    else
        hipLaunchKernelGGL(k_merge_scalar<bf16_t>, grid, dim3(256), 0, c->stream, (const bf16_t *)rows, invn, count,
                           c->dim, threshold, out_pairs, cap, counter);
    return siso_check_hip(c, hipGetLastError(), "k_merge_scalar");
}

// ============================================================================
// centroid update: one block per query; the block of the first member of a
// centroid sums all members in ascending order and rewrites the centroid.
// ============================================================================
#define UPD_MAXE (SISO_MAX_DIM / 256)

// Large batches: every block searching the whole index array for the members of its centroid costs
// n^2 / 256 steps.  A first pass notes, per centroid, its first member and the number of its members;
// then only the first member's block does anything, and it looks through the index array only if
// there is more than one member (queries of one batch rarely share a centroid).
#define UPD_NO_OWNER 0x7FFFFFFF
__global__ void k_update_mark(const int *__restrict__ idx, const unsigned char *__restrict__ hit, long n, long count,
                              int *owner, int *members) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n || (hit && !hit[i])) return;
    const int k = idx[i];
    if (k < 0 || k >= count) return;
    atomicMin(&owner[k], (int)i);
    atomicAdd(&members[k], 1);
}
__global__ void k_update_mark_init(int *owner, int *members, long capacity) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < capacity) {
        owner[i] = UPD_NO_OWNER;
        members[i] = 0;
    }
}

// One member of a centroid: x = this thread's elements (t + 256 e) of the query; the query at unit length is
// added to acc (queries without length or with a non-finite element are passed over).  Uniform over the
// block.  Every operation is spelled out with its rounding, here and in update_write, so that k_update and
// k_finalize_update do the same arithmetic whatever the compiler would fuse in either of them.
template <int UPD_MAXE_T>
__device__ __forceinline__ bool fold_member(const float (&x)[UPD_MAXE_T], float (&acc)[UPD_MAXE_T], float *sh) {
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) ss = __fmaf_rn(x[e], x[e], ss);
    const float n2 = block_sum256(ss, sh);
    const float inv = inv_length(n2);
    if (!(inv == inv && inv > 0.f)) return false;
    const float nrm = sqrtf(n2);
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) acc[e] = __fadd_rn(acc[e], __fdiv_rn(x[e], nrm));
    return true;
}

// The end of an update, by the block that leads centroid k: acc = the sum of its `members` unit-length members
// (this thread's elements t + 256 e), m_old / size_old = the mean and its weight as they were.  Writes the
// new mean and weight, the stored row (the mean at unit length, rounded to the storage type; left alone when
// the mean has no length: false then) and its inverse length; `stored` receives this thread's elements of the
// stored row.
template <typename T, int UPD_MAXE_T>
__device__ __forceinline__ bool update_write(int k, int d, int size_old, int members, const float (&m_old)[UPD_MAXE_T],
                                             const float (&acc)[UPD_MAXE_T], T *cent, float *mean, int *size, float *invn,
                                             float *sh, float (&stored)[UPD_MAXE_T]) {
    const int t = threadIdx.x;
    const float n_old = (float)size_old;
    const float n_new = n_old + (float)members;
    float m[UPD_MAXE_T];
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        const int col = t + e * 256;
        m[e] = 0.f;
        if (col < d) {
            m[e] = __fdiv_rn(__fmaf_rn(n_old, m_old[e], acc[e]), n_new);
            mean[(size_t)k * d + col] = m[e];
            ss = __fmaf_rn(m[e], m[e], ss);
        }
    }
    const float n2 = block_sum256(ss, sh);
    if (t == 0) size[k] = size_old + members;
    if (!(n2 > 0.f) || n2 > 3.0e38f) return false;
    const float nrm = sqrtf(n2);
    float cs = 0.f;
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        const int col = t + e * 256;
        stored[e] = 0.f;
        if (col < d) {
            T r;
            narrow(__fdiv_rn(m[e], nrm), &r);
            cent[(size_t)k * d + col] = r;
            const float back = widen(r);
            stored[e] = back;
            cs = __fmaf_rn(back, back, cs);
        }
    }
    const float c2 = block_sum256(cs, sh);
    if (t == 0) invn[k] = inv_length(c2);
    return true;
}

// UPD_MAXE_T = elements of a row per thread (4 for dim <= 1024, else 16).  owner / marked = the notes
// of k_update_mark, or NULL: then every block finds out by itself whether it is the first member.
template <typename T, int UPD_MAXE_T>
__global__ __launch_bounds__(256) void k_update(const T *__restrict__ Q, const int *__restrict__ idx,
                                                 const unsigned char *__restrict__ hit, long n, T *cent, float *mean,
                                                 int *size, float *invn, long count, int d, u64 *bad, int *owner,
                                                 int *marked) {
    __shared__ float sh[4];
    __shared__ u64 masks[4];
    const long me = blockIdx.x;
    const int t = threadIdx.x;
    // what does not depend on anything else is asked for first: the first 256 entries of the index
    // array (all of it in a small batch), this block's own entry
    const bool first_ok = !owner && t < n;
    const int first_idx = first_ok ? idx[t] : -1;
    const unsigned char first_hit = first_ok && hit ? hit[t] : 1;
    if (hit && !hit[me]) return;
    const int k = idx[me];
    if (k < 0) return;
    if (k >= count) {
        if (t == 0) atomicAdd(bad, 1ull);
        return;
    }
    // ... then this block's own query and the centroid's mean, before it is known whether this block
    // leads the centroid: most do, and the rows are on their way while the notes are read
    // (without notes the two loads read this block's own index entry instead: no branch, no wait here)
    const int lead_raw = *(owner ? owner + k : idx + me);
    const int noted_raw = *(owner ? marked + k : idx + me);
    // loads without conditions (a column past the end reads column 0 and is zeroed afterwards), so
    // that all of them are in flight together
    float x_me[UPD_MAXE_T], m_old[UPD_MAXE_T];
    T xr[UPD_MAXE_T];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        const int col = t + e * 256;
        xr[e] = Q[(size_t)me * d + (col < d ? col : 0)];
        m_old[e] = mean[(size_t)k * d + (col < d ? col : 0)];
    }
    const int size_old = size[k];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        x_me[e] = t + e * 256 < d ? widen(xr[e]) : 0.f;
        // the values exist from here on: otherwise the compiler moves the loads behind the test below,
        // where they would only start once the notes have arrived
        asm volatile("" ::"v"(x_me[e]), "v"(m_old[e]));
    }
    const long scan_from = 0, scan_to = n;
    if (owner && lead_raw != (int)me) return;  // an earlier member leads this centroid
    const bool alone = owner && noted_raw == 1;  // the only member: nothing to look for
    if (owner) {
        __syncthreads();  // everyone has read the notes
        if (t == 0) {     // leave them as they were found
            owner[k] = UPD_NO_OWNER;
            marked[k] = 0;
        }
    }
    float acc[UPD_MAXE_T];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) acc[e] = 0.f;
    int members = 0;
    // fold one query (its elements of this thread in x) into the sum; uniform over the block
    auto fold = [&](const float(&x)[UPD_MAXE_T]) {
        if (fold_member<UPD_MAXE_T>(x, acc, sh)) ++members;
    };
    if (alone) {
        fold(x_me);
    } else {
        for (long base = scan_from; base < scan_to; base += 256) {
            const long j = base + t;
            bool m;
            if (base == 0 && !owner)
                m = first_ok && first_idx == k && first_hit;
            else
                m = j < scan_to && idx[j] == k && (!hit || hit[j]);
            const u64 mask = __ballot(m);
            __syncthreads();
            if ((t & 63) == 0) masks[t >> 6] = mask;
            __syncthreads();
            for (int w = 0; w < 4; ++w) {
                u64 mm = masks[w];
                while (mm) {
                    const int b = __ffsll((long long)mm) - 1;
                    mm &= mm - 1;
                    const long jj = base + w * 64 + b;
                    if (jj < me) return;  // an earlier member leads this centroid (uniform over the block)
                    if (jj == me) {
                        fold(x_me);
                        continue;
                    }
                    T xr[UPD_MAXE_T];
                    float x[UPD_MAXE_T];
#pragma unroll
                    for (int e = 0; e < UPD_MAXE_T; ++e) {
                        const int col = t + e * 256;
                        xr[e] = Q[(size_t)jj * d + (col < d ? col : 0)];
                    }
#pragma unroll
                    for (int e = 0; e < UPD_MAXE_T; ++e) x[e] = t + e * 256 < d ? widen(xr[e]) : 0.f;
                    fold(x);
                }
            }
        }
    }
    if (members == 0) return;
    float stored[UPD_MAXE_T];
    update_write<T, UPD_MAXE_T>(k, d, size_old, members, m_old, acc, cent, mean, size, invn, sh, stored);
}

// ============================================================================
// The end of a small lookup and the update of its hits as one kernel (siso_lookup_update, at most 256
// queries, keys that name rows): block q does what k_lookup_finalize does for query q, then what k_update
// does for it, with the same arithmetic in the same order, so the outputs and the state are those of the
// two kernels bit for bit.  What a block needs from the others is their (index, hit) - to know whether it
// leads its centroid and which other queries fold into it - and that crosses the grid through a board of
// one 64-bit slot per query: (written, hit, index), written and read with device-scope atomic operations.
// The slots are emptied by the kernel before this one - the first phase of the same lookup, whose first
// block does it when siso_lookup_update asks for it - so the end of that kernel stands between the emptying
// and the first entry, also when the launches are replayed from a captured graph, and no fence is needed
// (the rows and means the blocks read were written by earlier kernels too).  All blocks of the grid
// are resident together (at most 256 small blocks), so the wait for the slots ends; it is bounded all the
// same: a block that gives up leaves its centroid as it was and counts its query as not applied.
// Saves a launch and the gap before it, and the loads of the update (own row, mean of the centroid) are on
// their way while the block waits for the board.
// With an 8-bit serving copy (siso_fp8_lookup_update) the keys and 1/|q| are the copy's, the centroid arrays the
// bf16 master's, and the block that rewrites a centroid quantises the new stored row into the copy as well
// (fp8_store_row: what k_fp8_quantize would store).
// ============================================================================
__device__ __forceinline__ u64 board_entry(bool hit, int idx) {
    return (1ull << 63) | ((u64)(hit ? 1 : 0) << 32) | (u64)(unsigned)idx;
}
template <typename T, int UPD_MAXE_T>
__global__ __launch_bounds__(256) void k_finalize_update(const T *__restrict__ Q, const u64 *__restrict__ keys, long n, long K,
                                                          int d, int slices, float theta, int vec, int *out_idx,
                                                          float *out_sim, unsigned char *out_hit, unsigned *access, T *cent,
                                                          float *mean, int *size, float *invn, u64 *board,
                                                          int spin_limit, u64 *gave_up, const float *__restrict__ q_inv,
                                                          unsigned char *copy_codes, float *copy_scale, float *copy_inv,
                                                          int *copy_size) {
    constexpr int EPC = 16 / (int)sizeof(T);
    __shared__ float sh[4];
    __shared__ float sh_f[4];
    __shared__ u64 sh_k[4];
    __shared__ u64 masks[4];
    __shared__ u64 sh_board[SISO_FOLD_BOARD];
    __shared__ int sh_all;
    const long me = blockIdx.x;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const T *qrow = Q + (size_t)me * d;
    // this block's own query in the layout of the update, asked for first
    T xr[UPD_MAXE_T];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        const int col = t + e * 256;
        xr[e] = qrow[col < d ? col : 0];
    }
    // --- k_lookup_finalize for keys that name rows: 1/|q| (given, if the batch was quantised) and the largest key
    float ss = 0.f;
    if (q_inv) {
    } else if (vec) {
        for (int e = t * EPC; e < d; e += 256 * EPC) {
            const u32x4_t v = *(const u32x4_t *)(qrow + e);
            ss += chunk_dot(v, v, T());
        }
    } else {
        for (int e = t; e < d; e += 256) ss += widen(qrow[e]) * widen(qrow[e]);
    }
    u64 key = 0;
    for (int s = t; s < slices; s += 256) {
        const u64 k2 = keys[(size_t)me * slices + s];
        key = k2 > key ? k2 : key;
    }
    ss = wave_sum(ss);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const u64 o = __shfl_xor(key, off);
        key = o > key ? o : key;
    }
    if (lane == 0) {
        sh_f[wave] = ss;
        sh_k[wave] = key;
    }
    __syncthreads();
    const float qi = q_inv ? q_inv[me] : inv_length((sh_f[0] + sh_f[1]) + (sh_f[2] + sh_f[3]));
#pragma unroll
    for (int w = 0; w < 4; ++w) key = sh_k[w] > key ? sh_k[w] : key;
    long best_i = -1;
    float best_s = -INFINITY;
    const bool finite_q = qi == qi;
    if (finite_q && K > 0 && key != 0) {
        best_i = (long)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull));
        best_s = unordered_bits((unsigned)(key >> 32)) * qi;
    }
    if (!finite_q) best_s = __uint_as_float(0x7FC00000u);
    const bool hit = best_i >= 0 && best_s > theta;
    if (t == 0) {
        out_idx[me] = (int)best_i;
        out_sim[me] = best_s;
        out_hit[me] = hit ? 1 : 0;
        if (hit && access && access[best_i] != SISO_ACCESS_INF) atomicAdd(&access[best_i], 1u);
        __hip_atomic_store(board + me, board_entry(hit, (int)best_i), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (!hit) return;
    // --- k_update for query `me`: its centroid's mean and weight, on their way during the wait
    const int k = (int)best_i;
    float x_me[UPD_MAXE_T], m_old[UPD_MAXE_T];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        const int col = t + e * 256;
        m_old[e] = mean[(size_t)k * d + (col < d ? col : 0)];
    }
    const int size_old = size[k];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) {
        x_me[e] = t + e * 256 < d ? widen(xr[e]) : 0.f;
        asm volatile("" ::"v"(x_me[e]), "v"(m_old[e]));  // (the loads are issued here, not behind the wait)
    }
    // the board: wave 0 reads the slots until all of them are written
    if (wave == 0) {
        bool all = false;
        for (int tries = 0; tries < spin_limit && !all; ++tries) {
            bool mine = true;
            for (int j = lane; j < (int)n; j += 64) {
                const u64 v = __hip_atomic_load(board + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sh_board[j] = v;
                mine = mine && (v >> 63) != 0;
            }
            all = __ballot(!mine) == 0;
            if (!all) __builtin_amdgcn_s_sleep(4);
        }
        if (lane == 0) sh_all = all ? 1 : 0;
    }
    __syncthreads();
    if (!sh_all) {
        if (t == 0) atomicAdd(gave_up, 1ull);
        return;
    }
    float acc[UPD_MAXE_T];
#pragma unroll
    for (int e = 0; e < UPD_MAXE_T; ++e) acc[e] = 0.f;
    int members = 0;
    auto fold = [&](const float(&x)[UPD_MAXE_T]) {
        if (fold_member<UPD_MAXE_T>(x, acc, sh)) ++members;
    };
    // the members of centroid k in ascending order (a hit whose index is k)
    const bool m = t < (int)n && sh_board[t] == board_entry(true, k);
    const u64 mask = __ballot(m);
    if (lane == 0) masks[wave] = mask;
    __syncthreads();
    for (int w = 0; w < 4; ++w) {
        u64 mm = masks[w];
        while (mm) {
            const int b = __ffsll((long long)mm) - 1;
            mm &= mm - 1;
            const long jj = w * 64 + b;
            if (jj < me) return;  // an earlier member leads this centroid (uniform over the block)
            if (jj == me) {
                fold(x_me);
                continue;
            }
            T yr[UPD_MAXE_T];
            float x[UPD_MAXE_T];
#pragma unroll
            for (int e = 0; e < UPD_MAXE_T; ++e) {
                const int col = t + e * 256;
                yr[e] = Q[(size_t)jj * d + (col < d ? col : 0)];
            }
#pragma unroll
            for (int e = 0; e < UPD_MAXE_T; ++e) x[e] = t + e * 256 < d ? widen(yr[e]) : 0.f;
            fold(x);
        }
    }
    if (members == 0) return;
    float stored[UPD_MAXE_T];
    const bool rewritten = update_write<T, UPD_MAXE_T>(k, d, size_old, members, m_old, acc, cent, mean, size, invn, sh, stored);
    if (copy_codes) {  // the 8-bit copy follows
        if (t == 0) copy_size[k] = size_old + members;
        if (rewritten) fp8_store_row<UPD_MAXE_T>(stored, d, copy_codes + (size_t)k * d, copy_scale + k, copy_inv + k, sh);
    }
}


// ============================================================================
// group merge: lock-free union-find (the lower index becomes the root), group
// means by the group's root, stable compaction.
// ============================================================================
__global__ void k_pairs_validate(const int *__restrict__ pairs, long n_pairs, long K, u64 *bad) {
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pairs) return;
    const int a = pairs[2 * p], b = pairs[2 * p + 1];
    if (a < 0 || b < 0 || a >= K || b >= K || a == b) atomicAdd(bad, 1ull);
}

__global__ void k_uf_init(int *parent, unsigned char *touched, int *members_of, int *cursor, long K) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K) {
        parent[i] = (int)i;
        touched[i] = 0;
        members_of[i] = 0;
        cursor[i] = 0;
    }
}

// Member lists of the groups: how many rows each root leads (itself included), then, once the counts
// have been scanned into list starts, the rows themselves (in the order they arrive; the root's block
// sorts its list).  Only rows that occur in a pair take part.
__global__ void k_group_count(const int *__restrict__ root, const unsigned char *__restrict__ touched, long K,
                              int *members_of) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K && touched[i]) atomicAdd(&members_of[root[i]], 1);
}
__global__ void k_group_fill(const int *__restrict__ root, const unsigned char *__restrict__ touched, long K,
                             const int *__restrict__ first, int *cursor, int *list) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= K || !touched[i]) return;
    const int r = root[i];
    list[first[r] + atomicAdd(&cursor[r], 1)] = (int)i;
}

__device__ __forceinline__ int uf_find(const int *parent, int x) {
    int p = __atomic_load_n(parent + x, __ATOMIC_RELAXED);
    while (p != x) {
        x = p;
        p = __atomic_load_n(parent + x, __ATOMIC_RELAXED);
    }
    return x;
}

// Parents only ever decrease, so every retry makes progress and the loop ends.
__global__ void k_uf_hook(const int *__restrict__ pairs, long n_pairs, int *parent, unsigned char *touched) {
    const long p = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= n_pairs) return;
    int a = pairs[2 * p], b = pairs[2 * p + 1];
    touched[a] = 1;
    touched[b] = 1;
    for (;;) {
        a = uf_find(parent, a);
        b = uf_find(parent, b);
        if (a == b) break;
        const int hi = a > b ? a : b, lo = a > b ? b : a;
        const int old = atomicCAS(parent + hi, hi, lo);
        if (old == hi) break;
        a = old;  // someone re-parented hi meanwhile: continue from there
        b = lo;
    }
}

__global__ void k_uf_roots(const int *__restrict__ parent, int *root, long K) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K) root[i] = uf_find(parent, (int)i);
}

// One block per row; only roots of groups with at least two rows work.
#define GROUP_LIST_MAX 1024  // members of a group that its block sorts in LDS; larger groups are searched for
template <typename T>
__global__ __launch_bounds__(256) void k_group_mean(const int *__restrict__ root, const unsigned char *__restrict__ touched,
                                                     long K, const int *__restrict__ members_of,
                                                     const int *__restrict__ first, const int *__restrict__ list,
                                                     T *cent, float *mean, int *size, float *invn,
                                                     float *locality, unsigned *access, int d) {
    __shared__ float sh[4];
    __shared__ u64 masks[4];
    __shared__ int raw[GROUP_LIST_MAX], sorted[GROUP_LIST_MAX];
    const long r = blockIdx.x;
    const int t = threadIdx.x;
    if (!touched[r] || root[r] != (int)r) return;
    float acc[UPD_MAXE];
#pragma unroll
    for (int e = 0; e < UPD_MAXE; ++e) acc[e] = 0.f;
    double wsum = 0.0;
    int members = 0;
    float loc = 0.f;  // cluster sizes of Algorithm 1 add up, in ascending order of the members
    u64 refs = 0;     // so do the access counts, saturating at infinity
    auto take = [&](long jj) {
        const float wgt = (float)size[jj];
#pragma unroll
        for (int e = 0; e < UPD_MAXE; ++e) {
            const int col = t + e * 256;
            if (col < d) acc[e] += wgt * mean[(size_t)jj * d + col];
        }
        wsum += (double)size[jj];
        loc = loc + locality[jj];
        refs += access[jj];
        ++members;
    };
    const int listed = members_of[r];
    if (listed <= GROUP_LIST_MAX) {
        // the list arrives in no particular order; the sums take the members in ascending order, so the
        // result does not depend on scheduling: every thread places its entries by counting the smaller ones
        const int lo = first[r];
        for (int i = t; i < listed; i += 256) raw[i] = list[lo + i];
        __syncthreads();
        for (int i = t; i < listed; i += 256) {
            const int mine = raw[i];
            int below = 0;
            for (int k = 0; k < listed; ++k) below += raw[k] < mine ? 1 : 0;
            sorted[below] = mine;
        }
        __syncthreads();
        for (int p = 0; p < listed; ++p) take(sorted[p]);
    } else
    for (long base = r - (r & 255); base < K; base += 256) {
        const long j = base + t;
        const bool m = j < K && j >= r && root[j] == (int)r;
        const u64 mask = __ballot(m);
        __syncthreads();
        if ((t & 63) == 0) masks[t >> 6] = mask;
        __syncthreads();
        for (int w = 0; w < 4; ++w) {
            u64 mm = masks[w];
            while (mm) {
                const int b = __ffsll((long long)mm) - 1;
                mm &= mm - 1;
                take(base + w * 64 + b);
            }
        }
    }
    if (members < 2) return;
    const float wtot = (float)wsum;
    float m[UPD_MAXE];
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < UPD_MAXE; ++e) {
        const int col = t + e * 256;
        m[e] = 0.f;
        if (col < d) {
            m[e] = acc[e] / wtot;
            mean[(size_t)r * d + col] = m[e];
            ss += m[e] * m[e];
        }
    }
    const float n2 = block_sum256(ss, sh);
    if (t == 0) {
        size[r] = wsum > 2147483647.0 ? 2147483647 : (int)wsum;
        locality[r] = loc;
        access[r] = refs >= (u64)SISO_ACCESS_INF ? SISO_ACCESS_INF : (unsigned)refs;
    }
    if (!(n2 > 0.f) || n2 > 3.0e38f) return;
    const float nrm = sqrtf(n2);
    float cs = 0.f;
#pragma unroll
    for (int e = 0; e < UPD_MAXE; ++e) {
        const int col = t + e * 256;
        if (col < d) {
            T v;
            narrow(m[e] / nrm, &v);
            cent[(size_t)r * d + col] = v;
            const float back = widen(v);
            cs += back * back;
        }
    }
    const float c2 = block_sum256(cs, sh);
    if (t == 0) invn[r] = inv_length(c2);
}

// Exclusive scan by one 1024-thread block, four entries per thread and trip; total -> *total.
// The entries are vals[i], or, without vals, the flags "row i survives" (root[i] == i).
__global__ __launch_bounds__(1024) void k_scan_exclusive(const int *__restrict__ vals, const int *__restrict__ root, long K,
                                                          int *out, u64 *total) {
    __shared__ int wsum[16];
    __shared__ int carry_s;
    const int t = threadIdx.x, lane = t & 63, w = t >> 6;
    if (t == 0) carry_s = 0;
    __syncthreads();
    for (long base = 0; base < K; base += 4096) {
        const long i0 = base + 4 * t;
        int v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const long i = i0 + k;
            v[k] = i < K ? (vals ? vals[i] : (root[i] == (int)i ? 1 : 0)) : 0;
        }
        const int mine = (v[0] + v[1]) + (v[2] + v[3]);
        int incl = mine;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off);
            if (lane >= off) incl += o;
        }
        if (lane == 63) wsum[w] = incl;
        __syncthreads();
        int before = carry_s;
        for (int k = 0; k < w; ++k) before += wsum[k];
        int run = before + incl - mine;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i0 + k < K) out[i0 + k] = run;
            run += v[k];
        }
        __syncthreads();
        if (t == 1023) carry_s = before + incl;
        __syncthreads();
    }
    if (total && t == 0) *total = (u64)carry_s;
}
template <typename T>
__global__ __launch_bounds__(256) void k_gather_rows(const int *__restrict__ root, const int *__restrict__ newpos,
                                                      const T *__restrict__ cent, const float *__restrict__ mean,
                                                      const int *__restrict__ size, const float *__restrict__ invn,
                                                      const float *__restrict__ locality,
                                                      const unsigned *__restrict__ access, T *cent2, float *mean2,
                                                      int *size2, float *invn2, float *locality2, unsigned *access2,
                                                      int d) {
    const long i = blockIdx.x;
    if (root[i] != (int)i) return;
    const long p = newpos[i];
    for (int e = threadIdx.x; e < d; e += 256) {
        cent2[(size_t)p * d + e] = cent[(size_t)i * d + e];
        mean2[(size_t)p * d + e] = mean[(size_t)i * d + e];
    }
    if (threadIdx.x == 0) {
        size2[p] = size[i];
        invn2[p] = invn[i];
        locality2[p] = locality[i];
        access2[p] = access[i];
    }
}

__global__ void k_survivor_map(const int *__restrict__ root, const int *__restrict__ newpos, long K, int *out) {
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < K) out[i] = newpos[root[i]];
}

// ============================================================================
// C ABI
// ============================================================================
// Key workspace of siso_lookup_static: part of the library's image, so a caller that must not allocate
// (graph capture, a serving loop, a harness that forbids it) still has room for the phase-1 keys.  Every
// GPU the library runs on holds its own copy at its own address until the process ends; in host code the
// array's name is only a handle for hipGetSymbolAddress, never an address to pass on.
#define SISO_STATIC_KEYS (1L << 20)  // 8 MiB
static __device__ __align__(256) u64 scratch[SISO_STATIC_KEYS];
#define SISO_MAX_DEVICES 64
static u64 *scratch_ptr[SISO_MAX_DEVICES];  // device address of `scratch` per device, resolved by siso_create_ex

// the current device's copy of the array (the device must be current)
static int resolve_scratch(int device, u64 **out) {
    *out = nullptr;
    if (device < 0 || device >= SISO_MAX_DEVICES) return SISO_EINVAL;
    if (!scratch_ptr[device]) {
        u64 *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return SISO_EHIP;
        }
        scratch_ptr[device] = ptr;
    }
    *out = scratch_ptr[device];
    return SISO_OK;
}

static int ensure_workspace(siso_cache *c, long n, int slices) {
    const long need_keys = n * (long)slices;
    if (need_keys > c->keys_cap) {
        if (c->keys) {
            HIP_TRY(c, hipStreamSynchronize(c->stream));
            HIP_TRY(c, hipFree(c->keys));
            c->keys = nullptr;
            c->keys_cap = 0;
        }
        if (hipMalloc((void **)&c->keys, (size_t)need_keys * sizeof(u64)) != hipSuccess) {
            (void)hipGetLastError();
            return siso_fail(c, SISO_ENOMEM, "workspace of %ld keys", need_keys);
        }
        c->keys_cap = need_keys;
    }
    return SISO_OK;
}

int siso_ensure_keys(siso_cache *c, long need) { return ensure_workspace(c, need, 1); }

int siso_second_set(siso_cache *c) {
    if (c->cent_b) return SISO_OK;
    const size_t cells = (size_t)c->capacity * c->dim;
    const size_t cent_bytes = (cells + (size_t)SISO_PAD_ROWS * c->dim) * elem_bytes(c->dtype);
    bool ok = hipMalloc(&c->cent_b, cent_bytes) == hipSuccess;
    ok = ok && hipMemset(c->cent_b, 0, cent_bytes) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->mean_b, cells * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->size_b, (size_t)c->capacity * sizeof(int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->invn_b, ((size_t)c->capacity + SISO_PAD_ROWS) * sizeof(float)) == hipSuccess;
    ok = ok && hipMemset(c->invn_b, 0, ((size_t)c->capacity + SISO_PAD_ROWS) * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->locality_b, (size_t)c->capacity * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->access_b, (size_t)c->capacity * sizeof(unsigned)) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        if (c->cent_b) (void)hipFree(c->cent_b);
        if (c->mean_b) (void)hipFree(c->mean_b);
        if (c->size_b) (void)hipFree(c->size_b);
        if (c->invn_b) (void)hipFree(c->invn_b);
        if (c->locality_b) (void)hipFree(c->locality_b);
        if (c->access_b) (void)hipFree(c->access_b);
        c->cent_b = nullptr;
        c->mean_b = nullptr;
        c->size_b = nullptr;
        c->invn_b = nullptr;
        c->locality_b = nullptr;
        c->access_b = nullptr;
        return siso_fail(c, SISO_ENOMEM, "second set of arrays for %ld centroids", c->capacity);
    }
    return SISO_OK;
}

// Work already enqueued keeps the pointers it was launched with; work enqueued from now on sees the new set.
void siso_swap_sets(siso_cache *c) {
    std::swap(c->cent, c->cent_b);
    std::swap(c->mean, c->mean_b);
    std::swap(c->size, c->size_b);
    std::swap(c->invn, c->invn_b);
    std::swap(c->locality, c->locality_b);
    std::swap(c->access, c->access_b);
}

extern "C" int siso_create_ex(int dim, long capacity, int dtype, siso_cache **out) {
    if (!out) return SISO_EINVAL;
    *out = nullptr;
    if (dim < 1 || dim > SISO_MAX_DIM || capacity < 1 || capacity > 2147483647L ||
        (dtype != SISO_F32 && dtype != SISO_BF16 && dtype != SISO_FP8))
        return SISO_EINVAL;
    if (dtype == SISO_FP8 && (dim % 128 != 0 || dim < 256)) return SISO_EINVAL;  // slabs of 128 codes, two per tile
    siso_cache *c = new (std::nothrow) siso_cache();
    if (!c) return SISO_ENOMEM;
    memset(c, 0, sizeof(*c));
    c->opt_fold_spin_limit = -1;
    c->dim = dim;
    c->capacity = capacity;
    c->dtype = dtype;
    c->path = SISO_PATH_AUTO;
    const size_t cells = (size_t)capacity * dim;
    bool ok = hipGetDevice(&c->device) == hipSuccess;
    ok = ok && resolve_scratch(c->device, &c->static_keys) == SISO_OK;
    // The stored centroids carry SISO_PAD_ROWS readable rows past the capacity, so that the
    // tiled kernels may load a whole last tile; their results are discarded.
    const size_t cent_bytes = (cells + (size_t)SISO_PAD_ROWS * dim) * elem_bytes(dtype);
    ok = ok && hipMalloc(&c->cent, cent_bytes) == hipSuccess;
    ok = ok && hipMemset(c->cent, 0, cent_bytes) == hipSuccess;
    if (dtype == SISO_FP8) ok = ok && hipMalloc((void **)&c->scale, (size_t)capacity * sizeof(float)) == hipSuccess;
    else ok = ok && hipMalloc((void **)&c->mean, cells * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->size, (size_t)capacity * sizeof(int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->invn, ((size_t)capacity + SISO_PAD_ROWS) * sizeof(float)) == hipSuccess;
    ok = ok && hipMemset(c->invn, 0, ((size_t)capacity + SISO_PAD_ROWS) * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->locality, (size_t)capacity * sizeof(float)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->access, (size_t)capacity * sizeof(unsigned)) == hipSuccess;
    // (behind the four counters: the board of siso_lookup_update, one slot per query of a small batch)
    ok = ok && hipMalloc((void **)&c->counters, (4 + SISO_FOLD_BOARD) * sizeof(u64)) == hipSuccess;
    ok = ok && hipHostMalloc((void **)&c->host_pin, 4 * sizeof(u64), hipHostMallocDefault) == hipSuccess;
    ok = ok && hipMemset(c->counters, 0, (4 + SISO_FOLD_BOARD) * sizeof(u64)) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        siso_destroy(c);
        return SISO_ENOMEM;
    }
    *out = c;
    return SISO_OK;
}

extern "C" int siso_create(int dim, long capacity, siso_cache **out) {
    return siso_create_ex(dim, capacity, SISO_BF16, out);
}

extern "C" void siso_destroy(siso_cache *c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    if (c->cent) (void)hipFree(c->cent);
    if (c->mean) (void)hipFree(c->mean);
    if (c->size) (void)hipFree(c->size);
    if (c->invn) (void)hipFree(c->invn);
    if (c->locality) (void)hipFree(c->locality);
    if (c->upd_owner) (void)hipFree(c->upd_owner);
    if (c->upd_members) (void)hipFree(c->upd_members);
    if (c->access) (void)hipFree(c->access);
    if (c->cent_b) (void)hipFree(c->cent_b);
    if (c->mean_b) (void)hipFree(c->mean_b);
    if (c->size_b) (void)hipFree(c->size_b);
    if (c->invn_b) (void)hipFree(c->invn_b);
    if (c->locality_b) (void)hipFree(c->locality_b);
    if (c->access_b) (void)hipFree(c->access_b);
    if (c->keys) (void)hipFree(c->keys);
    if (c->scale) (void)hipFree(c->scale);
    if (c->fp8_q) (void)hipFree(c->fp8_q);
    if (c->fp8_qinv) (void)hipFree(c->fp8_qinv);
    if (c->topk_tau) (void)hipFree(c->topk_tau);
    if (c->topk_cnt) (void)hipFree(c->topk_cnt);
    if (c->topk_cand) (void)hipFree(c->topk_cand);
    if (c->counters) (void)hipFree(c->counters);
    if (c->host_pin) (void)hipHostFree(c->host_pin);
    if (c->prof_ev) {
        for (int i = 0; i < 2 * SISO_PROF_MAX; ++i)
            if (c->prof_ev[i]) (void)hipEventDestroy(c->prof_ev[i]);
        free(c->prof_ev);
    }
    delete c;
}

extern "C" int siso_set_stream(siso_cache *c, void *hip_stream) {
    if (!c) return SISO_EINVAL;
    c->stream = (hipStream_t)hip_stream;
    return SISO_OK;
}

extern "C" int siso_set_lookup_path(siso_cache *c, int path) {
    if (!c) return SISO_EINVAL;
    if (c->dtype == SISO_FP8 && path == SISO_PATH_SCALAR) return siso_fail(c, SISO_EINVAL, "the 8-bit storage has no scalar kernel");
    if (path < SISO_PATH_AUTO || path > SISO_PATH_SKINNY) return siso_fail(c, SISO_EINVAL, "unknown lookup path %d", path);
    c->path = path;
    return SISO_OK;
}

extern "C" int siso_set_option(siso_cache *c, const char *name, long value) {
    if (!c || !name) return SISO_EINVAL;
    if (!strcmp(name, "fold_spin_limit") && value == -1) {
        c->opt_fold_spin_limit = -1;
        return SISO_OK;
    }
    if (value < 0 || value > 1000000) return siso_fail(c, SISO_EINVAL, "option %s: value %ld out of range", name, value);
    if (!strcmp(name, "mfma_config")) c->opt_mfma_config = (int)value;
    else if (!strcmp(name, "tiles_per_slice")) c->opt_tiles_per_slice = (int)value;
    else if (!strcmp(name, "merge_config")) c->opt_merge_config = (int)value;
    else if (!strcmp(name, "mfma_qblock")) c->opt_mfma_qblock = (int)value;
    else if (!strcmp(name, "fold_spin_limit")) c->opt_fold_spin_limit = (int)value;
    else if (!strcmp(name, "stream_hint") && value <= 2) c->opt_stream_hint = (int)value;
    else if (!strcmp(name, "second_set")) return value ? siso_second_set(c) : SISO_OK;
    else return siso_fail(c, SISO_EINVAL, "unknown option %s", name);
    return SISO_OK;
}

extern "C" long siso_count(const siso_cache *c) { return c ? c->count : (long)SISO_EINVAL; }

extern "C" const char *siso_last_error(const siso_cache *c) { return c ? c->err : "null cache"; }

__global__ void k_fill_nan(float *p, int count);

extern "C" int siso_load(siso_cache *c, const void *centroids, const int *counts, long k) {
    if (!c) return SISO_EINVAL;
    if (k < 0 || (k > 0 && !centroids)) return siso_fail(c, SISO_EINVAL, "siso_load: bad arguments");
    if (k > c->capacity) return siso_fail(c, SISO_ECAPACITY, "siso_load: %ld rows exceed capacity %ld", k, c->capacity);
    if (c->dtype == SISO_FP8) {
        const int rc = siso_fp8_load(c, centroids, counts, k);
        if (rc != SISO_OK) return rc;
    } else if (k > 0) {
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_load_rows<float>, dim3((unsigned)k), dim3(256), 0, c->stream, (const float *)centroids,
                               counts, (float *)c->cent, c->mean, c->size, c->invn, c->locality, c->access, c->dim);
        else
            hipLaunchKernelGGL(k_load_rows<bf16_t>, dim3((unsigned)k), dim3(256), 0, c->stream,
                               (const bf16_t *)centroids, counts, (bf16_t *)c->cent, c->mean, c->size, c->invn, c->locality,
                               c->access, c->dim);
        HIP_TRY(c, hipGetLastError());
    }
    hipLaunchKernelGGL(k_fill_nan, dim3(1), dim3(SISO_PAD_ROWS), 0, c->stream, c->invn + k, SISO_PAD_ROWS);
    HIP_TRY(c, hipGetLastError());
    c->count = k;
    return SISO_OK;
}

extern "C" int siso_import(siso_cache *c, const void *centroids, const float *means, const int *counts,
                           const float *cluster_size, const unsigned *access_count, long k) {
    if (!c) return SISO_EINVAL;
    if (k < 0 || (k > 0 && (!centroids || !means || !counts))) return siso_fail(c, SISO_EINVAL, "siso_import: bad arguments");
    SISO_NOT_FP8(c, "siso_import");
    if (k > c->capacity) return siso_fail(c, SISO_ECAPACITY, "siso_import: %ld rows exceed capacity %ld", k, c->capacity);
    if (k > 0) {
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_import_rows<float>, dim3((unsigned)k), dim3(256), 0, c->stream, (const float *)centroids,
                               means, counts, cluster_size, access_count, (float *)c->cent, c->mean, c->size, c->invn,
                               c->locality, c->access, c->dim);
        else
            hipLaunchKernelGGL(k_import_rows<bf16_t>, dim3((unsigned)k), dim3(256), 0, c->stream, (const bf16_t *)centroids,
                               means, counts, cluster_size, access_count, (bf16_t *)c->cent, c->mean, c->size, c->invn,
                               c->locality, c->access, c->dim);
        HIP_TRY(c, hipGetLastError());
    }
    hipLaunchKernelGGL(k_fill_nan, dim3(1), dim3(SISO_PAD_ROWS), 0, c->stream, c->invn + k, SISO_PAD_ROWS);
    HIP_TRY(c, hipGetLastError());
    c->count = k;
    return SISO_OK;
}

static int choose_path(const siso_cache *c, long n) {
    if (c->path != SISO_PATH_AUTO) return c->path;
    if (n <= 64 && siso_skinny_slices(c, n) > 0) return SISO_PATH_SKINNY;
    if (siso_mfma_slices(c, n) > 0) return SISO_PATH_MFMA;
    return SISO_PATH_SCALAR;
}

extern "C" int siso_lookup_static(siso_cache *c, const void *queries, long n, float threshold, int *out_idx,
                                  float *out_sim, unsigned char *out_hit) {
    if (!c) return SISO_EINVAL;
    if (n < 0 || (n > 0 && (!queries || !out_idx || !out_sim)))
        return siso_fail(c, SISO_EINVAL, "siso_lookup_static: bad arguments");
    // (an 8-bit cache quantises the batch into a workspace that siso_reserve sizes: this call does not grow it)
    if (c->dtype == SISO_FP8 && n > c->fp8_q_cap)
        return siso_fail(c, SISO_ECAPACITY, "siso_lookup_static: room for the codes of %ld queries, %ld asked for (siso_reserve sizes it)",
                         c->fp8_q_cap, n);
    if (!c->static_keys) return siso_fail(c, SISO_EHIP, "siso_lookup_static: the static workspace was not found on device %d", c->device);
    return siso_lookup_impl(c, queries, n, &threshold, 1, 0, out_idx, out_sim, out_hit, c->static_keys, SISO_STATIC_KEYS);
}

// keys a lookup of n queries writes in its first phase, for the kernel the library would choose
static long keys_needed(const siso_cache *c, long n) {
    if (n < 1 || c->count < 1) return n > 0 ? n : 0;
    int slices = 0;
    switch (choose_path(c, n)) {
        case SISO_PATH_SCALAR: slices = siso_scalar_slices(c, n); break;
        case SISO_PATH_MFMA: slices = siso_mfma_slices(c, n); break;
        case SISO_PATH_SKINNY: slices = siso_skinny_slices(c, n); break;
    }
    return slices > 0 ? n * (long)slices : 0;
}

static int ensure_update_notes(siso_cache *c) {
    if (c->upd_owner) return SISO_OK;
    bool ok = hipMalloc((void **)&c->upd_owner, (size_t)c->capacity * sizeof(int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&c->upd_members, (size_t)c->capacity * sizeof(int)) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        if (c->upd_owner) (void)hipFree(c->upd_owner);
        c->upd_owner = nullptr;
        return siso_fail(c, SISO_ENOMEM, "siso_update: notes for %ld centroids", c->capacity);
    }
    hipLaunchKernelGGL(k_update_mark_init, dim3((unsigned)((c->capacity + 255) / 256)), dim3(256), 0, c->stream,
                       c->upd_owner, c->upd_members, c->capacity);
    return siso_check_hip(c, hipGetLastError(), "k_update_mark_init");
}

extern "C" int siso_reserve(siso_cache *c, long n) {
    if (!c) return SISO_EINVAL;
    if (n < 0 || n > 2147483647L / 4) return siso_fail(c, SISO_EINVAL, "siso_reserve: bad batch size %ld", n);
    if (n == 0) return SISO_OK;
    // The number of keys per query depends on the batch size only through the number of query tiles (64 rows
    // is the smallest tile of any kernel) and on the number of centroids: take the largest need over all batch
    // sizes up to n, for the cache as full as it is now and for a full cache.
    long need = 0;
    siso_cache full = *c;
    full.count = c->capacity;
    for (long m = 64;; m += 64) {
        const long b = m < n ? m : n;
        const long a = keys_needed(c, b), f = keys_needed(&full, b);
        need = a > need ? a : need;
        need = f > need ? f : need;
        if (b == n) break;
    }
    if (need > c->keys_cap) {
        const int rc = ensure_workspace(c, need, 1);
        if (rc != SISO_OK) return rc;
    }
    if (c->dtype == SISO_FP8) return siso_fp8_ensure_batch(c, n);
    if (n > 256) return ensure_update_notes(c);
    return SISO_OK;
}

extern "C" int siso_lookup(siso_cache *c, const void *queries, long n, float threshold, int *out_idx, float *out_sim,
                           unsigned char *out_hit) {
    if (!c) return SISO_EINVAL;
    if (n < 0 || (n > 0 && (!queries || !out_idx || !out_sim)))
        return siso_fail(c, SISO_EINVAL, "siso_lookup: bad arguments");
    return siso_lookup_impl(c, queries, n, &threshold, 1, 0, out_idx, out_sim, out_hit);
}

extern "C" int siso_lookup_multi(siso_cache *c, const void *queries, long n, const float *thetas, int m, int count_index,
                                 int *out_idx, float *out_sim, unsigned char *out_hit) {
    if (!c) return SISO_EINVAL;
    if (n < 0 || m < 1 || m > SISO_MULTI_MAX || !thetas || count_index < -1 || count_index >= m ||
        (n > 0 && (!queries || !out_idx || !out_sim || !out_hit)))
        return siso_fail(c, SISO_EINVAL, "siso_lookup_multi: bad arguments (1 to %d thresholds)", SISO_MULTI_MAX);
    return siso_lookup_impl(c, queries, n, thetas, m, count_index, out_idx, out_sim, out_hit);
}

int siso_lookup_impl(siso_cache *c, const void *queries, long n, const float *thetas, int m, int count_index,
                     int *out_idx, float *out_sim, unsigned char *out_hit, u64 *static_keys, long static_cap, int *folded) {
    if (folded) *folded = 0;
    if (n == 0) return SISO_OK;
    if (n > 2147483647L / 4) return siso_fail(c, SISO_EINVAL, "siso_lookup: batch of %ld is too large", n);
    int slices = 1;
    const int path = c->count > 0 ? choose_path(c, n) : SISO_PATH_SCALAR;
    const bool fp8 = c->dtype == SISO_FP8;
    if (fp8 && c->count > 0 && path == SISO_PATH_SCALAR)
        return siso_fail(c, SISO_EINVAL, "siso_lookup: the 8-bit storage has no scalar kernel");
    if (c->count > 0) {
        switch (path) {
            case SISO_PATH_SCALAR: slices = siso_scalar_slices(c, n); break;
            case SISO_PATH_MFMA: slices = siso_mfma_slices(c, n); break;
            case SISO_PATH_SKINNY: slices = siso_skinny_slices(c, n); break;
        }
        if (slices <= 0)
            return siso_fail(c, SISO_EINVAL, "siso_lookup: path %d cannot serve dim %d, type %d, batch %ld", path,
                             c->dim, c->dtype, n);
    }
    int rc = SISO_OK;
    if (static_keys) {
        if (n * (long)slices > static_cap)
            return siso_fail(c, SISO_ECAPACITY,
                             "siso_lookup_static: %ld queries x %d slices of the centroids need %ld keys, the static "
                             "workspace holds %ld", n, slices, n * (long)slices, static_cap);
    } else {
        rc = ensure_workspace(c, n, slices);
        if (rc != SISO_OK) return rc;
    }
    u64 *keys = static_keys ? static_keys : c->keys;
    const void *kernel_queries = queries;
    if (fp8) {  // the batch as codes, quantised like the stored rows
        rc = siso_fp8_ensure_batch(c, n);
        if (rc == SISO_OK) rc = siso_fp8_quantize_batch(c, queries, n);
        if (rc != SISO_OK) return rc;
        kernel_queries = c->fp8_q;
    }
    const unsigned qblocks = (unsigned)n;
    const int vec = ((c->dim * elem_bytes(c->dtype)) % 16 == 0 && ((uintptr_t)queries & 15) == 0) ? 1 : 0;
    ThetaList tl;
    tl.m = m;
    tl.count_at = count_index;
    for (int j = 0; j < SISO_MULTI_MAX; ++j) tl.v[j] = j < m ? thetas[j] : 0.f;
    int row_keys = SISO_KEY_ROWS;  // what the keys of the chosen kernel carry: the winning row, or its group of four rows
    const bool may_fold = folded && n <= SISO_FOLD_BOARD && c->count > 0 && (!fp8 || c->fold_master) && m == 1 && out_hit;
    c->board_to_clear = may_fold ? c->counters + 4 : nullptr;
    if (c->count > 0) {
        if (!static_keys) siso_prof_begin(c);
        switch (path) {
            case SISO_PATH_SCALAR: rc = siso_scalar_launch(c, queries, n, slices, keys); break;
            case SISO_PATH_MFMA: rc = siso_mfma_launch(c, kernel_queries, n, slices, keys, &row_keys); break;
            case SISO_PATH_SKINNY: rc = siso_skinny_launch(c, kernel_queries, n, slices, keys, &row_keys); break;
        }
        if (!static_keys) siso_prof_end(c);
        if (rc != SISO_OK) {
            c->board_to_clear = nullptr;
            return rc;
        }
    }
    // (a kernel that empties the board takes the pointer; one that does not know of it leaves it)
    const bool board_emptied = may_fold && c->board_to_clear == nullptr;
    c->board_to_clear = nullptr;
    if (board_emptied && row_keys == SISO_KEY_ROWS) {
        const siso_cache *ms = c->fold_master;  // the bf16 cache behind an 8-bit copy, or NULL
        siso_cache *tgt = ms ? const_cast<siso_cache *>(ms) : c;
        // the end of the lookup and the update of its hits as one kernel (see k_finalize_update)
        // polls of the board (a microsecond or two each) before a block gives up
        const int spin_limit = c->opt_fold_spin_limit >= 0 ? c->opt_fold_spin_limit : 1 << 18;
#define SISO_LAUNCH_FOLD(T, E)                                                                                            \
    hipLaunchKernelGGL((k_finalize_update<T, E>), dim3(qblocks), dim3(256), 0, c->stream, (const T *)queries, keys, n, c->count, \
                       c->dim, slices, thetas[0], vec, out_idx, out_sim, out_hit, count_index >= 0 ? c->access : nullptr, \
                       (T *)tgt->cent, tgt->mean, tgt->size, tgt->invn, c->counters + 4, spin_limit, c->counters,         \
                       ms ? (const float *)c->fp8_qinv : (const float *)nullptr, ms ? (unsigned char *)c->cent : nullptr, \
                       ms ? c->scale : nullptr, ms ? c->invn : nullptr, ms ? c->size : nullptr)
        if (tgt->dtype == SISO_F32) {
            if (c->dim <= 1024) SISO_LAUNCH_FOLD(float, 4);
            else SISO_LAUNCH_FOLD(float, 16);
        } else {
            if (c->dim <= 1024) SISO_LAUNCH_FOLD(bf16_t, 4);
            else SISO_LAUNCH_FOLD(bf16_t, 16);
        }
#undef SISO_LAUNCH_FOLD
        HIP_TRY(c, hipGetLastError());
        *folded = 1;
        return SISO_OK;
    }
    const bool mark = c->mark_in_finalize == 1 && m == 1 && c->upd_owner != nullptr;
    if (c->dtype == SISO_F32)
        hipLaunchKernelGGL(k_lookup_finalize<float>, dim3(qblocks), dim3(256), 0, c->stream, (const float *)queries,
                           (const float *)c->cent, c->invn, keys, n, c->count, c->dim, slices, tl,
                           vec, row_keys, out_idx, out_sim, out_hit, count_index >= 0 ? c->access : nullptr,
                           (const float *)nullptr, mark ? c->upd_owner : nullptr, mark ? c->upd_members : nullptr);
    else
        hipLaunchKernelGGL(k_lookup_finalize<bf16_t>, dim3(qblocks), dim3(256), 0, c->stream, (const bf16_t *)queries,
                           (const bf16_t *)c->cent, c->invn, keys, n, c->count, c->dim, slices, tl,
                           vec, row_keys, out_idx, out_sim, out_hit, count_index >= 0 ? c->access : nullptr,
                           fp8 ? (const float *)c->fp8_qinv : (const float *)nullptr, mark ? c->upd_owner : nullptr,
                           mark ? c->upd_members : nullptr);
    HIP_TRY(c, hipGetLastError());
    if (mark) c->mark_in_finalize = 2;  // done
    return SISO_OK;
}

#define UPDATE_CHUNK 32768L

// premarked: the notes of this batch (one chunk) have been taken already, by the finalize step of its lookup
static int update_hits_impl(siso_cache *c, const void *queries, const int *idx, const unsigned char *hit, long n,
                            bool premarked) {
    if (!c) return SISO_EINVAL;
    SISO_NOT_FP8(c, "siso_update");
    if (n < 0 || (n > 0 && (!queries || !idx))) return siso_fail(c, SISO_EINVAL, "siso_update: bad arguments");
    // A running mean folds chunk after chunk to the same mean as one big batch,
    // so very large batches are cut to bound the member scan of each block.
    for (long off = 0; off < n; off += UPDATE_CHUNK) {
        const long m = (n - off < UPDATE_CHUNK) ? n - off : UPDATE_CHUNK;
        const unsigned char *h = hit ? hit + off : nullptr;
        const float *qf = (const float *)queries + (size_t)off * c->dim;
        const bf16_t *qh = (const bf16_t *)queries + (size_t)off * c->dim;
        const dim3 grid((unsigned)m), block(256);
        int *owner = nullptr, *marked = nullptr;
        if (m > 256) {
            const int rc = ensure_update_notes(c);
            if (rc != SISO_OK) return rc;
            owner = c->upd_owner;
            marked = c->upd_members;
            if (!premarked)
                hipLaunchKernelGGL(k_update_mark, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, c->stream, idx + off, h,
                                   m, c->count, owner, marked);
        }
#define SISO_LAUNCH_UPDATE(T, E, QP)                                                                            \
    hipLaunchKernelGGL((k_update<T, E>), grid, block, 0, c->stream, QP, idx + off, h, m, (T *)c->cent, c->mean, \
                       c->size, c->invn, c->count, c->dim, c->counters, owner, marked)
        if (c->dtype == SISO_F32) {
            if (c->dim <= 1024) SISO_LAUNCH_UPDATE(float, 4, qf);
            else SISO_LAUNCH_UPDATE(float, 16, qf);
        } else {
            if (c->dim <= 1024) SISO_LAUNCH_UPDATE(bf16_t, 4, qh);
            else SISO_LAUNCH_UPDATE(bf16_t, 16, qh);
        }
#undef SISO_LAUNCH_UPDATE
        HIP_TRY(c, hipGetLastError());
    }
    return SISO_OK;
}

extern "C" int siso_update_hits(siso_cache *c, const void *queries, const int *idx, const unsigned char *hit, long n) {
    return update_hits_impl(c, queries, idx, hit, n, false);
}

extern "C" int siso_fp8_lookup_update(siso_cache *copy, siso_cache *master, const void *queries, long n, float threshold,
                                      int *out_idx, float *out_sim, unsigned char *out_hit) {
    if (!copy) return SISO_EINVAL;
    if (!master || n < 0 || (n > 0 && (!queries || !out_idx || !out_sim || !out_hit)))
        return siso_fail(copy, SISO_EINVAL, "siso_fp8_lookup_update: bad arguments");
    if (copy->dtype != SISO_FP8 || master->dtype != SISO_BF16 || copy->dim != master->dim || copy->count != master->count)
        return siso_fail(copy, SISO_EINVAL, "siso_fp8_lookup_update: an 8-bit cache and a bf16 cache with the same centroids");
    if (copy->stream != master->stream)
        return siso_fail(copy, SISO_EINVAL, "siso_fp8_lookup_update: both caches must work on the same stream");
    if (n == 0) return SISO_OK;
    int folded = 0;
    copy->fold_master = master;
    const int rc = siso_lookup_impl(copy, queries, n, &threshold, 1, 0, out_idx, out_sim, out_hit, nullptr, 0, &folded);
    copy->fold_master = nullptr;
    if (rc != SISO_OK || folded) return rc;
    const int rc2 = siso_update_hits(master, queries, out_idx, out_hit, n);
    return rc2 != SISO_OK ? rc2 : siso_fp8_follow(copy, master, out_idx, out_hit, n);
}

extern "C" int siso_update(siso_cache *c, const void *queries, const int *idx, long n) {
    return siso_update_hits(c, queries, idx, nullptr, n);
}

extern "C" int siso_lookup_update(siso_cache *c, const void *queries, long n, float threshold, int *out_idx, float *out_sim,
                                  unsigned char *out_hit) {
    if (!c) return SISO_EINVAL;
    SISO_NOT_FP8(c, "siso_lookup_update");
    if (n < 0 || (n > 0 && (!queries || !out_idx || !out_sim || !out_hit)))
        return siso_fail(c, SISO_EINVAL, "siso_lookup_update: bad arguments");
    int folded = 0;
    // a large batch (one chunk of the update): the end of the lookup takes the update's notes itself
    c->mark_in_finalize = 0;
    if (n > 256 && n <= UPDATE_CHUNK && ensure_update_notes(c) == SISO_OK) c->mark_in_finalize = 1;
    const int rc = siso_lookup_impl(c, queries, n, &threshold, 1, 0, out_idx, out_sim, out_hit, nullptr, 0, &folded);
    const bool premarked = c->mark_in_finalize == 2;
    c->mark_in_finalize = 0;
    if (rc != SISO_OK || folded || n == 0) {
        if (premarked) {  // (a failure behind the notes: leave them as a fresh cache has them)
            hipLaunchKernelGGL(k_update_mark_init, dim3((unsigned)((c->capacity + 255) / 256)), dim3(256), 0, c->stream,
                               c->upd_owner, c->upd_members, c->capacity);
            (void)hipGetLastError();
        }
        return rc;
    }
    return update_hits_impl(c, queries, out_idx, out_hit, n, premarked);
}

int siso_read_counter(siso_cache *c, int which, u64 *value) {
    HIP_TRY(c, hipMemcpyAsync(c->host_pin, c->counters, 4 * sizeof(u64), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    *value = c->host_pin[which];
    return SISO_OK;
}

__global__ void k_zero_counter(u64 *p) { *p = 0; }

// The tiled kernels read the inverse lengths of a whole last tile; the entries just past the
// live centroids hold NaN so that those rows never win.
__global__ void k_fill_nan(float *p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = __uint_as_float(0x7FC00000u);
}

extern "C" int siso_export_meta(siso_cache *c, float *cluster_size, unsigned *access_count) {
    if (!c) return SISO_EINVAL;
    if (c->count == 0) return SISO_OK;
    if (cluster_size)
        HIP_TRY(c, hipMemcpyAsync(cluster_size, c->locality, (size_t)c->count * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
    if (access_count)
        HIP_TRY(c, hipMemcpyAsync(access_count, c->access, (size_t)c->count * sizeof(unsigned), hipMemcpyDeviceToDevice, c->stream));
    return SISO_OK;
}

extern "C" long siso_bad_indices(siso_cache *c) {
    if (!c) return SISO_EINVAL;
    u64 v = 0;
    const int rc = siso_read_counter(c, 0, &v);
    return rc != SISO_OK ? (long)rc : (long)v;
}

extern "C" long siso_merge(siso_cache *c, float threshold, int *out_pairs, long cap) {
    if (!c) return SISO_EINVAL;
    SISO_NOT_FP8(c, "siso_merge");
    if (cap < 0 || (cap > 0 && !out_pairs)) return siso_fail(c, SISO_EINVAL, "siso_merge: bad arguments");
    if (c->count < 2) return 0;
    hipLaunchKernelGGL(k_zero_counter, dim3(1), dim3(1), 0, c->stream, c->counters + 1);
    int rc = siso_check_hip(c, hipGetLastError(), "k_zero_counter");
    if (rc != SISO_OK) return rc;
    siso_prof_begin(c);
    if (siso_pairs_mfma_supported(c, c->count))
        rc = siso_pairs_mfma_launch(c, c->cent, c->invn, c->count, threshold, out_pairs, cap, c->counters + 1);
    else
        rc = siso_pairs_scalar_launch(c, c->cent, c->invn, c->count, threshold, out_pairs, cap, c->counters + 1);
    siso_prof_end(c);
    if (rc != SISO_OK) return rc;
    u64 total = 0;
    rc = siso_read_counter(c, 1, &total);
    return rc != SISO_OK ? (long)rc : (long)total;
}

extern "C" int siso_merge_apply(siso_cache *c, const int *pairs, long n_pairs, int *out_survivor) {
    if (!c) return SISO_EINVAL;
    SISO_NOT_FP8(c, "siso_merge_apply");
    if (n_pairs < 0 || (n_pairs > 0 && !pairs)) return siso_fail(c, SISO_EINVAL, "siso_merge_apply: bad arguments");
    const long K = c->count;
    if (K == 0) return SISO_OK;
    const int d = c->dim;
    const unsigned pb = (unsigned)((n_pairs + 255) / 256), kb = (unsigned)((K + 255) / 256);
    u64 v = 0;
    if (n_pairs > 0) {
        hipLaunchKernelGGL(k_zero_counter, dim3(1), dim3(1), 0, c->stream, c->counters + 2);
        hipLaunchKernelGGL(k_pairs_validate, dim3(pb), dim3(256), 0, c->stream, pairs, n_pairs, K, c->counters + 2);
        HIP_TRY(c, hipGetLastError());
        int rc = siso_read_counter(c, 2, &v);
        if (rc != SISO_OK) return rc;
        if (v != 0) return siso_fail(c, SISO_EINVAL, "siso_merge_apply: %llu invalid pairs", v);
    }
    int *parent = nullptr, *root = nullptr, *newpos = nullptr, *members_of = nullptr, *cursor = nullptr, *first = nullptr,
        *list = nullptr;
    unsigned char *touched = nullptr;
    // every valid pair joins two rows, so the survivors will be gathered into the second set of arrays: make
    // sure it exists before anything is changed in place (a failure here leaves the cache as it was)
    int rc = n_pairs > 0 ? siso_second_set(c) : SISO_OK;
    if (rc != SISO_OK) return rc;
    bool ok = hipMalloc((void **)&parent, (size_t)K * sizeof(int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&root, (size_t)K * sizeof(int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&newpos, (size_t)K * sizeof(int)) == hipSuccess;
    ok = ok && hipMalloc((void **)&touched, (size_t)K) == hipSuccess;
    ok = ok && hipMalloc((void **)&members_of, (size_t)K * 4 * sizeof(int)) == hipSuccess;  // four arrays of K
    if (!ok) {
        (void)hipGetLastError();
        rc = siso_fail(c, SISO_ENOMEM, "siso_merge_apply: temporaries");
    } else {
        cursor = members_of + K;
        first = cursor + K;
        list = first + K;
    }
    long live = K;
    if (rc == SISO_OK) {
        hipLaunchKernelGGL(k_uf_init, dim3(kb), dim3(256), 0, c->stream, parent, touched, members_of, cursor, K);
        if (n_pairs > 0)
            hipLaunchKernelGGL(k_uf_hook, dim3(pb), dim3(256), 0, c->stream, pairs, n_pairs, parent, touched);
        hipLaunchKernelGGL(k_uf_roots, dim3(kb), dim3(256), 0, c->stream, parent, root, K);
        hipLaunchKernelGGL(k_group_count, dim3(kb), dim3(256), 0, c->stream, root, touched, K, members_of);
        hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, members_of, root, K, first, (u64 *)nullptr);
        hipLaunchKernelGGL(k_group_fill, dim3(kb), dim3(256), 0, c->stream, root, touched, K, first, cursor, list);
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_group_mean<float>, dim3((unsigned)K), dim3(256), 0, c->stream, root, touched, K, members_of,
                               first, list, (float *)c->cent, c->mean, c->size, c->invn, c->locality, c->access, d);
        else
            hipLaunchKernelGGL(k_group_mean<bf16_t>, dim3((unsigned)K), dim3(256), 0, c->stream, root, touched, K, members_of,
                               first, list, (bf16_t *)c->cent, c->mean, c->size, c->invn, c->locality, c->access, d);
        hipLaunchKernelGGL(k_scan_exclusive, dim3(1), dim3(1024), 0, c->stream, (const int *)nullptr, root, K, newpos,
                           c->counters + 3);
        rc = siso_check_hip(c, hipGetLastError(), "merge_apply kernels");
        if (rc == SISO_OK) rc = siso_read_counter(c, 3, &v);
        if (rc == SISO_OK) live = (long)v;
    }
    if (rc == SISO_OK && out_survivor) {
        hipLaunchKernelGGL(k_survivor_map, dim3(kb), dim3(256), 0, c->stream, root, newpos, K, out_survivor);
        rc = siso_check_hip(c, hipGetLastError(), "k_survivor_map");
    }
    if (rc == SISO_OK && live < K) {
        // survivors packed to the front of the second set, which then becomes the cache
        if (c->dtype == SISO_F32)
            hipLaunchKernelGGL(k_gather_rows<float>, dim3((unsigned)K), dim3(256), 0, c->stream, root, newpos,
                               (const float *)c->cent, c->mean, c->size, c->invn, c->locality, c->access,
                               (float *)c->cent_b, c->mean_b, c->size_b, c->invn_b, c->locality_b, c->access_b, d);
        else
            hipLaunchKernelGGL(k_gather_rows<bf16_t>, dim3((unsigned)K), dim3(256), 0, c->stream, root, newpos,
                               (const bf16_t *)c->cent, c->mean, c->size, c->invn, c->locality, c->access,
                               (bf16_t *)c->cent_b, c->mean_b, c->size_b, c->invn_b, c->locality_b, c->access_b, d);
        rc = siso_check_hip(c, hipGetLastError(), "k_gather_rows");
        if (rc == SISO_OK) siso_swap_sets(c);
    }
    if (rc == SISO_OK) {
        hipLaunchKernelGGL(k_fill_nan, dim3(1), dim3(SISO_PAD_ROWS), 0, c->stream, c->invn + live, SISO_PAD_ROWS);
        rc = siso_check_hip(c, hipGetLastError(), "k_fill_nan");
    }
    (void)hipStreamSynchronize(c->stream);
    if (rc == SISO_OK) c->count = live;
    if (parent) (void)hipFree(parent);
    if (root) (void)hipFree(root);
    if (newpos) (void)hipFree(newpos);
    if (touched) (void)hipFree(touched);
    if (members_of) (void)hipFree(members_of);
    return rc;
}

extern "C" int siso_profile_enable(siso_cache *c, int on) {
    if (!c) return SISO_EINVAL;
    if (on < 0) return siso_fail(c, SISO_EINVAL, "siso_profile_enable: negative period");
    c->profile_on = on;
    c->prof_calls = 0;
    if (on > 0) {
        // A pair of events with nothing between them already measures some microseconds: the smallest of
        // a few such readings is taken off every bracket, so that short kernels are not overstated.
        hipEvent_t e[2] = {nullptr, nullptr};
        double least = -1.0;
        if (hipEventCreate(&e[0]) == hipSuccess && hipEventCreate(&e[1]) == hipSuccess) {
            for (int i = 0; i < 12; ++i) {
                float ms = 0.f;
                if (hipEventRecord(e[0], c->stream) != hipSuccess || hipEventRecord(e[1], c->stream) != hipSuccess) break;
                if (hipStreamSynchronize(c->stream) != hipSuccess) break;
                if (hipEventElapsedTime(&ms, e[0], e[1]) != hipSuccess) break;
                if (least < 0.0 || ms < least) least = ms;
            }
        }
        if (e[0]) (void)hipEventDestroy(e[0]);
        if (e[1]) (void)hipEventDestroy(e[1]);
        (void)hipGetLastError();
        c->prof_empty_ms = least > 0.0 ? least : 0.0;
    }
    return SISO_OK;
}

extern "C" int siso_profile_read(siso_cache *c, double *total_ms, long *launches) {
    if (!c) return SISO_EINVAL;
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    double sum = 0.0;
    for (int i = 0; i < c->prof_count; ++i) {
        float ms = 0.f;
        hipEvent_t *e = c->prof_ev + 2 * i;
        if (hipEventElapsedTime(&ms, e[0], e[1]) == hipSuccess) sum += ms > c->prof_empty_ms ? ms - c->prof_empty_ms : 0.0;
        (void)hipEventDestroy(e[0]);
        (void)hipEventDestroy(e[1]);
        e[0] = e[1] = nullptr;
    }
    if (total_ms) *total_ms = sum;
    if (launches) *launches = c->prof_count;
    c->prof_count = 0;
    return SISO_OK;
}

extern "C" int siso_export(siso_cache *c, void *centroids, float *means, int *counts) {
    if (!c) return SISO_EINVAL;
    if (c->dtype == SISO_FP8 && means) return siso_fail(c, SISO_EINVAL, "siso_export: the 8-bit storage keeps no running means");
    const size_t cells = (size_t)c->count * c->dim;
    if (c->count == 0) return SISO_OK;
    if (centroids)
        HIP_TRY(c, hipMemcpyAsync(centroids, c->cent, cells * elem_bytes(c->dtype), hipMemcpyDeviceToDevice, c->stream));
    if (means) HIP_TRY(c, hipMemcpyAsync(means, c->mean, cells * sizeof(float), hipMemcpyDeviceToDevice, c->stream));
    if (counts)
        HIP_TRY(c, hipMemcpyAsync(counts, c->size, (size_t)c->count * sizeof(int), hipMemcpyDeviceToDevice, c->stream));
    return SISO_OK;
}

// ----------------------------------------------------------------------------
// Threshold-to-hit-ratio table and the SLO-aware choice of the retrieval threshold
// (section 4.3, "Adjusting theta_R to meet SLO")
// ----------------------------------------------------------------------------
#define SISO_T2H_MAX 1024

// hits[j] += number of queries of this block whose similarity exceeds thetas[j]
__global__ void k_t2h_count(const float *__restrict__ sim, long n, const float *__restrict__ thetas, int m,
                            u64 *__restrict__ hits) {
    __shared__ unsigned local[SISO_T2H_MAX];
    for (int j = threadIdx.x; j < m; j += blockDim.x) local[j] = 0;
    __syncthreads();
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const float s = i < n ? sim[i] : __uint_as_float(0x7FC00000u);  // NaN hits nothing
    for (int j = 0; j < m; ++j) {
        const u64 above = __ballot(s > thetas[j]);
        if ((threadIdx.x & 63) == 0 && above != 0) atomicAdd(&local[j], (unsigned)__popcll(above));
    }
    __syncthreads();
    for (int j = threadIdx.x; j < m; j += blockDim.x)
        if (local[j] != 0) atomicAdd(&hits[j], (u64)local[j]);
}

extern "C" int siso_t2h(siso_cache *c, const void *queries, long n, const float *thetas, int m, long *out_hits) {
    if (!c) return SISO_EINVAL;
    if (n < 0 || m < 0 || m > SISO_T2H_MAX || (m > 0 && (!thetas || !out_hits)) || (n > 0 && !queries))
        return siso_fail(c, SISO_EINVAL, "siso_t2h: bad arguments (at most %d thresholds)", SISO_T2H_MAX);
    for (int j = 0; j < m; ++j) out_hits[j] = 0;
    if (n == 0 || m == 0) return SISO_OK;
    // one lookup of the sample, then every threshold is a comparison against the same similarities
    char *ws = nullptr;
    const size_t off_sim = (size_t)n * sizeof(int), off_th = off_sim + (size_t)n * sizeof(float);
    const size_t off_hits = (off_th + (size_t)m * sizeof(float) + 7) & ~(size_t)7;
    if (hipMalloc((void **)&ws, off_hits + (size_t)m * sizeof(u64)) != hipSuccess) {
        (void)hipGetLastError();
        return siso_fail(c, SISO_ENOMEM, "siso_t2h: workspace for %ld queries", n);
    }
    int *idx = (int *)ws;
    float *sim = (float *)(ws + off_sim), *d_th = (float *)(ws + off_th);
    u64 *d_hits = (u64 *)(ws + off_hits);
    int rc = SISO_OK;
    hipError_t e = hipMemcpyAsync(d_th, thetas, (size_t)m * sizeof(float), hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(d_hits, 0, (size_t)m * sizeof(u64), c->stream);
    if (e != hipSuccess) rc = siso_check_hip(c, e, "siso_t2h: set-up");
    const float no_theta = 0.f;
    if (rc == SISO_OK) rc = siso_lookup_impl(c, queries, n, &no_theta, 1, -1, idx, sim, nullptr);  // test lookups are no references
    u64 host_hits[SISO_T2H_MAX];
    if (rc == SISO_OK) {
        hipLaunchKernelGGL(k_t2h_count, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, c->stream, sim, n, d_th, m, d_hits);
        e = hipGetLastError();
        if (e == hipSuccess)
            e = hipMemcpyAsync(host_hits, d_hits, (size_t)m * sizeof(u64), hipMemcpyDeviceToHost, c->stream);
        if (e != hipSuccess) rc = siso_check_hip(c, e, "siso_t2h: count");
    }
    e = hipStreamSynchronize(c->stream);
    if (rc == SISO_OK && e != hipSuccess) rc = siso_check_hip(c, e, "siso_t2h: synchronize");
    (void)hipFree(ws);
    if (rc == SISO_OK)
        for (int j = 0; j < m; ++j) out_hits[j] = (long)host_hits[j];
    return rc;
}

// Equation 2.  rho = lambda E is the load of the single server; the mean time in an M/D/1 system
// is the serving time plus rho E / (2 (1 - rho)) of queueing.
extern "C" double siso_md1_wait(double llm_time, double arrival_rate, double hit_ratio) {
    const double serve = llm_time * (1.0 - hit_ratio);
    const double load = arrival_rate * serve;
    if (load >= 1.0 || load != load) return HUGE_VAL;
    return serve + load * serve / (2.0 * (1.0 - load));
}

extern "C" int siso_pick_threshold(const float *thetas, const double *hit_ratio, int m, double llm_time,
                                   double arrival_rate, double slo, int *out_index) {
    if (!out_index) return SISO_EINVAL;
    *out_index = -1;
    if (m < 0 || (m > 0 && (!thetas || !hit_ratio))) return SISO_EINVAL;
    float chosen_theta = 0.f;
    for (int j = 0; j < m; ++j) {
        if (!(siso_md1_wait(llm_time, arrival_rate, hit_ratio[j]) < slo)) continue;
        if (*out_index < 0 || thetas[j] > chosen_theta) {
            *out_index = j;
            chosen_theta = thetas[j];
        }
    }
    return SISO_OK;
}

extern "C" int siso_adjust_threshold(const float *thetas, int m, int index, double wait_estimated, double wait_measured) {
    if (!thetas || index < 0 || index >= m) return index;
    const bool longer = wait_measured > 1.1 * wait_estimated, shorter = wait_measured < 0.9 * wait_estimated;
    if (!longer && !shorter) return index;
    // the neighbour in the order of the thresholds: the largest one below, or the smallest one above
    int neighbour = index;
    for (int j = 0; j < m; ++j) {
        const bool right_side = longer ? thetas[j] < thetas[index] : thetas[j] > thetas[index];
        if (!right_side) continue;
        if (neighbour == index || (longer ? thetas[j] > thetas[neighbour] : thetas[j] < thetas[neighbour])) neighbour = j;
    }
    return neighbour;
}

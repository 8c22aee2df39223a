// Phase 1 of the bf16 lookup: a fused MFMA GEMM whose epilogue keeps a running
// maximum per query in registers, so the similarity matrix (queries x centroids;
// CosineSimilarity inside FindClosestCentroid, Algorithm 1) never leaves the
// compute unit.  One kernel template serves the large-batch path (256 x 256 tiles,
// bound by the matrix cores) and the small-batch path (256 centroids x 64 queries,
// a deeper ring of stages, bound by memory bandwidth).
//
// Mapping onto v_mfma_f32_32x32x16_bf16 (D = A x B, fp32 accumulate):
//   A rows    = 32 centroids      (lane l supplies row l%32, k = 8*(l/32) .. +8)
//   B columns = 32 queries        (lane l supplies column l%32, same k)
//   D         = lane l holds column l%32 (one query); its 16 registers are the
//               centroid rows 8*(i/4) + 4*(l/32) + i%4.
// So the maximum over centroids is taken inside a lane (over its registers and
// over all tiles the workgroup walks through); lanes l and l^32 are combined
// once at the end, and the waves that share a query column meet in LDS.
//
// A workgroup owns one tile of BQ queries and walks through `tiles_per_slice`
// tiles of BC centroids, as one continuous stream of slabs of 64 elements of the
// dimension.  Global -> LDS goes by direct loads (no staging registers): every
// wave instruction moves 8 rows x 128 bytes, i.e. whole 128-byte lines, which is
// the pattern that reaches the full memory bandwidth.
//
// LDS layout of a stage: tile row r (centroid rows first, then query rows) is 128
// bytes = 8 chunks of 16 bytes; chunk c of row r sits in slot c ^ ((r >> 1) & 7).
// LDS has 64 banks of 4 bytes and serves a 128-bit read 16 lanes at a time; with
// this swizzle the 16 rows x 16 bytes of a fragment read cover all 64 banks.  A
// direct load of one wave fills 1 KiB = 8 consecutive rows: lane i writes slot
// i % 8 of row i / 8, so it fetches chunk (i % 8) ^ ((r >> 1) & 7) of that row.
//
// The same stream of tiles, with another epilogue, is the pair search behind
// MergeCentroids: the "query" tile is a tile of centroids too, a workgroup walks
// through the centroid tiles at or right of it (upper triangle), and every
// product above the threshold is emitted as a pair (i, j), i < j.
#include "siso_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int WC_, int WQ_, int NWC_, int NWQ_, int NSTAGE_, int BK_ = 64>
struct PipeCfg {
    static constexpr int WC = WC_, WQ = WQ_, NWC = NWC_, NWQ = NWQ_, NSTAGE = NSTAGE_;
    static constexpr int BK = BK_;            // elements of the dimension per slab (64; or 32: half lines)
    static constexpr int RB = BK * 2;         // bytes of a tile row in a stage
    static constexpr int CPR = BK / 8;        // 16-byte chunks per tile row
    static constexpr int RPI = 64 / CPR;      // tile rows one direct load of a wave fills
    static constexpr int RP = 256 / RB;       // tile rows per 256 bytes (all 64 banks)
    static constexpr int KK = BK / 16;        // MFMA steps per slab
    static constexpr int BC = 32 * WC * NWC;  // centroid rows per tile
    static constexpr int BQ = 32 * WQ * NWQ;  // query rows per tile
    static constexpr int NW = NWC * NWQ, NT = 64 * NW;
    static constexpr int STAGE = (BC + BQ) * RB;
    static constexpr int NLA = BC / RPI / NW, NLB = BQ / RPI / NW;  // direct loads per wave and slab
    static_assert(BK == 64 || BK == 32, "slab of 64 or 32 elements");
    static constexpr int NL = NLA + NLB;
    static constexpr int LDS_BYTES = NSTAGE * STAGE + 2 * BC * 4;
    static_assert((BC / RPI) % NW == 0 && (BQ / RPI) % NW == 0, "whole row groups per wave");
    static_assert(BC <= SISO_PAD_ROWS && BC <= NT && BC % 64 == 0, "tile of inverse lengths: one direct load per wave");
    static_assert(BQ * NWC * 8 <= NSTAGE * STAGE, "reduction scratch fits in the stage buffers");
    static_assert(NSTAGE >= 2 && LDS_BYTES <= 160 * 1024, "stages fit in LDS");
    static_assert((NSTAGE - 1) * NL <= 63, "wait count fits the counter");
};

// direct global -> LDS loads: lane i of the wave writes its 16 (4) bytes at lds_wave_base + 16 (4) * i
__device__ __forceinline__ void gload_lds16(const void *g, void *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}
// the same with the non-temporal hint: data that is read once should not push reusable lines out of L2
__device__ __forceinline__ void gload_lds16_nt(const void *g, void *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 2);
}
__device__ __forceinline__ void gload_lds4(const void *g, void *lds_wave_base) {
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 4, 0, 0);
}

// LDS fragment reads and their waits are written out by hand: while direct loads are in
// flight the compiler waits for *all* outstanding LDS reads before every use, which would
// serialise the fragment double buffering.  LDS operations complete in order, so
// "lgkmcnt(N)" = everything but the newest N reads has arrived.  Each read and its wait sit
// in the same straight-line stretch of code.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_frag(unsigned addr) {
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2 ; hand-scheduled" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
    return __builtin_bit_cast(bf16x8, v);
}
template <int N, int NA, int NB>
__device__ __forceinline__ void lds_wait(bf16x8 (&a)[NA], bf16x8 (&b)[NB]) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a[0]) : "n"(N));
#pragma unroll
    for (int i = 1; i < NA; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
    for (int i = 0; i < NB; ++i) asm volatile("" : "+v"(b[i]));
}
// SUB = bytes between the 32-row blocks of a wave's tile (32 tile rows)
template <int SUB, int NA, int NB>
__device__ __forceinline__ void lds_frags(bf16x8 (&a)[NA], bf16x8 (&b)[NB], unsigned addr_a, unsigned addr_b) {
    static_assert(NA <= 4 && NB <= 4, "fragment offsets are spelled out up to four");
    a[0] = lds_frag<0>(addr_a);
    if constexpr (NA > 1) a[1] = lds_frag<SUB>(addr_a);
    if constexpr (NA > 2) a[2] = lds_frag<2 * SUB>(addr_a);
    if constexpr (NA > 3) a[3] = lds_frag<3 * SUB>(addr_a);
    b[0] = lds_frag<0>(addr_b);
    if constexpr (NB > 1) b[1] = lds_frag<SUB>(addr_b);
    if constexpr (NB > 2) b[2] = lds_frag<2 * SUB>(addr_b);
    if constexpr (NB > 3) b[3] = lds_frag<3 * SUB>(addr_b);
}
template <int N>
__device__ __forceinline__ void vm_wait() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

#define PIPE_LOOKUP 0
#define PIPE_PAIRS 1

template <class Cfg, int MODE>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_lookup_pipe(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ C, const float *__restrict__ invn, long n, long K, int d,
    int tiles_per_slice, int slices, int nqt, int qb, int nt_centroids, u64 *__restrict__ keys, float threshold,
    int *__restrict__ out_pairs, long cap, u64 *__restrict__ counter) {
    constexpr int WC = Cfg::WC, WQ = Cfg::WQ, NWC = Cfg::NWC, BC = Cfg::BC, BQ = Cfg::BQ, NT = Cfg::NT, NW = Cfg::NW,
                  STAGE = Cfg::STAGE, NLA = Cfg::NLA, NLB = Cfg::NLB, NL = Cfg::NL, NSTAGE = Cfg::NSTAGE, BK = Cfg::BK,
                  RB = Cfg::RB, CPR = Cfg::CPR, RPI = Cfg::RPI, RP = Cfg::RP, KK = Cfg::KK, SUB = 32 * Cfg::RB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *inv_s = (float *)(smem + NSTAGE * STAGE);  // [2][BC], by tile parity

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wc = wave % NWC, wq = wave / NWC;
    const int h = lane >> 5, l32 = lane & 31;

    // Block -> (query tile qt, slice s of the centroid tiles).  Workgroups are handed to the 8 XCDs
    // round robin and every XCD has its own L2.  The 32 workgroups that run together on one XCD are
    // made a block of qb query tiles x 32/qb slices, so that a centroid tile fetched into that L2
    // serves qb workgroups and qb query tiles stay resident in it; an XCD owns every eighth group of
    // 32/qb slices and walks through all query tiles for it before moving on.
    // In the pair search the query tile is a centroid tile too and only the tiles at or right of it
    // are visited (upper triangle); slices are absolute ranges of tiles, so that the workgroups of a
    // block still walk through the same centroid tiles in step.
    static_assert(MODE == PIPE_LOOKUP || Cfg::BC == Cfg::BQ, "pair search walks square tiles");
    const int total_ct = (int)((K + BC - 1) / BC);
    int qt, s, ct_begin, ct_end;
    {
        const int sb = 32 / qb;
        const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
        const int nqb = (nqt + qb - 1) / qb;
        const int grp = local / (nqb * 32), rem = local % (nqb * 32);
        const int i = rem & 31;
        qt = (rem >> 5) * qb + i % qb;
        s = (grp * 8 + xcd) * sb + i / qb;
        if (qt >= nqt || s >= slices) return;
        ct_begin = s * tiles_per_slice;
        ct_end = (ct_begin + tiles_per_slice < total_ct) ? ct_begin + tiles_per_slice : total_ct;
        if (MODE == PIPE_PAIRS) {
            if (ct_begin < qt) ct_begin = qt;
            if (ct_begin >= ct_end) return;
        }
    }
    const long q0 = (long)qt * BQ;
    const int nk = d / BK;
    const int T = (ct_end - ct_begin) * nk;  // slabs this workgroup walks through

    // direct-load addressing
    const int lr = lane / CPR, slot = lane % CPR;
    unsigned a_off[NLA], b_off[NLB];
#pragma unroll
    for (int j = 0; j < NLA; ++j) {
        const int row = (j * NW + wave) * RPI + lr;
        a_off[j] = (unsigned)(row * d + ((slot ^ ((row / RP) % CPR)) * 8));
    }
#pragma unroll
    for (int j = 0; j < NLB; ++j) {
        const int row = (j * NW + wave) * RPI + lr;
        long qr = q0 + row;
        if (qr > n - 1) qr = n - 1;
        b_off[j] = (unsigned)((qr - q0) * d + ((slot ^ ((row / RP) % CPR)) * 8));
    }
    const bf16_t *qbase = Q + (size_t)q0 * d;

    // fragment read addresses of this lane: LDS byte offset of its row in the centroid / query
    // part of stage 0, plus the swizzled 16-byte slot of each of the four 16-element steps
    const int sw = (l32 / RP) % CPR;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned row_a = lds0 + (unsigned)(((wc * WC) * 32 + l32) * RB);
    const unsigned row_b = lds0 + (unsigned)(BC * RB + ((wq * WQ) * 32 + l32) * RB);
    unsigned so[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) so[kk] = (unsigned)(((kk * 2 + h) ^ sw) * 16);

    float bv[WQ];
    unsigned bb[WQ];
#pragma unroll
    for (int b = 0; b < WQ; ++b) {
        bv[b] = -INFINITY;
        bb[b] = 0xFFFFFFFFu;
    }
    float wi[WQ];  // pairs: 1/|c| of this lane's columns (NaN past the live centroids)
#pragma unroll
    for (int b = 0; b < WQ; ++b) wi[b] = MODE == PIPE_PAIRS ? invn[q0 + (wq * WQ + b) * 32 + l32] : 0.f;
    f32x16 acc[WC][WQ];
#pragma unroll
    for (int a = 0; a < WC; ++a)
#pragma unroll
        for (int b = 0; b < WQ; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // slab t lives in stage t % NSTAGE; (ld_ct, ld_ks, ld_stage) name the slab the next issue fetches.
    // With slab 0 of a tile travel the inverse lengths of the tile's centroids (the rows past the
    // live ones hold NaN), one 4-byte direct load per lane of the first BC/64 waves.
    int ld_ct = ct_begin, ld_ks = 0, ld_stage = 0;
    auto issue = [&]() {
        if (ld_ks == 0 && wave < BC / 64)
            gload_lds4(invn + (size_t)ld_ct * BC + wave * 64 + lane, inv_s + (ld_ct & 1) * BC + wave * 64);
        const bf16_t *cb = C + (size_t)ld_ct * BC * d + ld_ks * BK;
        const bf16_t *qb = qbase + ld_ks * BK;
        unsigned char *sb = smem + ld_stage * STAGE;
        if (nt_centroids) {
#pragma unroll
            for (int j = 0; j < NLA; ++j) gload_lds16_nt(cb + a_off[j], sb + (j * NW + wave) * 1024);
        } else {
#pragma unroll
            for (int j = 0; j < NLA; ++j) gload_lds16(cb + a_off[j], sb + (j * NW + wave) * 1024);
        }
#pragma unroll
        for (int j = 0; j < NLB; ++j) gload_lds16(qb + b_off[j], sb + BC * RB + (j * NW + wave) * 1024);
        if (++ld_ks == nk) {
            ld_ks = 0;
            ++ld_ct;
        }
        if (++ld_stage == NSTAGE) ld_stage = 0;
    };

    // Pipeline:
    //   all but the last step of slab t | wait: own reads of slab t done, own loads of slab t+1 landed | barrier |
    //   issue the loads of slab t+NSTAGE into the stage just vacated | read step-0 fragments of slab t+1 |
    //   last step of slab t | epilogue if the tile is complete
    // so the loads have NSTAGE-1 slabs of time to land and the MFMAs of step 3 cover the barrier's
    // tail.  Loads complete in order: "all but the newest (NSTAGE-2)*NL" = slab t+1 has landed.  (The
    // inverse lengths ride along as one more load now and then, which only makes a wait stricter; they
    // are older than the slab issued with them, so they have landed one barrier later at the latest,
    // and the epilogue of their tile comes after that barrier because a tile has at least two slabs.)
    constexpr int NF = WC + WQ;  // fragment reads per step
    bf16x8 af[2][WC], bf[2][WQ];
    for (int i = 0; i < NSTAGE && i < T; ++i) issue();
    if (T >= NSTAGE) vm_wait<(NSTAGE - 1) * NL>();
    else vm_wait<0>();
    __syncthreads();
    if (T > 0) lds_frags<SUB>(af[0], bf[0], row_a + so[0], row_b + so[0]);

    int ct = ct_begin, ks = 0;
    unsigned sto = 0;  // byte offset of the stage of slab t
    for (int t = 0; t < T; ++t) {
        const unsigned sto_next = (sto + STAGE == NSTAGE * STAGE) ? 0u : sto + STAGE;
#pragma unroll
        for (int kk = 0; kk < KK - 1; ++kk) {
            lds_frags<SUB>(af[(kk + 1) & 1], bf[(kk + 1) & 1], row_a + sto + so[kk + 1], row_b + sto + so[kk + 1]);
            lds_wait<NF>(af[kk & 1], bf[kk & 1]);
            __builtin_amdgcn_sched_barrier(0);
            if (kk == 0 && ks == 0) {
                // first step of a tile: start from zero instead of clearing the accumulators
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int a = 0; a < WC; ++a)
#pragma unroll
                    for (int b = 0; b < WQ; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[0][a], bf[0][b], zero, 0, 0, 0);
            } else {
#pragma unroll
                for (int a = 0; a < WC; ++a)
#pragma unroll
                    for (int b = 0; b < WQ; ++b)
                        acc[a][b] =
                            __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][a], bf[kk & 1][b], acc[a][b], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_wait<0>(af[1], bf[1]);
        if (t + NSTAGE <= T) vm_wait<(NSTAGE - 2) * NL>();
        else vm_wait<0>();
        __syncthreads();
        if (t + NSTAGE < T) issue();
        if (t + 1 < T) lds_frags<SUB>(af[0], bf[0], row_a + sto_next + so[0], row_b + sto_next + so[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int a = 0; a < WC; ++a)
#pragma unroll
            for (int b = 0; b < WQ; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[1][a], bf[1][b], acc[a][b], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (ks == nk - 1) {
            // tile done: scale by 1/|c|, fold into the running maximum of each query column
            const long c0 = (long)ct * BC;
            const float *inv_t = inv_s + (ct & 1) * BC;
#pragma unroll
            for (int a = 0; a < WC; ++a) {
                const int rb = (wc * WC + a) * 32;
                f32x4 w[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) w[g] = *(const f32x4 *)(inv_t + rb + 8 * g + 4 * h);
                const unsigned blk = (unsigned)((c0 + rb) / SISO_RUN_ROWS) * 4u + 2u * (unsigned)h;
#pragma unroll
                for (int b = 0; b < WQ; ++b) {
                    float m = -INFINITY;
#pragma unroll
                    for (int i = 0; i < 16; ++i) m = fmaxf(m, acc[a][b][i] * w[i >> 2][i & 3]);
                    if (MODE == PIPE_LOOKUP) {
                        if (m > bv[b]) {
                            bv[b] = m;
                            bb[b] = blk;
                        }
                    } else if (__ballot(m * wi[b] > threshold) != 0) {
                        // rare: some product of this 32 x 32 block is above the threshold
                        const long icol = q0 + (wq * WQ + b) * 32 + l32;
#pragma unroll
                        for (int i = 0; i < 16; ++i) {
                            const long jrow = c0 + rb + 8 * (i >> 2) + 4 * h + (i & 3);
                            const float sim = acc[a][b][i] * w[i >> 2][i & 3] * wi[b];
                            emit_pair(sim > threshold && icol < jrow, (int)icol, (int)jrow, out_pairs, cap, counter);
                        }
                    }
                }
            }
            ks = 0;
            ++ct;
        } else {
            ++ks;
        }
        sto = sto_next;
    }
    __syncthreads();
    if (MODE == PIPE_PAIRS) return;

    // lanes l and l^32 hold the same query column
#pragma unroll
    for (int b = 0; b < WQ; ++b) {
        const float ov = __shfl_xor(bv[b], 32);
        const unsigned ob = __shfl_xor(bb[b], 32);
        siso_merge_candidate(bv[b], bb[b], ov, ob);
    }
    // waves with the same wq share query columns: meet in LDS (stage memory is free now)
    float *red_v = (float *)smem;  // [NWC][BQ]
    unsigned *red_b = (unsigned *)(smem + NWC * BQ * 4);
    if (h == 0) {
#pragma unroll
        for (int b = 0; b < WQ; ++b) {
            const int col = (wq * WQ + b) * 32 + l32;
            red_v[wc * BQ + col] = bv[b];
            red_b[wc * BQ + col] = bb[b];
        }
    }
    __syncthreads();
    for (int col = tid; col < BQ; col += NT) {
        float v = red_v[col];
        unsigned blk = red_b[col];
#pragma unroll
        for (int w2 = 1; w2 < NWC; ++w2) siso_merge_candidate(v, blk, red_v[w2 * BQ + col], red_b[w2 * BQ + col]);
        const long q = q0 + col;
        if (q < n) keys[(size_t)q * slices + s] = (blk == 0xFFFFFFFFu) ? 0ull : pack_key(v, blk);
    }
}

typedef PipeCfg<4, 2, 2, 4, 2> PipeLarge;  // 256 x 256 tile, waves of 128 x 64, two stages
typedef PipeCfg<2, 2, 4, 2, 3> PipeMid;    // 256 x 128 tile, waves of 64 x 64, three stages
typedef PipeCfg<1, 2, 8, 1, 3> PipeSmall;  // 256 x 64 tile, waves of 32 x 64, three stages
typedef PipeCfg<4, 2, 2, 4, 4, 32> PipeLarge32;  // 256 x 256 tile, slabs of 32 elements, four stages

// ----------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------
struct PipePlan {
    int cfg, bc, bq, tiles_per_slice, slices, nqt, qb;
    long grid;
};

// cfg: 1 = PipeLarge, 2 = PipeMid, 3 = PipeSmall, 4 = PipeLarge32
static bool pipe_plan(const siso_cache *c, long n, int cfg, long want_wgs, PipePlan *p) {
    if (c->dtype != SISO_BF16 || c->dim % 64 != 0 || c->dim < 128 || c->count < 1 || n < 1) return false;
    if (cfg < 1 || cfg > 4) return false;
    p->cfg = cfg;
    p->bc = 256;
    p->bq = cfg == 2 ? PipeMid::BQ : cfg == 3 ? PipeSmall::BQ : PipeLarge::BQ;
    const long nqt = (n + p->bq - 1) / p->bq;
    const long ct = (c->count + p->bc - 1) / p->bc;
    long tps = c->opt_tiles_per_slice;
    if (tps <= 0) {
        tps = (ct * nqt + want_wgs - 1) / want_wgs;
        if (tps < 1) tps = 1;
        // With several query tiles a slice is read once per block of query tiles.  Short slices keep
        // what the 8 XCDs read at a time (8 x 4 slices) near 128 MB, so that those repeats come from
        // the 256 MB memory-side cache instead of HBM.
        const long mall_tps = 8192 / c->dim > 2 ? 8192 / c->dim : 2;
        if (nqt > 1 && tps > mall_tps) tps = mall_tps;
    }
    if (tps > ct) tps = ct;
    const long slices = (ct + tps - 1) / tps;
    if (nqt * slices > 2147483647L || slices > 1000000) return false;
    p->tiles_per_slice = (int)tps;
    p->slices = (int)slices;
    p->nqt = (int)nqt;
    // query tiles per XCD block: 8 when there are that many (a centroid tile fetched into an XCD's L2
    // then serves 8 workgroups, and 8 query tiles are about what stays resident in a 4 MB L2), fewer when the batch is small, more when there are so few slices that
    // some XCD would otherwise stay idle (an XCD owns every eighth group of 32/qb slices)
    int qb = c->opt_mfma_qblock > 0 ? c->opt_mfma_qblock : 8;
    if (qb != 1 && qb != 2 && qb != 4 && qb != 8 && qb != 16 && qb != 32) return false;
    if (c->opt_mfma_qblock <= 0) {
        while (qb > 1 && qb > nqt) qb >>= 1;
        while (qb < 32 && slices * qb < 256) qb <<= 1;
    }
    p->qb = qb;
    const long sb = 32 / qb, groups = (slices + sb - 1) / sb, nqb = (nqt + qb - 1) / qb;
    p->grid = 8 * ((groups + 7) / 8) * nqb * 32;
    if (p->grid > 2147483647L) return false;
    return true;
}

static bool mfma_plan(const siso_cache *c, long n, PipePlan *p) {
    int cfg = c->opt_mfma_config;
    if (cfg == 0) cfg = n <= 64 ? 3 : n <= 128 ? 2 : 1;
    // about two workgroups per compute unit when there is enough work
    return pipe_plan(c, n, cfg, 512, p);
}

static bool skinny_plan(const siso_cache *c, long n, PipePlan *p) {
    if (n > 64) return false;
    // exactly one workgroup per compute unit: every one streams an equal share of the centroids
    return pipe_plan(c, n, 3, 256, p);
}

template <class Cfg>
static int launch_cfg(siso_cache *c, const void *queries, long n, const PipePlan &p) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lookup_pipe<Cfg, PIPE_LOOKUP>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(k_lookup_pipe)");
        attr_done = true;
    }
    hipLaunchKernelGGL((k_lookup_pipe<Cfg, PIPE_LOOKUP>), dim3((unsigned)p.grid), dim3(Cfg::NT), Cfg::LDS_BYTES,
                       c->stream, (const bf16_t *)queries, (const bf16_t *)c->cent, c->invn, n, c->count, c->dim,
                       p.tiles_per_slice, p.slices, p.nqt, p.qb, c->opt_mfma_nt ? 0 : 1, c->keys, 0.f, (int *)nullptr, 0L, (u64 *)nullptr);
    return siso_check_hip(c, hipGetLastError(), "k_lookup_pipe");
}

static int pipe_launch(siso_cache *c, const void *queries, long n, const PipePlan &p) {
    if (((uintptr_t)queries & 15) != 0) return siso_fail(c, SISO_EINVAL, "bf16 lookup: queries must be 16-byte aligned");
    switch (p.cfg) {
        case 1: return launch_cfg<PipeLarge>(c, queries, n, p);
        case 2: return launch_cfg<PipeMid>(c, queries, n, p);
        case 3: return launch_cfg<PipeSmall>(c, queries, n, p);
        default: return launch_cfg<PipeLarge32>(c, queries, n, p);
    }
}

int siso_mfma_slices(const siso_cache *c, long n) {
    PipePlan p;
    return mfma_plan(c, n, &p) ? p.slices : 0;
}

int siso_mfma_launch(siso_cache *c, const void *queries, long n, int slices) {
    PipePlan p;
    if (!mfma_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "mfma lookup: plan mismatch");
    return pipe_launch(c, queries, n, p);
}

int siso_skinny_slices(const siso_cache *c, long n) {
    PipePlan p;
    return skinny_plan(c, n, &p) ? p.slices : 0;
}

int siso_skinny_launch(siso_cache *c, const void *queries, long n, int slices) {
    PipePlan p;
    if (!skinny_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "skinny lookup: plan mismatch");
    return pipe_launch(c, queries, n, p);
}

// ----------------------------------------------------------------------------
// pair search (siso_merge) on the same kernel
// ----------------------------------------------------------------------------
int siso_merge_mfma_supported(const siso_cache *c) {
    if (c->opt_merge_config == 1) return 0;  // 1 = force the scalar kernel
    return c->dtype == SISO_BF16 && c->dim % 64 == 0 && c->dim >= 128 && c->count >= 2;
}

int siso_merge_mfma_launch(siso_cache *c, float threshold, int *out_pairs, long cap) {
    typedef PipeLarge Cfg;
    const long T = (c->count + Cfg::BC - 1) / Cfg::BC;
    // one tile pair per workgroup (the triangle balances best in small pieces), blocks of 8 tiles x 4
    // slices per XCD; workgroups whose slice lies left of their own tile exit at once
    long tps = c->opt_tiles_per_slice > 0 ? c->opt_tiles_per_slice : 1;
    if (tps > T) tps = T;
    const long slices = (T + tps - 1) / tps;
    int qb = 8;
    while (qb > 1 && qb > T) qb >>= 1;
    while (qb < 32 && slices * qb < 256) qb <<= 1;
    const long sb = 32 / qb, groups = (slices + sb - 1) / sb, nqb = (T + qb - 1) / qb;
    const long grid = 8 * ((groups + 7) / 8) * nqb * 32;
    if (grid > 2147483647L) return siso_fail(c, SISO_EINVAL, "pair search: too many tiles");
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lookup_pipe<Cfg, PIPE_PAIRS>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(pair search)");
        attr_done = true;
    }
    hipLaunchKernelGGL((k_lookup_pipe<Cfg, PIPE_PAIRS>), dim3((unsigned)grid), dim3(Cfg::NT), Cfg::LDS_BYTES, c->stream,
                       (const bf16_t *)c->cent, (const bf16_t *)c->cent, c->invn, c->count, c->count, c->dim, (int)tps,
                       (int)slices, (int)T, qb, 0, (u64 *)nullptr, threshold, out_pairs, cap, c->counters + 1);
    return siso_check_hip(c, hipGetLastError(), "pair search kernel");
}

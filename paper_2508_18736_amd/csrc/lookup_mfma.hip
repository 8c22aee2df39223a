// Phase 1 of the large-batch lookup: a fused bf16 MFMA GEMM whose epilogue keeps a
// running maximum per query in registers, so the similarity matrix (queries x
// centroids; CosineSimilarity inside FindClosestCentroid, Algorithm 1) never
// leaves the compute unit.
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
// tiles of BC centroids.  Both operand tiles go through LDS in slabs of BK
// elements of the dimension, double buffered, with a 16-byte-chunk XOR swizzle
// so that the 128-bit fragment reads of a wave spread over all banks.
#include "siso_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int WC_, int WQ_, int NWC_, int NWQ_, int BK_, int WPE_>
struct LookupCfg {
    static constexpr int WC = WC_, WQ = WQ_, NWC = NWC_, NWQ = NWQ_, BK = BK_;
    static constexpr int WPE = WPE_;          // waves per SIMD the register budget is set for
    static constexpr int BC = 32 * WC * NWC;  // centroid rows per tile
    static constexpr int BQ = 32 * WQ * NWQ;  // query rows per tile
    static constexpr int NT = 64 * NWC * NWQ; // threads
    static constexpr int CPR = BK / 8;        // 16-byte chunks per tile row
    static constexpr int RP = 256 / (BK * 2); // tile rows per 256 bytes of LDS (64 banks x 4 bytes)
    static constexpr int NA = BC * CPR / NT;  // chunks per thread, centroid tile
    static constexpr int NB = BQ * CPR / NT;  // chunks per thread, query tile
    static constexpr int STAGE = (BC + BQ) * BK * 2;
    static constexpr int LDS_BYTES = 2 * STAGE + 2 * BC * 4;
    static_assert(BK == 32 || BK == 64, "slab of 32 or 64 elements");
    static_assert((BC * CPR) % NT == 0 && (BQ * CPR) % NT == 0, "whole chunks per thread");
    static_assert(BQ * NWC * 8 <= 2 * STAGE, "reduction scratch fits in the stage buffers");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(Cfg::WPE, Cfg::WPE))) void k_lookup_mfma(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ C,
                                                          const float *__restrict__ invn, long n, long K, int d,
                                                          int tiles_per_slice, int slices, int nqt,
                                                          u64 *__restrict__ keys) {
    constexpr int WC = Cfg::WC, WQ = Cfg::WQ, NWC = Cfg::NWC, BK = Cfg::BK, BC = Cfg::BC, BQ = Cfg::BQ,
                  NT = Cfg::NT, CPR = Cfg::CPR, RP = Cfg::RP, NA = Cfg::NA, NB = Cfg::NB, STAGE = Cfg::STAGE;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *inv_s = (float *)(smem + 2 * STAGE);  // [2][BC], by tile parity

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int wc = wave % NWC, wq = wave / NWC;
    const int h = lane >> 5, l32 = lane & 31;

    const int qt = blockIdx.x % nqt, s = blockIdx.x / nqt;
    const long q0 = (long)qt * BQ;
    const long total_ct = (K + BC - 1) / BC;
    const long ct_begin = (long)s * tiles_per_slice;
    const long ct_end = (ct_begin + tiles_per_slice < total_ct) ? ct_begin + tiles_per_slice : total_ct;
    const int nk = d / BK;

    // global -> LDS chunk assignment of this thread: chunk id = tid + j*NT, row = id / CPR,
    // c = id % CPR, LDS slot = c ^ ((row / RP) % CPR).  Successive j move RSTEP rows down,
    // which changes neither c nor the swizzle term.
    constexpr int RSTEP = NT / CPR;
    static_assert(RSTEP % (RP * CPR) == 0, "row step keeps the swizzle term");
    const int row0 = tid / CPR, c0k = tid % CPR;
    const int lds0 = (row0 * CPR + (c0k ^ ((row0 / RP) % CPR))) * 16;
    unsigned b_off[NB];  // element offsets from Q + q0*d, rows clamped into the batch
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        long qr = q0 + row0 + j * RSTEP;
        if (qr > n - 1) qr = n - 1;
        b_off[j] = (unsigned)((qr - q0) * d + c0k * 8);
    }
    const bf16_t *qbase = Q + (size_t)q0 * d;

    // fragment read offsets of this lane inside a stage
    const int sw = (l32 / RP) % CPR;
    int fa[WC], fb[WQ];
#pragma unroll
    for (int a = 0; a < WC; ++a) fa[a] = ((wc * WC + a) * 32 + l32) * CPR * 16;
#pragma unroll
    for (int b = 0; b < WQ; ++b) fb[b] = BC * BK * 2 + ((wq * WQ + b) * 32 + l32) * CPR * 16;

    float bv[WQ];
    unsigned bb[WQ];
#pragma unroll
    for (int b = 0; b < WQ; ++b) {
        bv[b] = -INFINITY;
        bb[b] = 0xFFFFFFFFu;
    }

    for (long ct = ct_begin; ct < ct_end; ++ct) {
        const long c0 = ct * BC;
        float *inv_t = inv_s + (ct & 1) * BC;
        for (int r = tid; r < BC; r += NT) inv_t[r] = (c0 + r < K) ? invn[c0 + r] : __uint_as_float(0x7FC00000u);

        // rows past K are readable (the centroid array is padded by a tile) and never win
        const bf16_t *abase = C + (size_t)(c0 + row0) * d + c0k * 8;
        const size_t astep = (size_t)RSTEP * d;

        f32x16 acc[WC][WQ];
#pragma unroll
        for (int a = 0; a < WC; ++a)
#pragma unroll
            for (int b = 0; b < WQ; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

        u32x4 pa[NA], pb[NB];
#pragma unroll
        for (int j = 0; j < NA; ++j) pa[j] = *(const u32x4 *)(abase + j * astep);
#pragma unroll
        for (int j = 0; j < NB; ++j) pb[j] = *(const u32x4 *)(qbase + b_off[j]);
#pragma unroll
        for (int j = 0; j < NA; ++j) *(u32x4 *)(smem + lds0 + j * (RSTEP * BK * 2)) = pa[j];
#pragma unroll
        for (int j = 0; j < NB; ++j) *(u32x4 *)(smem + BC * BK * 2 + lds0 + j * (RSTEP * BK * 2)) = pb[j];
        __syncthreads();

        for (int it = 0; it < nk; ++it) {
            const unsigned char *st = smem + (it & 1) * STAGE;
            const bool more = it + 1 < nk;
            if (more) {
                const int koff = (it + 1) * BK;
#pragma unroll
                for (int j = 0; j < NA; ++j) pa[j] = *(const u32x4 *)(abase + j * astep + koff);
#pragma unroll
                for (int j = 0; j < NB; ++j) pb[j] = *(const u32x4 *)(qbase + b_off[j] + koff);
            }
#pragma unroll
            for (int kk = 0; kk < BK / 16; ++kk) {
                const int slot = ((kk * 2 + h) ^ sw) * 16;
                bf16x8 af[WC], bf[WQ];
#pragma unroll
                for (int a = 0; a < WC; ++a) af[a] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(st + fa[a] + slot));
#pragma unroll
                for (int b = 0; b < WQ; ++b) bf[b] = __builtin_bit_cast(bf16x8, *(const u32x4 *)(st + fb[b] + slot));
#pragma unroll
                for (int a = 0; a < WC; ++a)
#pragma unroll
                    for (int b = 0; b < WQ; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
            }
            if (more) {
                unsigned char *nx = smem + ((it + 1) & 1) * STAGE;
#pragma unroll
                for (int j = 0; j < NA; ++j) *(u32x4 *)(nx + lds0 + j * (RSTEP * BK * 2)) = pa[j];
#pragma unroll
                for (int j = 0; j < NB; ++j) *(u32x4 *)(nx + BC * BK * 2 + lds0 + j * (RSTEP * BK * 2)) = pb[j];
            }
            __syncthreads();
        }

        // epilogue: scale by 1/|c|, fold into the running maximum of each query column
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
                if (m > bv[b]) {
                    bv[b] = m;
                    bb[b] = blk;
                }
            }
        }
    }

    // lanes l and l^32 hold the same query column
#pragma unroll
    for (int b = 0; b < WQ; ++b) {
        const float ov = __shfl_xor(bv[b], 32);
        const unsigned ob = __shfl_xor(bb[b], 32);
        siso_merge_candidate(bv[b], bb[b], ov, ob);
    }
    // waves with the same wq share query columns: meet in LDS (stage memory is free now)
    float *red_v = (float *)smem;               // [NWC][BQ]
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
        for (int w2 = 1; w2 < NWC; ++w2) {
            siso_merge_candidate(v, blk, red_v[w2 * BQ + col], red_b[w2 * BQ + col]);
        }
        const long q = q0 + col;
        if (q < n) keys[(size_t)q * slices + s] = (blk == 0xFFFFFFFFu) ? 0ull : pack_key(v, blk);
    }
}

// ----------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------
typedef LookupCfg<4, 4, 2, 2, 64, 1> CfgA;  // 256 x 256 tile, 4 waves of 128 x 128
typedef LookupCfg<4, 2, 2, 4, 64, 2> CfgB;  // 256 x 256 tile, 8 waves of 128 x 64
typedef LookupCfg<4, 2, 2, 2, 32, 2> CfgC;  // 256 x 128 tile, 4 waves of 128 x 64, several workgroups per CU

struct MfmaPlan {
    int cfg, bc, bq, tiles_per_slice, slices, nqt;
};

static bool mfma_plan(const siso_cache *c, long n, MfmaPlan *p) {
    if (c->dtype != SISO_BF16 || c->dim % 64 != 0 || c->count < 1 || n < 1) return false;
    int cfg = c->opt_mfma_config;
    if (cfg == 0) cfg = 2;
    if (cfg < 1 || cfg > 3) return false;
    p->cfg = cfg;
    p->bc = cfg == 1 ? CfgA::BC : cfg == 2 ? CfgB::BC : CfgC::BC;
    p->bq = cfg == 1 ? CfgA::BQ : cfg == 2 ? CfgB::BQ : CfgC::BQ;
    const long nqt = (n + p->bq - 1) / p->bq;
    const long ct = (c->count + p->bc - 1) / p->bc;
    long tps = c->opt_tiles_per_slice;
    if (tps <= 0) {
        // about eight workgroups per compute unit when there is enough work
        const long want_wgs = 2048;
        tps = (ct * nqt + want_wgs - 1) / want_wgs;
        if (tps < 1) tps = 1;
    }
    if (tps > ct) tps = ct;
    const long slices = (ct + tps - 1) / tps;
    if (nqt * slices > 2147483647L || slices > 1000000) return false;
    p->tiles_per_slice = (int)tps;
    p->slices = (int)slices;
    p->nqt = (int)nqt;
    return true;
}

int siso_mfma_slices(const siso_cache *c, long n) {
    MfmaPlan p;
    return mfma_plan(c, n, &p) ? p.slices : 0;
}

template <class Cfg>
static int launch_cfg(siso_cache *c, const void *queries, long n, const MfmaPlan &p) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lookup_mfma<Cfg>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           Cfg::LDS_BYTES);
        if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(k_lookup_mfma)");
        attr_done = true;
    }
    hipLaunchKernelGGL(k_lookup_mfma<Cfg>, dim3((unsigned)(p.nqt * p.slices)), dim3(Cfg::NT), Cfg::LDS_BYTES, c->stream,
                       (const bf16_t *)queries, (const bf16_t *)c->cent, c->invn, n, c->count, c->dim,
                       p.tiles_per_slice, p.slices, p.nqt, c->keys);
    return siso_check_hip(c, hipGetLastError(), "k_lookup_mfma");
}

int siso_mfma_launch(siso_cache *c, const void *queries, long n, int slices) {
    MfmaPlan p;
    if (!mfma_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "mfma lookup: plan mismatch");
    if (((uintptr_t)queries & 15) != 0) return siso_fail(c, SISO_EINVAL, "mfma lookup: queries must be 16-byte aligned");
    switch (p.cfg) {
        case 1: return launch_cfg<CfgA>(c, queries, n, p);
        case 2: return launch_cfg<CfgB>(c, queries, n, p);
        default: return launch_cfg<CfgC>(c, queries, n, p);
    }
}

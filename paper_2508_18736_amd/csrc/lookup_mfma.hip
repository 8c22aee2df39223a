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
// once at the end (v_permlane32_swap), and the waves that share a query column meet in LDS.
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
// The same pipeline, fed with pairs of centroid tiles and with another epilogue, is
// the pair search behind MergeCentroids (k_pairs_stream): every product above the
// threshold in the upper triangle is emitted as a pair (i, j), i < j.
#include "siso_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ROWS: the keys of the lookup carry the winning row itself instead of its group of four rows (more
// compares per product, affordable where the kernel waits for memory anyway; the finalize step then
// has no centroid rows to read)
// ES: bytes per element: 2 = bf16; 1 = the 8-bit storage variant (E4M3 codes: a slab then holds 128 elements
// in the same 128 bytes per row, and a 16-byte fragment feeds two v_mfma_f32_32x32x16_fp8_fp8, one per half)
template <int WC_, int WQ_, int NWC_, int NWQ_, int NSTAGE_, int BK_ = 64, bool ROWS_ = false, int ES_ = 2, bool K64_ = false>
struct PipeCfg {
    static constexpr int WC = WC_, WQ = WQ_, NWC = NWC_, NWQ = NWQ_, NSTAGE = NSTAGE_;
    static constexpr bool ROWS = ROWS_;
    static constexpr int ES = ES_;
    static constexpr bool K64 = K64_;  // codes only: 64-deep MFMAs, 32 bytes per lane and operand (see k_lookup_pipe)
    static_assert(!K64_ || ES_ == 1, "the 64-deep form is for one-byte elements");
    static constexpr int BK = BK_;            // elements of the dimension per slab (64; or 32: half lines; 128 codes)
    static constexpr int RB = BK * ES;        // bytes of a tile row in a stage
    static constexpr int CPR = RB / 16;       // 16-byte chunks per tile row
    static constexpr int RPI = 64 / CPR;      // tile rows one direct load of a wave fills
    static constexpr int RP = 256 / RB;       // tile rows per 256 bytes (all 64 banks)
    static constexpr int KK = RB / 32;        // fragment steps per slab (a step = one 16-byte chunk per lane half)
    static constexpr int BC = 32 * WC * NWC;  // centroid rows per tile
    static constexpr int BQ = 32 * WQ * NWQ;  // query rows per tile
    static constexpr int NW = NWC * NWQ, NT = 64 * NW;
    static constexpr int STAGE = (BC + BQ) * RB;
    static constexpr int NLA = BC / RPI / NW, NLB = BQ / RPI / NW;  // direct loads per wave and slab
    static_assert((ES == 2 && (BK == 64 || BK == 32)) || (ES == 1 && BK == 128), "slab of 64 or 32 bf16 elements, or 128 codes");
    static constexpr int NL = NLA + NLB;
    static constexpr int NINV = 3;  // tiles whose inverse lengths are kept at a time (see k_lookup_pipe)
    static constexpr int LDS_BYTES = NSTAGE * STAGE + NINV * BC * 4;
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
// the same for the fragments of the 64-deep form (two chunks per block row; B in two buffers)
template <int N, int NA, int NB>
__device__ __forceinline__ void lds_wait64(bf16x8 (&al)[NA], bf16x8 (&ah)[NA], bf16x8 (&bl)[2][NB], bf16x8 (&bh)[2][NB]) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(al[0]) : "n"(N));
#pragma unroll
    for (int i = 0; i < NA; ++i) asm volatile("" : "+v"(al[i]), "+v"(ah[i]));
#pragma unroll
    for (int i = 0; i < NB; ++i) asm volatile("" : "+v"(bl[0][i]), "+v"(bh[0][i]), "+v"(bl[1][i]), "+v"(bh[1][i]));
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

// compile-time loop: f(IC<0>{}), f(IC<1>{}), ...
template <int I>
struct IC {
    static constexpr int value = I;
};
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(IC<I>{});
        static_for<I + 1, N>(f);
    }
}

// The accumulator blocks of a wave: WC x WQ blocks of 32 x 32, 16 registers per lane each.
// Up to 8 blocks they are ordinary values and the compiler places them.
// One fragment step: 16 bytes per lane of either operand.  bf16: one MFMA over 16 elements (8 per lane half);
// E4M3 codes: two MFMAs over 16 codes each (the low and the high 8 bytes of both fragments: both operands
// split their bytes the same way, which is all a dot product asks of the order of its terms).
template <bool F8>
__device__ __forceinline__ f32x16 frag_mma(bf16x8 a, bf16x8 b, f32x16 c) {
    if constexpr (F8) {
        typedef long l2 __attribute__((ext_vector_type(2)));
        const l2 a2 = __builtin_bit_cast(l2, a), b2 = __builtin_bit_cast(l2, b);
        c = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a2[0], b2[0], c, 0, 0, 0);
        return __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(a2[1], b2[1], c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
}

// The 64-deep form over E4M3 codes: 32 bytes per lane of either operand = two 16-byte chunks (scales of 2^0).
__device__ __forceinline__ f32x16 frag_mma64(bf16x8 a_lo, bf16x8 a_hi, bf16x8 b_lo, bf16x8 b_hi, f32x16 c) {
    typedef int i4 __attribute__((ext_vector_type(4)));
    typedef int i8 __attribute__((ext_vector_type(8)));
    const i8 a = __builtin_shufflevector(__builtin_bit_cast(i4, a_lo), __builtin_bit_cast(i4, a_hi), 0, 1, 2, 3, 4, 5, 6, 7);
    const i8 b = __builtin_shufflevector(__builtin_bit_cast(i4, b_lo), __builtin_bit_cast(i4, b_hi), 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
}

template <bool FIXED, int WC, int WQ, bool F8 = false>
struct Acc {
    f32x16 v[WC][WQ];
    template <int A, int B>
    __device__ __forceinline__ void first(bf16x8 a, bf16x8 b) {  // start from zero
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        v[A][B] = frag_mma<F8>(a, b, zero);
    }
    template <int A, int B>
    __device__ __forceinline__ void mac(bf16x8 a, bf16x8 b) {
        v[A][B] = frag_mma<F8>(a, b, v[A][B]);
    }
    template <int A, int B, int I>
    __device__ __forceinline__ float get() const {
        return v[A][B][I];
    }
    __device__ __forceinline__ void reserve() {}
};
// With 16 blocks the accumulators fill the AGPR half of the register file exactly, which the
// register allocator cannot pack (it spills).  So block (A, B) sits in a[16*(A*WQ+B) .. +15] by
// hand: the MFMAs and the reads are written out, and the compiler only learns that those
// registers are taken.  It knows of no dependence between these statements, so all of them are
// volatile (kept in program order), and the hardware's rules are kept by construction: a block
// is read back only after 15 more MFMAs have been issued behind the one that wrote it (or, for
// the last blocks, after the whole scaling of the blocks before them), far beyond the 8 passes
// such an MFMA takes; and a block is overwritten only by an MFMA issued after it was read.
template <int WC, int WQ>
struct Acc<true, WC, WQ, false> {
    template <int A, int B>
    __device__ __forceinline__ void first(bf16x8 a, bf16x8 b) {
        constexpr int R = 16 * (A * WQ + B);
        asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, 0 ; hand-placed" ::"v"(a), "v"(b), "n"(R), "n"(R + 15));
    }
    template <int A, int B>
    __device__ __forceinline__ void mac(bf16x8 a, bf16x8 b) {
        constexpr int R = 16 * (A * WQ + B);
        asm volatile("v_mfma_f32_32x32x16_bf16 a[%2:%3], %0, %1, a[%2:%3] ; hand-placed" ::"v"(a), "v"(b), "n"(R),
                     "n"(R + 15));
    }
    template <int A, int B, int I>
    __device__ __forceinline__ float get() const {
        float x;
        asm volatile("v_accvgpr_read_b32 %0, a[%1] ; hand-placed" : "=v"(x) : "n"(16 * (A * WQ + B) + I));
        return x;
    }
    // tells the compiler (and through it the kernel descriptor) that a0 .. a255 and the fragment
    // registers are in use (it warns that some of them are not its to hand out anyway)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
    __device__ __forceinline__ void reserve() {
        static_assert(WC * WQ == 16, "all 256 AGPRs");
        asm volatile("; fragments: v[208:255]" ::: "v208", "v255");
        asm volatile("; accumulators: a[0:255]" ::: "a0", "a15", "a16", "a31", "a32", "a47", "a48", "a63", "a64", "a79", "a80",
                     "a95", "a96", "a111", "a112", "a127", "a128", "a143", "a144", "a159", "a160", "a175", "a176", "a191",
                     "a192", "a207", "a208", "a223", "a224", "a239", "a240", "a255");
    }
#pragma clang diagnostic pop
};

// Block -> (query tile qt, slice s of the centroid tiles).  Workgroups are handed to the 8 XCDs
// round robin and every XCD has its own L2.  The 32 workgroups that run together on one XCD are
// made a unit of qb query tiles x 32/qb slices, so that a centroid tile fetched into that L2
// serves qb workgroups and qb query tiles stay resident in it.  With many groups of 32/qb slices
// an XCD owns every eighth group and walks through all blocks of query tiles for it before moving
// on (the same slices again and again: repeats come from the caches); with at most four groups
// the XCDs also split the blocks of query tiles among them, so that none stays idle.
// False = nothing to do for this block.
__host__ __device__ __forceinline__ int pipe_group_split(int groups) { return groups <= 1 ? 1 : groups == 2 ? 2 : 4; }
static long pipe_grid(long slices, long nqt, int qb) {
    const long sb = 32 / qb, groups = (slices + sb - 1) / sb, nqb = (nqt + qb - 1) / qb;
    if (groups > 4) return 8 * ((groups + 7) / 8) * nqb * 32;
    const long r = 8 / pipe_group_split((int)groups);  // XCDs per group of slices
    return 8 * ((nqb + r - 1) / r) * 32;
}
template <int BC>
__device__ __forceinline__ bool pipe_map_block(long K, int tiles_per_slice, int slices, int nqt, int qb, int &qt, int &s,
                                               int &ct_begin, int &ct_end) {
    const int total_ct = (int)((K + BC - 1) / BC);
    const int sb = 32 / qb, groups = (slices + sb - 1) / sb, nqb = (nqt + qb - 1) / qb;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int i = local & 31, u = local >> 5;  // place in the unit, number of the unit on this XCD
    int g, b;
    if (groups > 4) {
        g = (u / nqb) * 8 + xcd;
        b = u % nqb;
    } else {
        const int gp = pipe_group_split(groups);
        g = xcd % gp;
        b = xcd / gp + (8 / gp) * u;
    }
    if (g >= groups || b >= nqb || i >= qb * sb) return false;  // (qb need not divide 32: the last places stay empty)
    qt = b * qb + i % qb;
    s = g * sb + i / qb;
    if (qt >= nqt || s >= slices) return false;
    ct_begin = s * tiles_per_slice;
    ct_end = (ct_begin + tiles_per_slice < total_ct) ? ct_begin + tiles_per_slice : total_ct;
    return true;
}

// End of a lookup workgroup: every lane holds (best value, block) per query column of its wave.
// Lanes l and l^32 hold the same column; waves with the same wq share columns and meet in LDS
// (red = at least NWC * BQ * 8 bytes that nobody reads any more).
// (value, id): the larger value, then the lower id; 0xFFFFFFFF = none
__device__ __forceinline__ void pipe_merge(float &v, unsigned &b, float ov, unsigned ob) {
    if (ov > v || (ov == v && ob < b)) {
        v = ov;
        b = ob;
    }
}

// The largest of the 16 scaled products a lane holds for one query column in block (A, B), and which of
// its four register groups holds it (the lowest among equal maxima): group g = rows 8*g + 4*h .. + 3.
// The weights of rows past the end are NaN; fmaxf and ">" pass those over.
template <int A, int B, int G, class AccT>
__device__ __forceinline__ float group_max(const AccT &acc, const f32x4 &w) {
    return fmaxf(fmaxf(acc.template get<A, B, 4 * G>() * w[0], acc.template get<A, B, 4 * G + 1>() * w[1]),
                 fmaxf(acc.template get<A, B, 4 * G + 2>() * w[2], acc.template get<A, B, 4 * G + 3>() * w[3]));
}
template <int A, int B, class AccT>
__device__ __forceinline__ void block_max(const AccT &acc, const f32x4 (&w)[4], float &m, unsigned &g) {
    m = -INFINITY;
    g = 0;
    static_for<0, 4>([&](auto gg) __attribute__((always_inline)) {
        constexpr int G = decltype(gg)::value;
        const float a = group_max<A, B, G>(acc, w[G]);
        if (a > m) {  // groups ascend: ">" keeps the lowest among equal maxima
            m = a;
            g = G;
        }
    });
}

// The value lane l ^ 32 holds: v_permlane32_swap exchanges the upper half of its first register with the
// lower half of its second; given the same value twice, the first then holds the lower half in both halves
// and the second the upper half in both.  One instruction, no LDS crossbar.
__device__ __forceinline__ unsigned other_half(unsigned v) {
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (threadIdx.x & 32) ? r[0] : r[1];
}

template <int WQ, int NWC, int BQ, int NT, bool ROWS = false>  // ROWS: the keys may be read within the launch
__device__ __forceinline__ void pipe_reduce_keys(float (&bv)[WQ], unsigned (&bb)[WQ], unsigned char *red, int wc, int wq,
                                                 int h, int l32, int tid, long q0, long n, int slices, int s,
                                                 u64 *__restrict__ keys) {
#pragma unroll
    for (int b = 0; b < WQ; ++b) {
        const float ov = __uint_as_float(other_half(__float_as_uint(bv[b])));
        const unsigned ob = other_half(bb[b]);
        pipe_merge(bv[b], bb[b], ov, ob);
    }
    float *red_v = (float *)red;  // [NWC][BQ]
    unsigned *red_b = (unsigned *)(red + NWC * BQ * 4);
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
        for (int w2 = 1; w2 < NWC; ++w2) pipe_merge(v, blk, red_v[w2 * BQ + col], red_b[w2 * BQ + col]);
        const long q = q0 + col;
        if (q < n) keys[(size_t)q * slices + s] = (blk == 0xFFFFFFFFu) ? 0ull : pack_key(v, blk);
    }
}

// COLLECT: instead of keeping the running maximum, every product that reaches the bound of its query is
// listed (second pass of a top-k lookup): tau[q] = the bound of query q in the units of the products
// (<q, c> / |c|), cand[q * cand_cap + i] = the i-th listed row, cand_cnt[q] = how many rows reached the bound
// (also beyond cand_cap).  A row is listed exactly once: every product is formed by one lane.
// STREAM: the centroid loads carry the non-temporal hint (see stream_hint below).
template <class Cfg, bool COLLECT = false, bool STREAM = false>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_lookup_pipe(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ C, const float *__restrict__ invn, long n, long K, int d,
    int tiles_per_slice, int slices, int nqt, int qb, u64 *__restrict__ keys, const float *__restrict__ tau,
    int *__restrict__ cand, int *__restrict__ cand_cnt, int cand_cap, u64 *__restrict__ board) {
    constexpr int WC = Cfg::WC, WQ = Cfg::WQ, NWC = Cfg::NWC, BC = Cfg::BC, BQ = Cfg::BQ, NT = Cfg::NT, NW = Cfg::NW,
                  STAGE = Cfg::STAGE, NLA = Cfg::NLA, NLB = Cfg::NLB, NL = Cfg::NL, NSTAGE = Cfg::NSTAGE, BK = Cfg::BK,
                  RB = Cfg::RB, CPR = Cfg::CPR, RPI = Cfg::RPI, RP = Cfg::RP, KK = Cfg::KK, SUB = 32 * Cfg::RB, ES = Cfg::ES;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // (a step that ends in k_finalize_update: the slots of its board are emptied here, a kernel ahead)
    if (board != nullptr && blockIdx.x == 0 && threadIdx.x < SISO_FOLD_BOARD) board[threadIdx.x] = 0;
    // Inverse lengths of the tiles in flight, [NINV][BC], tile ct in buffer (ct - ct_begin) % NINV.  Those of
    // tile X are requested NSTAGE slabs ahead of its first slab, i.e. while slab X * nk - NSTAGE is multiplied,
    // into the buffer that tile X - NINV used; that tile's epilogue ran with slab (X - NINV + 1) * nk - 1.  So
    // the buffer is free as long as (NINV - 1) * nk >= NSTAGE, which three buffers give for every nk >= 2 (the
    // smallest dimension has two slabs) and NSTAGE <= 4; two buffers did not for nk = 2 with three stages.
    constexpr int NINV = Cfg::NINV;
    static_assert((NINV - 1) * 2 >= NSTAGE, "a tile's inverse lengths outlive the requests that run ahead");
    float *inv_s = (float *)(smem + NSTAGE * STAGE);

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wc = wave % NWC, wq = wave / NWC;
    const int h = lane >> 5, l32 = lane & 31;

    int qt, s, ct_begin, ct_end;
    if (!pipe_map_block<BC>(K, tiles_per_slice, slices, nqt, qb, qt, s, ct_begin, ct_end)) return;
    const long q0 = (long)qt * BQ;
    const int nk = d / BK;
    const int T = (ct_end - ct_begin) * nk;  // slabs this workgroup walks through
    if (T <= 0) return;

    // direct-load addressing: byte offset of this lane's 16 bytes from the slab's first element, per load
    const int lr = lane / CPR, slot = lane % CPR;
    unsigned a_off[NLA], b_off[NLB];
#pragma unroll
    for (int j = 0; j < NLA; ++j) {
        const int row = (j * NW + wave) * RPI + lr;
        a_off[j] = (unsigned)(row * d * ES + ((slot ^ ((row / RP) % CPR)) * 16));
    }
#pragma unroll
    for (int j = 0; j < NLB; ++j) {
        const int row = (j * NW + wave) * RPI + lr;
        long qr = q0 + row;
        if (qr > n - 1) qr = n - 1;
        b_off[j] = (unsigned)((qr - q0) * d * ES + ((slot ^ ((row / RP) % CPR)) * 16));
    }
    const char *qbase = (const char *)Q + (size_t)q0 * d * ES;

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
    Acc<false, WC, WQ, ES == 1> acc;  // every tile starts from a zero operand, so nothing to clear
    acc.reserve();
    float tq[WQ];  // COLLECT: the bounds of this lane's query columns (nothing reaches +inf: rows past the batch)
    if constexpr (COLLECT) {
#pragma unroll
        for (int b = 0; b < WQ; ++b) {
            const long q = q0 + (wq * WQ + b) * 32 + l32;
            tq[b] = q < n ? tau[q] : INFINITY;
        }
    }

    // slab t lives in stage t % NSTAGE; (ld_ct, ld_ks, ld_stage) name the slab the next issue fetches.
    // With slab 0 of a tile travel the inverse lengths of the tile's centroids (the rows past the
    // live ones hold NaN), one 4-byte direct load per lane of the first BC/64 waves.
    int ld_ct = ct_begin, ld_ks = 0, ld_stage = 0;
    // One part = one direct load of this wave; part NL - 1 also moves on to the next slab, but
    // never past the last one (the wide path issues unconditionally and so fetches the last slab
    // again, into a stage nobody reads any more).  With STREAM the centroid loads carry the
    // non-temporal hint (stream_hint decides per launch).
    const char *ld_c = (const char *)C + (size_t)ct_begin * BC * d * ES;  // first element of the slab, centroid side
    const char *ld_q = qbase;                                              // and query side
    unsigned char *ld_sb = smem + wave * 1024;                             // this wave's first KiB of the stage
    int ld_t = 0;
    int ld_inv = 0, cp_inv = 0;  // buffer of inverse lengths of the tile being requested / multiplied
    auto issue_part = [&](auto jj) {
        constexpr int j = decltype(jj)::value;
        if constexpr (j == 0) {
            if (ld_ks == 0 && wave < BC / 64)
                gload_lds4(invn + (size_t)ld_ct * BC + wave * 64 + lane, inv_s + ld_inv * BC + wave * 64);
        }
        // (the empty statement keeps the 32-bit offset next to its use, which lets the load take the
        // uniform base from scalar registers instead of a 64-bit address per lane)
        if constexpr (j < NLA) {
            unsigned off = a_off[j];
            asm volatile("" : "+v"(off));
            if constexpr (STREAM) gload_lds16_nt(ld_c + off, ld_sb + j * NW * 1024);
            else gload_lds16(ld_c + off, ld_sb + j * NW * 1024);
        } else {
            unsigned off = b_off[j - NLA];
            asm volatile("" : "+v"(off));
            gload_lds16(ld_q + off, ld_sb + BC * RB + (j - NLA) * NW * 1024);
        }
        if constexpr (j == NL - 1) {
            if (ld_t + 1 < T) {
                ++ld_t;
                if (++ld_ks == nk) {
                    ld_ks = 0;
                    ++ld_ct;
                    ld_inv = ld_inv + 1 == NINV ? 0 : ld_inv + 1;
                    ld_c += (size_t)(BC - 1) * d * ES;  // with the step below: on to the next tile's first slab
                    ld_q = qbase - RB;
                }
                ld_c += RB;
                ld_q += RB;
            }
            ld_sb = (++ld_stage == NSTAGE) ? (ld_stage = 0, smem + wave * 1024) : ld_sb + STAGE;
        }
    };
    auto issue = [&]() { static_for<0, NL>(issue_part); };

    // Pipeline:
    //   all but the last step of slab t | wait: own reads of slab t done, own loads of slab t+1 landed | barrier |
    //   issue the loads of slab t+NSTAGE into the stage just vacated | read step-0 fragments of slab t+1 |
    //   last step of slab t | epilogue if the tile is complete
    // so the loads have NSTAGE-1 slabs of time to land and the MFMAs of step 3 cover the barrier's
    // tail.  Loads complete in order: "all but the newest (NSTAGE-2)*NL" = slab t+1 has landed.  (The
    // inverse lengths ride along as one more load now and then, which only makes a wait stricter; they
    // are older than the slab issued with them, so they have landed one barrier later at the latest,
    // and the epilogue of their tile comes after that barrier because a tile has at least two slabs.)
    int ct = ct_begin, ks = 0;
    // A tile is done: its products are scaled by 1/|c| and folded into the running maximum of each query
    // column.  (The tile and the buffer of its inverse lengths come by value: counters that a closure
    // changes through a reference stay in memory.)
    auto fold_tile = [&](const int tile, const int inv_buf) {
        const long c0 = (long)tile * BC;
        const float *inv_t = inv_s + inv_buf * BC;
        static_for<0, WC>([&](auto ia) {
            constexpr int A = decltype(ia)::value;
            const int rb = (wc * WC + A) * 32;
            f32x4 w[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) w[g] = *(const f32x4 *)(inv_t + rb + 8 * g + 4 * h);
            const unsigned grp = (unsigned)((c0 + rb) >> 2) + (unsigned)h;  // group of four rows: 8 * run + 2 * g + h
            static_for<0, WQ>([&](auto ib) {
                constexpr int B = decltype(ib)::value;
                float m = -INFINITY;
                if constexpr (COLLECT) {
                    static_for<0, 16>([&](auto ii) {
                        constexpr int I = decltype(ii)::value;
                        m = fmaxf(m, acc.template get<A, B, I>() * w[I >> 2][I & 3]);
                    });
                    if (__ballot(m >= tq[B]) != 0) {
                        const long q = q0 + (wq * WQ + B) * 32 + l32;
                        const int row0 = (int)(c0 + rb) + 4 * h;  // register I holds row row0 + 8 * (I / 4) + I % 4
                        static_for<0, 16>([&](auto ii) {
                            constexpr int I = decltype(ii)::value;
                            // (the weights of rows past the end are NaN: never listed)
                            if (acc.template get<A, B, I>() * w[I >> 2][I & 3] >= tq[B]) {
                                const int slot = atomicAdd(cand_cnt + q, 1);
                                if (slot < cand_cap) cand[(size_t)q * cand_cap + slot] = row0 + 8 * (I >> 2) + (I & 3);
                            }
                        });
                    }
                } else if constexpr (Cfg::ROWS) {
                    // the rows of a lane ascend with the register number, the tiles of a workgroup with
                    // time: ">" keeps the lowest row among equal values
                    unsigned mi = 0;
                    static_for<0, 16>([&](auto ii) {
                        constexpr int I = decltype(ii)::value;
                        const float v = acc.template get<A, B, I>() * w[I >> 2][I & 3];
                        if (v > m) {
                            m = v;
                            mi = (unsigned)(8 * (I >> 2) + (I & 3));
                        }
                    });
                    if (m > bv[B]) {
                        bv[B] = m;
                        bb[B] = (unsigned)(c0 + rb) + 4u * (unsigned)h + mi;
                    }
                } else {
                    unsigned g;
                    block_max<A, B>(acc, w, m, g);
                    if (m > bv[B]) {
                        bv[B] = m;
                        bb[B] = grp + 2u * g;
                    }
                }
            });
        });
    };
    if constexpr (Cfg::K64) {
        // 64-deep MFMAs over codes: a slab of 128 codes is two steps; per step a lane reads two 16-byte chunks
        // of its row of either operand (chunks 4 s + 2 h and 4 s + 2 h + 1: every lane takes them in this order,
        // so both operands pair the same codes).  The fragments of a step are 32 bytes per block row: with six
        // block rows two buffers of them do not fit beside 128 accumulators, so the A fragments have one buffer
        // (a block row's fragment is read again, for the next step, behind the last MFMA that uses it: an MFMA
        // has taken its operands when the next instruction issues, and LDS data takes far longer to come) and
        // the B fragments two.  LDS operations complete in order; outstanding at the wait of a step, oldest
        // first: B of this step, A of this step, B of the next step.
        constexpr int KS = RB / 64;
        static_assert(KS == 2, "two steps per slab");
        bf16x8 al[WC], ah[WC], bl[2][WQ], bh[2][WQ];
        unsigned so0[KS], so1[KS];
#pragma unroll
        for (int st = 0; st < KS; ++st) {
            so0[st] = (unsigned)(((4 * st + 2 * h) ^ sw) * 16);
            so1[st] = (unsigned)(((4 * st + 2 * h + 1) ^ sw) * 16);
        }
        auto read_b = [&](auto bufc, unsigned base, int st) __attribute__((always_inline)) {
            constexpr int buf = decltype(bufc)::value;
            static_for<0, WQ>([&](auto ib) __attribute__((always_inline)) {
                constexpr int B = decltype(ib)::value;
                bl[buf][B] = lds_frag<B * SUB>(row_b + base + so0[st]);
                bh[buf][B] = lds_frag<B * SUB>(row_b + base + so1[st]);
            });
        };
        auto read_a = [&](auto ia, unsigned base, int st) __attribute__((always_inline)) {
            constexpr int A = decltype(ia)::value;
            al[A] = lds_frag<A * SUB>(row_a + base + so0[st]);
            ah[A] = lds_frag<A * SUB>(row_a + base + so1[st]);
        };
        auto wait_all_but = [&](auto nn) __attribute__((always_inline)) {
            lds_wait64<decltype(nn)::value>(al, ah, bl, bh);
        };
        // one step: the MFMAs of block row A, then that row's fragment of the next step (from `next`, step nst)
        auto step = [&](auto bufc, bool first, unsigned next, int nst) __attribute__((always_inline)) {
            constexpr int buf = decltype(bufc)::value;
            static_for<0, WC>([&](auto ia) __attribute__((always_inline)) {
                constexpr int A = decltype(ia)::value;
                static_for<0, WQ>([&](auto ib) __attribute__((always_inline)) {
                    constexpr int B = decltype(ib)::value;
                    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                    acc.v[A][B] = frag_mma64(al[A], ah[A], bl[buf][B], bh[buf][B], first ? zero : acc.v[A][B]);
                });
                __builtin_amdgcn_sched_barrier(0);
                read_a(ia, next, nst);
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        for (int i = 0; i < NSTAGE && i < T; ++i) issue();
        if (T >= NSTAGE) vm_wait<(NSTAGE - 1) * NL>();
        else vm_wait<0>();
        __syncthreads();
        read_b(IC<0>{}, 0u, 0);
        static_for<0, WC>([&](auto ia) __attribute__((always_inline)) { read_a(ia, 0u, 0); });
        unsigned sto = 0;  // byte offset of the stage of slab t
        for (int t = 0; t < T; ++t) {
            const unsigned sto_next = (sto + STAGE == NSTAGE * STAGE) ? 0u : sto + STAGE;
            read_b(IC<1>{}, sto, 1);
            wait_all_but(IC<2 * WQ>{});
            __builtin_amdgcn_sched_barrier(0);
            if (ks == 0) step(IC<0>{}, true, sto, 1);
            else step(IC<0>{}, false, sto, 1);
            wait_all_but(IC<0>{});
            if (t + NSTAGE <= T) vm_wait<(NSTAGE - 2) * NL>();
            else vm_wait<0>();
            __syncthreads();
            if (t + NSTAGE < T) issue();
            // (behind the last slab these read the stage of a slab that does not exist: within LDS, never used)
            read_b(IC<0>{}, sto_next, 0);
            __builtin_amdgcn_sched_barrier(0);
            step(IC<1>{}, false, sto_next, 0);
            if (ks == nk - 1) {
                fold_tile(ct, cp_inv);
                cp_inv = cp_inv + 1 == NINV ? 0 : cp_inv + 1;
                ks = 0;
                ++ct;
            } else {
                ++ks;
            }
            sto = sto_next;
        }
    } else {
        constexpr int NF = WC + WQ;  // fragment reads per step
        bf16x8 af[2][WC], bf[2][WQ];
        for (int i = 0; i < NSTAGE && i < T; ++i) issue();
        if (T >= NSTAGE) vm_wait<(NSTAGE - 1) * NL>();
        else vm_wait<0>();
        __syncthreads();
        lds_frags<SUB>(af[0], bf[0], row_a + so[0], row_b + so[0]);

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
                    static_for<0, WC>([&](auto ia) {
                        static_for<0, WQ>([&](auto ib) {
                            constexpr int A = decltype(ia)::value, B = decltype(ib)::value;
                            acc.template first<A, B>(af[0][A], bf[0][B]);
                        });
                    });
                } else {
                    static_for<0, WC>([&](auto ia) {
                        static_for<0, WQ>([&](auto ib) {
                            constexpr int A = decltype(ia)::value, B = decltype(ib)::value;
                            acc.template mac<A, B>(af[kk & 1][A], bf[kk & 1][B]);
                        });
                    });
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
            static_for<0, WC>([&](auto ia) {
                static_for<0, WQ>([&](auto ib) {
                    constexpr int A = decltype(ia)::value, B = decltype(ib)::value;
                    acc.template mac<A, B>(af[1][A], bf[1][B]);
                });
            });
            __builtin_amdgcn_sched_barrier(0);
            if (ks == nk - 1) {
                fold_tile(ct, cp_inv);
                cp_inv = cp_inv + 1 == NINV ? 0 : cp_inv + 1;
                ks = 0;
                ++ct;
            } else {
                ++ks;
            }
            sto = sto_next;
        }
    }
    if constexpr (!COLLECT) {
        __syncthreads();
        pipe_reduce_keys<WQ, NWC, BQ, NT, Cfg::ROWS>(bv, bb, smem, wc, wq, h, l32, tid, q0, n, slices, s, keys);
    }
}

// ----------------------------------------------------------------------------
// The wide variant of the same kernel: four waves (one per SIMD), each with a tile of 128 x 128
// = 16 accumulator blocks, so that a fragment read from LDS feeds four MFMAs instead of two
// or four-thirds.  With one wave per SIMD nothing hides a stall, and a direct load into LDS
// can only be issued once its stage is free, i.e. one slab ahead, which is less than such a
// load takes under full traffic.  So the global loads go through registers here: the loads of slab
// t+4 are issued while slab t is being multiplied, land in one of two register buffers, and are
// written to the LDS stage of slab t+2 two slabs later: two slabs of flight time instead of one.
//
// Per slab t (parity p = t & 1, stage p, register buffer G[p]):
//   steps 0..2: MFMAs; behind them the fragment reads of the next step and, one per four MFMAs, parts
//               4..15 of buffer 1-p: write to stage 1-p (slab t+1), load again (slab t+3)
//   wait for own LDS traffic | barrier: everyone has read all of stage p and written all of stage 1-p
//   step 3:     MFMAs; behind them the first fragment reads of slab t+1 and parts 0..3 of buffer p:
//               write to stage p (slab t+2), load again (slab t+4)
//   epilogue if the tile is complete
// Behind the last slabs the loads fetch the last slab again and the writes put it into a stage
// nobody reads any more: one code path, no conditions between the MFMAs.
// ----------------------------------------------------------------------------
// ----------------------------------------------------------------------------
// Pair search as one stream of tile pairs per workgroup.  A workgroup that handles a single tile
// pair spends a good part of its life filling and draining the pipeline and waiting to be
// replaced (with 130 KB of LDS only one fits a compute unit), so here 8 x 32 workgroups stay and
// each walks through its share of the upper triangle: the slabs of consecutive tile pairs follow
// each other without a gap, only the accumulators start from zero again.
// The 32 workgroups of an XCD take the tile pairs of one unit (8 column tiles x 4 row tiles) at a
// time, as in the lookup, so that a tile fetched into that L2 serves several of them; the XCDs own
// the groups of four row tiles in turns, in alternating direction and from the longest rows to the
// shortest, which gives each an equal share of the triangle.
// ----------------------------------------------------------------------------
struct PairItems {
    int xcd, i, qb, sb, nqb, groups, tiles, units, u;
    __device__ __forceinline__ void init(int tiles_, int qb_) {
        xcd = blockIdx.x & 7;
        i = (blockIdx.x >> 3) & 31;
        tiles = tiles_;
        qb = qb_;
        sb = 32 / qb;
        nqb = (tiles + qb - 1) / qb;
        groups = (tiles + sb - 1) / sb;
        units = ((groups + 7) / 8) * nqb;
        u = 0;
    }
    // next tile pair (column tile qt <= row tile ct) of this workgroup; false = none left
    __device__ __forceinline__ bool next(int &qt, int &ct) {
        while (u < units) {
            const int round = u / nqb, b = u % nqb;
            ++u;
            // (the groups from the bottom of the triangle upwards: the round that not every XCD takes part in is
            // then the one with the least work - 196 row tiles: 28 % more than its share on one XCD otherwise)
            const int gi = round * 8 + ((round & 1) ? 7 - xcd : xcd);
            const int g = groups - 1 - gi;
            const int q = b * qb + i % qb, s = g * sb + i / qb;
            if (gi >= groups || q >= tiles || s >= tiles || s < q) continue;
            qt = q;
            ct = s;
            return true;
        }
        return false;
    }
};

#define PAIR_STAGE 2048  // pairs a workgroup collects in LDS
template <class Cfg>
__global__ __launch_bounds__(Cfg::NT) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_pairs_stream(
    const bf16_t *__restrict__ C, const float *__restrict__ invn, long K, int d, int qb, float threshold,
    int *__restrict__ out_pairs, long cap, u64 *__restrict__ counter) {
    constexpr int WC = Cfg::WC, WQ = Cfg::WQ, NWC = Cfg::NWC, BC = Cfg::BC, BQ = Cfg::BQ, NW = Cfg::NW,
                  STAGE = Cfg::STAGE, NLA = Cfg::NLA, NLB = Cfg::NLB, NL = Cfg::NL, NSTAGE = Cfg::NSTAGE, BK = Cfg::BK,
                  RB = Cfg::RB, CPR = Cfg::CPR, RPI = Cfg::RPI, RP = Cfg::RP, KK = Cfg::KK, SUB = 32 * Cfg::RB;
    static_assert(BC == BQ && BC / 64 + BQ / 64 <= NW, "square tiles; one wave per 64 inverse lengths of either side");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *inv_a = (float *)(smem + NSTAGE * STAGE);  // [2][BC] inverse lengths of the row tile, by parity of the pair's number
    float *inv_b = inv_a + 2 * BC;                    // [2][BQ] and of the column tile
    // pairs are collected here and moved to the global list when the buffer is half full, and at the end
    int *stage = (int *)(inv_b + 2 * BQ);             // [PAIR_STAGE][2]
    int *staged = stage + 2 * PAIR_STAGE;             // entries taken (may run past PAIR_STAGE)
    u64 *flush_slot = (u64 *)(staged + 2);
    if (threadIdx.x == 0) *staged = 0;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wc = wave % NWC, wq = wave / NWC;
    const int h = lane >> 5, l32 = lane & 31;
    const int nk = d / BK;
    const int tiles = (int)((K + BC - 1) / BC);

    PairItems ld_items, cp_items;  // the same sequence twice: the loads run ahead of the MFMAs
    ld_items.init(tiles, qb);
    cp_items.init(tiles, qb);
    int ld_qt = 0, ld_ct = 0, cp_qt = 0, cp_ct = 0;
    bool ld_more = ld_items.next(ld_qt, ld_ct);
    if (!ld_more) return;
    cp_items.next(cp_qt, cp_ct);

    // direct-load addressing (rows past the live ones exist and are never above the threshold)
    const int lr = lane / CPR, slot = lane % CPR;
    unsigned a_off[NLA], b_off[NLB];
#pragma unroll
    for (int j = 0; j < NLA; ++j) {
        const int row = (j * NW + wave) * RPI + lr;
        a_off[j] = (unsigned)(row * d + ((slot ^ ((row / RP) % CPR)) * 8)) * 2u;
    }
#pragma unroll
    for (int j = 0; j < NLB; ++j) b_off[j] = a_off[j];
    const int sw = (l32 / RP) % CPR;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned row_a = lds0 + (unsigned)(((wc * WC) * 32 + l32) * RB);
    const unsigned row_b = lds0 + (unsigned)(BC * RB + ((wq * WQ) * 32 + l32) * RB);
    unsigned so[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) so[kk] = (unsigned)(((kk * 2 + h) ^ sw) * 16);

    Acc<false, WC, WQ> acc;

    // loader: slab ld_ks of the pair (ld_qt, ld_ct), the ld_seq-th pair of this workgroup
    int ld_ks = 0, ld_seq = 0, ld_stage = 0, issued = 0;
    auto issue = [&]() {
        unsigned char *sb = smem + ld_stage * STAGE + wave * 1024;
        const char *ca = (const char *)(C + ((size_t)ld_ct * BC * d + (size_t)ld_ks * BK));
        const char *cq = (const char *)(C + ((size_t)ld_qt * BQ * d + (size_t)ld_ks * BK));
        if (ld_ks == 0) {
            // the inverse lengths of both tiles travel with the pair's first slab
            if (wave < BC / 64) gload_lds4(invn + (size_t)ld_ct * BC + wave * 64 + lane, inv_a + (ld_seq & 1) * BC + wave * 64);
            else if (wave < BC / 64 + BQ / 64)
                gload_lds4(invn + (size_t)ld_qt * BQ + (wave - BC / 64) * 64 + lane, inv_b + (ld_seq & 1) * BQ + (wave - BC / 64) * 64);
        }
        static_for<0, NLA>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            unsigned off = a_off[j];
            asm volatile("" : "+v"(off));
            gload_lds16(ca + off, sb + j * NW * 1024);
        });
        static_for<0, NLB>([&](auto jj) {
            constexpr int j = decltype(jj)::value;
            unsigned off = b_off[j];
            asm volatile("" : "+v"(off));
            gload_lds16(cq + off, sb + BC * RB + j * NW * 1024);
        });
        if (++ld_ks == nk) {
            ld_ks = 0;
            ++ld_seq;
            ld_more = ld_items.next(ld_qt, ld_ct);
        }
        if (++ld_stage == NSTAGE) ld_stage = 0;
        ++issued;
    };

    constexpr int NF = WC + WQ;
    bf16x8 af[2][WC], bf[2][WQ];
    for (int s = 0; s < NSTAGE && ld_more; ++s) issue();
    if (issued == NSTAGE) vm_wait<(NSTAGE - 1) * NL>();
    else vm_wait<0>();
    __syncthreads();
    lds_frags<SUB>(af[0], bf[0], row_a + so[0], row_b + so[0]);

    int ks = 0, cp_seq = 0, consumed = 0;
    unsigned sto = 0;
    for (;;) {
        const unsigned sto_next = (sto + STAGE == NSTAGE * STAGE) ? 0u : sto + STAGE;
#pragma unroll
        for (int kk = 0; kk < KK - 1; ++kk) {
            lds_frags<SUB>(af[(kk + 1) & 1], bf[(kk + 1) & 1], row_a + sto + so[kk + 1], row_b + sto + so[kk + 1]);
            lds_wait<NF>(af[kk & 1], bf[kk & 1]);
            __builtin_amdgcn_sched_barrier(0);
            if (kk == 0 && ks == 0) {
                static_for<0, WC>([&](auto ia) {
                    static_for<0, WQ>([&](auto ib) {
                        constexpr int A = decltype(ia)::value, B = decltype(ib)::value;
                        acc.template first<A, B>(af[0][A], bf[0][B]);
                    });
                });
            } else {
                static_for<0, WC>([&](auto ia) {
                    static_for<0, WQ>([&](auto ib) {
                        constexpr int A = decltype(ia)::value, B = decltype(ib)::value;
                        acc.template mac<A, B>(af[kk & 1][A], bf[kk & 1][B]);
                    });
                });
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_wait<0>(af[1], bf[1]);
        // the next slab has landed: all but the loads of the slabs behind it may still be in flight
        if (issued - consumed >= NSTAGE) vm_wait<(NSTAGE - 2) * NL>();
        else vm_wait<0>();
        __syncthreads();
        if (ld_more) issue();
        const bool has_next = issued > consumed + 1;
        if (has_next) lds_frags<SUB>(af[0], bf[0], row_a + sto_next + so[0], row_b + sto_next + so[0]);
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, WC>([&](auto ia) {
            static_for<0, WQ>([&](auto ib) {
                constexpr int A = decltype(ia)::value, B = decltype(ib)::value;
                acc.template mac<A, B>(af[1][A], bf[1][B]);
            });
        });
        __builtin_amdgcn_sched_barrier(0);
        if (ks == nk - 1) {
            // pair done: every product above the threshold is a pair (column index < row index)
            const long c0 = (long)cp_ct * BC, q0 = (long)cp_qt * BQ;
            const float *inv_t = inv_a + (cp_seq & 1) * BC;
            const float *inv_q = inv_b + (cp_seq & 1) * BQ;
            float wi[WQ];
#pragma unroll
            for (int b = 0; b < WQ; ++b) wi[b] = inv_q[(wq * WQ + b) * 32 + l32];
            static_for<0, WC>([&](auto ia) {
                constexpr int A = decltype(ia)::value;
                const int rb = (wc * WC + A) * 32;
                f32x4 w[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) w[g] = *(const f32x4 *)(inv_t + rb + 8 * g + 4 * h);
                static_for<0, WQ>([&](auto ib) {
                    constexpr int B = decltype(ib)::value;
                    float m = -INFINITY;
                    static_for<0, 16>([&](auto ii) {
                        constexpr int I = decltype(ii)::value;
                        m = fmaxf(m, acc.template get<A, B, I>() * w[I >> 2][I & 3]);
                    });
                    if (__ballot(m * wi[B] > threshold) != 0) {
                        const long icol = q0 + (wq * WQ + B) * 32 + l32;
                        const long jrow0 = c0 + rb + 4 * h;  // register I holds row jrow0 + 8 * (I / 4) + I % 4
                        unsigned found = 0;
                        static_for<0, 16>([&](auto ii) {
                            constexpr int I = decltype(ii)::value;
                            const float sim = acc.template get<A, B, I>() * w[I >> 2][I & 3] * wi[B];
                            if (sim > threshold && icol < jrow0 + 8 * (I >> 2) + (I & 3)) found |= 1u << I;
                        });
                        emit_pairs_staged(found, (int)icol, [&](int I) { return (int)(jrow0 + 8 * (I >> 2) + (I & 3)); }, stage,
                                          staged, PAIR_STAGE, out_pairs, cap, counter);
                    }
                });
            });
            ks = 0;
            ++cp_seq;
            cp_items.next(cp_qt, cp_ct);
            // the pairs of this tile pair are staged (own LDS traffic done, then the barrier by hand: the
            // compiler's barrier would also wait for the direct loads in flight)
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (*staged > PAIR_STAGE / 2) flush_staged_pairs(stage, staged, PAIR_STAGE, flush_slot, out_pairs, cap, counter);
        } else {
            ++ks;
        }
        ++consumed;
        sto = sto_next;
        if (!has_next) break;
    }
    flush_staged_pairs(stage, staged, PAIR_STAGE, flush_slot, out_pairs, cap, counter);
}

// Fragments at fixed registers, for the wide kernel: a value that the compiler knows about can be
// copied or moved by it at any time, also while the LDS read that produces it is still in flight.
// With one wave per SIMD the reads must stay in flight across branches and the loop edge, so the
// wide kernel keeps its fragments out of the compiler's sight, in v[WIDE_FRAG0 .. 255], which the
// kernel's register limit takes away from the allocator.
#define WIDE_FRAG0 208
template <int REG, int OFF>
__device__ __forceinline__ void frag_read(unsigned addr) {
    asm volatile("ds_read_b128 v[%1:%2], %0 offset:%3 ; hand-placed" ::"v"(addr), "n"(REG), "n"(REG + 3), "n"(OFF) : "memory");
}
template <int ACC, int RA, int RB>
__device__ __forceinline__ void frag_mac() {
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%0:%1], v[%2:%3], v[%4:%5], a[%0:%1] ; hand-placed" ::"n"(ACC), "n"(ACC + 15),
                 "n"(RA), "n"(RA + 3), "n"(RB), "n"(RB + 3));
}
template <int ACC, int RA, int RB>
__device__ __forceinline__ void frag_first() {
    asm volatile("v_mfma_f32_32x32x16_bf16 a[%0:%1], v[%2:%3], v[%4:%5], 0 ; hand-placed" ::"n"(ACC), "n"(ACC + 15), "n"(RA),
                 "n"(RA + 3), "n"(RB), "n"(RB + 3));
}
template <int N>
__device__ __forceinline__ void lgkm_wait() {
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}

struct WideCfg {
    static constexpr int WC = 4, WQ = 4, NWC = 2, NWQ = 2, NW = 4, NT = 256;
    static constexpr int BC = 256, BQ = 256, BK = 64, RB = 128, KK = 4;
    static constexpr int STAGE = (BC + BQ) * RB;  // 64 KiB
    static constexpr int NLA = BC / 8 / NW, NLB = BQ / 8 / NW, NL = NLA + NLB;  // 16-byte loads per lane and slab
    static constexpr int LDS_BYTES = 2 * STAGE + 2 * BC * 4;
    static_assert(NL == WC * WQ, "one load and one write behind every MFMA of a step");
    // fragment registers: A fragment k (one buffer), B fragment k of buffer b (two buffers)
    static constexpr int ra(int k) { return WIDE_FRAG0 + 4 * k; }
    static constexpr int rb(int b, int k) { return WIDE_FRAG0 + 4 * WC + 4 * WQ * b + 4 * k; }
    static_assert(WIDE_FRAG0 + 4 * WC + 8 * WQ == 256, "fragments fill the registers behind the allocator's share");
};

// STREAM: the centroid loads carry the non-temporal hint (stream_hint_wide decides per launch).
template <bool STREAM>
__global__ __launch_bounds__(WideCfg::NT) __attribute__((amdgpu_waves_per_eu(1, 1), amdgpu_num_vgpr(WIDE_FRAG0))) void k_lookup_wide(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ C, const float *__restrict__ invn, long n, long K, int d,
    int tiles_per_slice, int slices, int nqt, int qb, u64 *__restrict__ keys) {
    typedef WideCfg Cfg;
    constexpr int WC = Cfg::WC, WQ = Cfg::WQ, NWC = Cfg::NWC, BC = Cfg::BC, BQ = Cfg::BQ, NT = Cfg::NT, NW = Cfg::NW,
                  STAGE = Cfg::STAGE, NLA = Cfg::NLA, NL = Cfg::NL, BK = Cfg::BK, RB = Cfg::RB, KK = Cfg::KK,
                  SUB = 32 * Cfg::RB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *inv_s = (float *)(smem + 2 * STAGE);  // [2][BC], by tile parity

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wc = wave % NWC, wq = wave / NWC;
    const int h = lane >> 5, l32 = lane & 31;

    int qt, s, ct_begin, ct_end;
    if (!pipe_map_block<BC>(K, tiles_per_slice, slices, nqt, qb, qt, s, ct_begin, ct_end)) return;
    const long q0 = (long)qt * BQ;
    const int nk = d / BK;
    const int T = (ct_end - ct_begin) * nk;  // slabs this workgroup walks through
    if (T <= 0) return;

    // Global loads: load j of a wave covers the 8 tile rows (4 j + wave) * 8 .. + 8, 128 bytes each;
    // lane i takes the 16 bytes that belong in slot i % 8 of row i / 8 (the swizzle of the LDS layout
    // is applied to the global chunk; it does not depend on j because rows advance by 32).
    const int lr = lane >> 3, slot = lane & 7;
    const int row0 = wave * 8 + lr;
    const unsigned chunk = (unsigned)((slot ^ ((row0 >> 1) & 7)) * 16);
    const unsigned a_voff = (unsigned)row0 * (unsigned)d * 2u + chunk;
    const int last_q = (int)((n - 1 - q0 < BQ - 1) ? n - 1 - q0 : BQ - 1);  // rows past the batch read its last row
    const bf16_t *qbase = Q + (size_t)q0 * d;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    unsigned char *wr = smem + wave * 1024 + lane * 16;  // this lane's 16 bytes of load 0 in stage 0
    // (and in stage 1, as a value of its own: an LDS instruction's offset field ends at 64 KiB, and the
    // compiler would rather keep one address per write of that stage than one base)
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
    lds_byte *wr1 = (lds_byte *)(wr + STAGE);
    asm volatile("" : "+v"(wr1));

    // fragment read addresses, as in k_lookup_pipe
    const int sw = (l32 >> 1) & 7;
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
    Acc<true, WC, WQ> acc;
    acc.reserve();

    // register buffers: G[p][j] = the 16 bytes of load j of a slab of parity p; gi = inverse lengths
    // of the slab's tile when it is the tile's first slab (they travel with it into inv_s)
    u32x4 G[2][NL];
    float gi0 = 0.f, gi1 = 0.f;
    int gs0 = -1, gs1 = -1;  // where gi belongs in inv_s (tile parity), -1 = nothing to write
    const char *ld_c = (const char *)(C + (size_t)ct_begin * BC * d);  // first element of the slab to load, centroid side
    const char *ld_q = (const char *)qbase;                              // and query side
    int ld_t = 0, ld_ks = 0, ld_ct = ct_begin;
    auto load_part = [&](auto pp, auto jj) __attribute__((always_inline)) {
        constexpr int p = decltype(pp)::value, j = decltype(jj)::value;
        if constexpr (j == 0) {
            float &gi = p == 0 ? gi0 : gi1;
            int &gs = p == 0 ? gs0 : gs1;
            gs = -1;
            if (ld_ks == 0) {
                gi = invn[(size_t)ld_ct * BC + wave * 64 + lane];
                gs = ld_ct & 1;
            }
        }
        if constexpr (j < NLA) {
            unsigned off = a_voff;
            asm volatile("" : "+v"(off));  // keeps the 32-bit offset next to its use: scalar base + lane offset
            const u32x4 *src = (const u32x4 *)(ld_c + (size_t)j * 64 * d + off);
            if constexpr (STREAM) G[p][j] = __builtin_nontemporal_load(src);
            else G[p][j] = *src;
        } else {
            // (computed here every time: eight more loop-invariant registers would not fit)
            int row = row0;
            asm volatile("" : "+v"(row));
            row += 32 * (j - NLA);
            row = row < last_q ? row : last_q;
            const unsigned off = (unsigned)row * (unsigned)d * 2u + chunk;
            G[p][j] = *(const u32x4 *)(ld_q + off);
        }
        if constexpr (j == NL - 1) {
            if (ld_t + 1 < T) {
                ++ld_t;
                if (++ld_ks == nk) {
                    ld_ks = 0;
                    ++ld_ct;
                    ld_c += (size_t)(BC - 1) * d * 2;  // with the step below: on to the next tile's first slab
                    ld_q = (const char *)qbase - BK * 2;
                }
                ld_c += BK * 2;
                ld_q += BK * 2;
            }
        }
    };
    auto write_part = [&](auto pp, auto jj) __attribute__((always_inline)) {
        constexpr int p = decltype(pp)::value, j = decltype(jj)::value;
        if constexpr (j == 0) {
            const float gi = p == 0 ? gi0 : gi1;
            const int gs = p == 0 ? gs0 : gs1;
            if (gs >= 0) inv_s[gs * BC + wave * 64 + lane] = gi;
        }
        // loads 0 .. NLA-1 fill the centroid rows of the stage, the others the query rows behind them
        if constexpr (p == 0) *(u32x4 *)(wr + j * NW * 1024) = G[p][j];
        else *(lds_u32x4 *)(wr1 + j * NW * 1024) = G[p][j];
    };
    // One step = 16 MFMAs, block (A, B) = A fragment A x B fragment B of buffer `cur`, A-major.  The
    // fragments of the next step are read meanwhile: the four B fragments behind the first four
    // MFMAs into the other B buffer, and A fragment k into its own registers behind the last MFMA
    // that uses it (an MFMA has taken its operands when the next instruction issues, and LDS data
    // takes far longer to come).  So a step may start when all but the newest read (A fragment 3)
    // have arrived, and waits for that one before its 13th MFMA (by then at most the 4 reads and
    // writes issued last are younger than it needs to be).
    auto step = [&](auto first_tag, auto cur_tag, unsigned addr_a, unsigned addr_b, auto &&extra) __attribute__((always_inline)) {
        constexpr int cur = decltype(cur_tag)::value;
        lgkm_wait<1>();
        static_for<0, WC * WQ>([&](auto ii) __attribute__((always_inline)) {
            constexpr int i = decltype(ii)::value, A = i / WQ, B = i % WQ;
            if constexpr (i == (WC - 1) * WQ) lgkm_wait<4>();
            if constexpr (decltype(first_tag)::value) frag_first<16 * i, Cfg::ra(A), Cfg::rb(cur, B)>();
            else frag_mac<16 * i, Cfg::ra(A), Cfg::rb(cur, B)>();
            extra(ii);
            if constexpr (i < WQ) frag_read<Cfg::rb(1 - cur, i), i * SUB>(addr_b);
            if constexpr (B == WQ - 1) frag_read<Cfg::ra(A), A * SUB>(addr_a);
        });
    };
    auto lds_barrier = [&]() __attribute__((always_inline)) {
        // own LDS reads and writes are done (lgkmcnt(0) just before); global loads stay in flight
        asm volatile("s_barrier" ::: "memory");
    };

    // Part j of a buffer is written to its stage and loaded again right away, one part behind every
    // fourth MFMA: the traffic is even over time (a burst of loads would hold up the wave, and with
    // it the MFMAs, while the texture unit works it off) and every load has two slabs to land.
    // The stage of parity p is free between the barrier of slab t (parity p) and that of slab t+1:
    // parts 0..3 of buffer p go with step 3 of slab t, parts 4..15 with steps 0..2 of slab t+1.
    auto xfer = [&](auto pp, auto jj) __attribute__((always_inline)) {
        write_part(pp, jj);
        load_part(pp, jj);
    };
    // prologue: slab 0 in stage 0, slab 2 on its way into buffer 0; the first four parts of slab 1 in
    // stage 1 and those of slab 3 on their way, the other parts of slab 1 still in buffer 1, as if
    // a slab of parity 1 had just gone by
    static_for<0, NL>([&](auto jj) __attribute__((always_inline)) { load_part(IC<0>{}, jj); });
    static_for<0, NL>([&](auto jj) __attribute__((always_inline)) { load_part(IC<1>{}, jj); });
    static_for<0, NL>([&](auto jj) __attribute__((always_inline)) { xfer(IC<0>{}, jj); });
    static_for<0, 4>([&](auto jj) __attribute__((always_inline)) { xfer(IC<1>{}, jj); });
    lgkm_wait<0>();
    lds_barrier();
    static_for<0, WQ>([&](auto kk) __attribute__((always_inline)) {
        constexpr int k = decltype(kk)::value;
        frag_read<Cfg::rb(0, k), k * SUB>(row_b + so[0]);
    });
    static_for<0, WC>([&](auto kk) __attribute__((always_inline)) {
        constexpr int k = decltype(kk)::value;
        frag_read<Cfg::ra(k), k * SUB>(row_a + so[0]);
    });

    int ct = ct_begin, ks = 0;
    // One slab of parity p.  The B fragments of step kk are in buffer kk & 1; KK is even, so every
    // slab starts in buffer 0.
    static_assert(KK == 4, "steps are spelled out");
    auto slab = [&](auto pp) __attribute__((always_inline)) {
        constexpr int p = decltype(pp)::value;
        constexpr unsigned sto = p * STAGE, sto_next = (1 - p) * STAGE;
        // (read addresses are summed up here every time: more loop-invariant registers would not fit)
        auto at = [&](unsigned row, unsigned stage, int k) __attribute__((always_inline)) {
            unsigned sk = so[k];
            asm volatile("" : "+v"(sk));
            return row + stage + sk;
        };
        // the part that goes behind MFMA i of step kk: buffer and first part by step, one per four MFMAs
        auto part = [&](auto bb_, auto j0, auto ii) __attribute__((always_inline)) {
            constexpr int i = decltype(ii)::value;
            if constexpr (i % 4 == 1) xfer(bb_, IC<decltype(j0)::value + i / 4>{});
        };
        if (ks == 0)  // a tile starts from zero
            step(IC<1>{}, IC<0>{}, at(row_a, sto, 1), at(row_b, sto, 1), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<4>{}, ii); });
        else
            step(IC<0>{}, IC<0>{}, at(row_a, sto, 1), at(row_b, sto, 1), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<4>{}, ii); });
        step(IC<0>{}, IC<1>{}, at(row_a, sto, 2), at(row_b, sto, 2), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<8>{}, ii); });
        step(IC<0>{}, IC<0>{}, at(row_a, sto, 3), at(row_b, sto, 3), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<12>{}, ii); });
        // all own reads of this stage have been issued; the barrier needs them, and the LDS writes
        // into the other stage, complete
        lgkm_wait<0>();
        lds_barrier();
        step(IC<0>{}, IC<1>{}, at(row_a, sto_next, 0), at(row_b, sto_next, 0), [&](auto ii) __attribute__((always_inline)) { part(pp, IC<0>{}, ii); });
        __builtin_amdgcn_sched_barrier(0);
        const bool tile_done = ks == nk - 1;
        if (tile_done) {
            // scale by 1/|c|, fold into the running maximum of each query column
            const long c0 = (long)ct * BC;
            const float *inv_t = inv_s + (ct & 1) * BC;
            static_for<0, WC>([&](auto ia) __attribute__((always_inline)) {
                constexpr int A = decltype(ia)::value;
                const int rb = (wc * WC + A) * 32;
                f32x4 w[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) w[g] = *(const f32x4 *)(inv_t + rb + 8 * g + 4 * h);
                const unsigned grp = (unsigned)((c0 + rb) >> 2) + (unsigned)h;  // group of four rows: 8 * run + 2 * g + h
                static_for<0, WQ>([&](auto ib) __attribute__((always_inline)) {
                    constexpr int B = decltype(ib)::value;
                    float m;
                    unsigned g;
                    block_max<A, B>(acc, w, m, g);
                    if (m > bv[B]) {
                        bv[B] = m;
                        bb[B] = grp + 2u * g;
                    }
                });
            });
        }
        ct += tile_done ? 1 : 0;
        ks = tile_done ? 0 : ks + 1;
    };
    // (two slabs per trip with nothing conditional between them: the compiler counts the loads in
    // flight itself and must see that those of the other parity are always the younger ones)
    int t = 0;
    for (; t + 1 < T; t += 2) {
        slab(IC<0>{});
        slab(IC<1>{});
    }
    if (t < T) slab(IC<0>{});
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // reads, loads and writes of the tail have landed
    lds_barrier();
    pipe_reduce_keys<WQ, NWC, BQ, NT>(bv, bb, smem, wc, wq, h, l32, tid, q0, n, slices, s, keys);
}

// ----------------------------------------------------------------------------
// Pair search on the wide tile: the stream of tile pairs of k_pairs_stream (same units, same order, same
// staging of the pairs found) through the pipeline of k_lookup_wide.  Both operands are tiles of the
// centroid array (rows past the live ones exist and have NaN for an inverse length, so they never
// reach the threshold); the inverse lengths of both tiles travel with the first slab of a pair into
// one of two buffers, by the parity of the pair's number: the slab is written to LDS two slabs before
// its first MFMA, i.e. (a pair has at least two slabs) behind the barrier that follows the epilogue
// of the pair before the previous one.
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(WideCfg::NT) __attribute__((amdgpu_waves_per_eu(1, 1), amdgpu_num_vgpr(WIDE_FRAG0))) void k_pairs_wide(
    const bf16_t *__restrict__ C, const float *__restrict__ invn, long K, int d, int qb, float threshold,
    int *__restrict__ out_pairs, long cap, u64 *__restrict__ counter) {
    typedef WideCfg Cfg;
    constexpr int WC = Cfg::WC, WQ = Cfg::WQ, NWC = Cfg::NWC, BC = Cfg::BC, BQ = Cfg::BQ, NW = Cfg::NW, STAGE = Cfg::STAGE,
                  NLA = Cfg::NLA, NL = Cfg::NL, BK = Cfg::BK, RB = Cfg::RB, KK = Cfg::KK, SUB = 32 * Cfg::RB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *inv_a = (float *)(smem + 2 * STAGE);  // [2][BC] inverse lengths of the row tile, by parity of the pair's number
    float *inv_b = inv_a + 2 * BC;               // [2][BQ] and of the column tile
    int *stage = (int *)(inv_b + 2 * BQ);        // [PAIR_STAGE][2] pairs found, moved to the global list when half full
    int *staged = stage + 2 * PAIR_STAGE;
    u64 *flush_slot = (u64 *)(staged + 2);
    unsigned short *masks = (unsigned short *)(flush_slot + 1);  // [NW][WC * WQ][64]: per wave, hit block and lane
    if (threadIdx.x == 0) *staged = 0;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int wc = wave % NWC, wq = wave / NWC;
    const int h = lane >> 5, l32 = lane & 31;
    const int nk = d / BK;
    const int tiles = (int)((K + BC - 1) / BC);

    // the pairs of this workgroup: counted once, then the same sequence twice (loads run ahead of the MFMAs)
    PairItems ld_items, cp_items;
    ld_items.init(tiles, qb);
    cp_items.init(tiles, qb);
    int ld_qt = 0, ld_ct = 0, cp_qt = 0, cp_ct = 0;
    int npairs = 0;
    while (cp_items.next(cp_qt, cp_ct)) ++npairs;
    if (npairs == 0) return;
    const int T = npairs * nk;  // slabs this workgroup walks through
    cp_items.init(tiles, qb);
    cp_items.next(cp_qt, cp_ct);
    ld_items.next(ld_qt, ld_ct);

    // global loads and LDS layout as in k_lookup_wide
    const int lr = lane >> 3, slot = lane & 7;
    const int row0 = wave * 8 + lr;
    const unsigned chunk = (unsigned)((slot ^ ((row0 >> 1) & 7)) * 16);
    const unsigned a_voff = (unsigned)row0 * (unsigned)d * 2u + chunk;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char *)smem;
    unsigned char *wr = smem + wave * 1024 + lane * 16;  // this lane's 16 bytes of load 0 in stage 0
    // (and in stage 1, as a value of its own: an LDS instruction's offset field ends at 64 KiB, and the
    // compiler would rather keep one address per write of that stage than one base)
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
    lds_byte *wr1 = (lds_byte *)(wr + STAGE);
    asm volatile("" : "+v"(wr1));
    const int sw = (l32 >> 1) & 7;
    const unsigned row_a = lds0 + (unsigned)(((wc * WC) * 32 + l32) * RB);
    const unsigned row_b = lds0 + (unsigned)(BC * RB + ((wq * WQ) * 32 + l32) * RB);
    // swizzled 16-byte slot of step kk: ((2 kk + h) ^ sw) * 16 = so0 ^ 32 kk (one register instead of four)
    const unsigned so0 = (unsigned)((h ^ sw) * 16);

    Acc<true, WC, WQ> acc;
    acc.reserve();

    u32x4 G[2][NL];
    float ga0 = 0.f, ga1 = 0.f, gb0 = 0.f, gb1 = 0.f;  // inverse lengths that travel with a pair's first slab
    int gs0 = -1, gs1 = -1;                            // their buffer (parity of the pair's number), -1 = none
    const char *ld_c = (const char *)(C + (size_t)ld_ct * BC * d);  // first element of the slab to load, row tile
    const char *ld_q = (const char *)(C + (size_t)ld_qt * BQ * d);  // and column tile
    int ld_t = 0, ld_ks = 0, ld_seq = 0;
    auto load_part = [&](auto pp, auto jj) __attribute__((always_inline)) {
        constexpr int p = decltype(pp)::value, j = decltype(jj)::value;
        if constexpr (j == 0) {
            float &ga = p == 0 ? ga0 : ga1;
            float &gb = p == 0 ? gb0 : gb1;
            int &gs = p == 0 ? gs0 : gs1;
            gs = -1;
            if (ld_ks == 0) {
                ga = invn[(size_t)ld_ct * BC + wave * 64 + lane];
                gb = invn[(size_t)ld_qt * BQ + wave * 64 + lane];
                gs = ld_seq & 1;
            }
        }
        // (the 32-bit offset is summed up next to its use: a scalar base, the same eight row offsets for both tiles)
        unsigned off = a_voff;
        asm volatile("" : "+v"(off));
        off += (unsigned)((j % NLA) * 64) * (unsigned)d;
        if constexpr (j < NLA) G[p][j] = *(const u32x4 *)(ld_c + off);
        else G[p][j] = *(const u32x4 *)(ld_q + off);
        if constexpr (j == NL - 1) {
            if (ld_t + 1 < T) {
                ++ld_t;
                if (++ld_ks == nk) {
                    ld_ks = 0;
                    ++ld_seq;
                    ld_items.next(ld_qt, ld_ct);
                    ld_c = (const char *)(C + (size_t)ld_ct * BC * d);
                    ld_q = (const char *)(C + (size_t)ld_qt * BQ * d);
                } else {
                    ld_c += BK * 2;
                    ld_q += BK * 2;
                }
            }
        }
    };
    auto write_part = [&](auto pp, auto jj) __attribute__((always_inline)) {
        constexpr int p = decltype(pp)::value, j = decltype(jj)::value;
        if constexpr (j == 0) {
            const int gs = p == 0 ? gs0 : gs1;
            if (gs >= 0) {
                inv_a[gs * BC + wave * 64 + lane] = p == 0 ? ga0 : ga1;
                inv_b[gs * BQ + wave * 64 + lane] = p == 0 ? gb0 : gb1;
            }
        }
        if constexpr (p == 0) *(u32x4 *)(wr + j * NW * 1024) = G[p][j];
        else *(lds_u32x4 *)(wr1 + j * NW * 1024) = G[p][j];
    };
    // steps, barriers and the dealing out of loads and writes between the MFMAs: see k_lookup_wide
    auto step = [&](auto first_tag, auto cur_tag, unsigned addr_a, unsigned addr_b, auto &&extra) __attribute__((always_inline)) {
        constexpr int cur = decltype(cur_tag)::value;
        lgkm_wait<1>();
        static_for<0, WC * WQ>([&](auto ii) __attribute__((always_inline)) {
            constexpr int i = decltype(ii)::value, A = i / WQ, B = i % WQ;
            if constexpr (i == (WC - 1) * WQ) lgkm_wait<4>();
            if constexpr (decltype(first_tag)::value) frag_first<16 * i, Cfg::ra(A), Cfg::rb(cur, B)>();
            else frag_mac<16 * i, Cfg::ra(A), Cfg::rb(cur, B)>();
            extra(ii);
            if constexpr (i < WQ) frag_read<Cfg::rb(1 - cur, i), i * SUB>(addr_b);
            if constexpr (B == WQ - 1) frag_read<Cfg::ra(A), A * SUB>(addr_a);
        });
    };
    auto lds_barrier = [&]() __attribute__((always_inline)) { asm volatile("s_barrier" ::: "memory"); };
    auto xfer = [&](auto pp, auto jj) __attribute__((always_inline)) {
        write_part(pp, jj);
        load_part(pp, jj);
    };
    static_for<0, NL>([&](auto jj) __attribute__((always_inline)) { load_part(IC<0>{}, jj); });
    static_for<0, NL>([&](auto jj) __attribute__((always_inline)) { load_part(IC<1>{}, jj); });
    static_for<0, NL>([&](auto jj) __attribute__((always_inline)) { xfer(IC<0>{}, jj); });
    static_for<0, 4>([&](auto jj) __attribute__((always_inline)) { xfer(IC<1>{}, jj); });
    lgkm_wait<0>();
    lds_barrier();
    static_for<0, WQ>([&](auto kk) __attribute__((always_inline)) {
        constexpr int k = decltype(kk)::value;
        frag_read<Cfg::rb(0, k), k * SUB>(row_b + so0);
    });
    static_for<0, WC>([&](auto kk) __attribute__((always_inline)) {
        constexpr int k = decltype(kk)::value;
        frag_read<Cfg::ra(k), k * SUB>(row_a + so0);
    });

    int ks = 0, cp_seq = 0;
    static_assert(KK == 4, "steps are spelled out");
    auto slab = [&](auto pp) __attribute__((always_inline)) {
        constexpr int p = decltype(pp)::value;
        constexpr unsigned sto = p * STAGE, sto_next = (1 - p) * STAGE;
        auto at = [&](unsigned row, unsigned stg, int k) __attribute__((always_inline)) {
            unsigned sk = so0;
            asm volatile("" : "+v"(sk));  // (summed up here every time instead of kept)
            return (sk ^ (unsigned)(k * 32)) + (row + stg);
        };
        auto part = [&](auto bb_, auto j0, auto ii) __attribute__((always_inline)) {
            constexpr int i = decltype(ii)::value;
            if constexpr (i % 4 == 1) xfer(bb_, IC<decltype(j0)::value + i / 4>{});
        };
        if (ks == 0)  // a pair starts from zero
            step(IC<1>{}, IC<0>{}, at(row_a, sto, 1), at(row_b, sto, 1), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<4>{}, ii); });
        else
            step(IC<0>{}, IC<0>{}, at(row_a, sto, 1), at(row_b, sto, 1), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<4>{}, ii); });
        step(IC<0>{}, IC<1>{}, at(row_a, sto, 2), at(row_b, sto, 2), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<8>{}, ii); });
        step(IC<0>{}, IC<0>{}, at(row_a, sto, 3), at(row_b, sto, 3), [&](auto ii) __attribute__((always_inline)) { part(IC<1 - p>{}, IC<12>{}, ii); });
        lgkm_wait<0>();
        lds_barrier();
        step(IC<0>{}, IC<1>{}, at(row_a, sto_next, 0), at(row_b, sto_next, 0), [&](auto ii) __attribute__((always_inline)) { part(pp, IC<0>{}, ii); });
        __builtin_amdgcn_sched_barrier(0);
        const bool pair_done = ks == nk - 1;
        if (pair_done) {
            // Every product above the threshold is a pair (column index < row index).  Per block the largest
            // product under a wave ballot; a block with a pair (few have one) leaves a bit mask of its pairs per
            // lane in LDS, and the masks are turned into list entries afterwards, block after block, by code that
            // exists once.
            const long c0 = (long)cp_ct * BC, q0 = (long)cp_qt * BQ;
            const int ahead = (int)(c0 - q0 < 4096 ? c0 - q0 : 4096);  // rows by which the row tile is ahead: 0 on the diagonal
            const float *inv_t = inv_a + (cp_seq & 1) * BC;
            const float *inv_q = inv_b + (cp_seq & 1) * BQ;
            unsigned short *my_masks = masks + wave * (WC * WQ * 64) + lane;  // [hit][lane] of this wave
            // (taken from the optimiser's sight: it would keep one register per block and product, all through the
            // kernel, for the sums this value goes into)
            int lane_part = l32 - 4 * h;
            asm volatile("" : "+v"(lane_part));
            int nhit = 0;
            u64 hit_blocks = 0;  // four bits per hit: A * WQ + B
            {
                float wi[WQ];
#pragma unroll
                for (int b = 0; b < WQ; ++b) wi[b] = inv_q[(wq * WQ + b) * 32 + l32];
                static_for<0, WC>([&](auto ia) __attribute__((always_inline)) {
                    constexpr int A = decltype(ia)::value;
                    f32x4 w[4];
#pragma unroll
                    for (int g = 0; g < 4; ++g) w[g] = *(const f32x4 *)(inv_t + (wc * WC + A) * 32 + 8 * g + 4 * h);
                    static_for<0, WQ>([&](auto ib) __attribute__((always_inline)) {
                        constexpr int B = decltype(ib)::value;
                        const float m = fmaxf(fmaxf(group_max<A, B, 0>(acc, w[0]), group_max<A, B, 1>(acc, w[1])),
                                              fmaxf(group_max<A, B, 2>(acc, w[2]), group_max<A, B, 3>(acc, w[3])));
                        if (__ballot(m * wi[B] > threshold) != 0) {
                            // product I belongs to row (wc * WC + A) * 32 + 4 * h + 8 * (I / 4) + I % 4 of the row tile,
                            // which is a pair if the column comes before it: column - first row < 8 * (I / 4) + I % 4
                            const int before = lane_part - ahead + ((wq * WQ + B) - (wc * WC + A)) * 32;
                            unsigned found = 0;
                            static_for<0, 16>([&](auto ii) __attribute__((always_inline)) {
                                constexpr int I = decltype(ii)::value;
                                const float sim = acc.template get<A, B, I>() * w[I >> 2][I & 3] * wi[B];
                                if (sim > threshold && before < 8 * (I >> 2) + (I & 3)) found |= 1u << I;
                            });
                            my_masks[nhit * 64] = (unsigned short)found;
                            hit_blocks |= (u64)(A * WQ + B) << (4 * nhit);
                            ++nhit;
                        }
                    });
                });
            }
            for (int e = 0; e < nhit; ++e) {
                const int blk = (int)(hit_blocks >> (4 * e)) & 15;
                const unsigned found = my_masks[e * 64];
                const int icol = (int)q0 + (wq * WQ + blk % WQ) * 32 + l32;
                const int jrow0 = (int)c0 + (wc * WC + blk / WQ) * 32 + 4 * h;
                emit_pairs_staged(found, icol, [&](int I) { return jrow0 + 8 * (I >> 2) + (I & 3); }, stage, staged, PAIR_STAGE,
                                  out_pairs, cap, counter);
            }
            ++cp_seq;
            cp_items.next(cp_qt, cp_ct);
            // the pairs of this tile pair are staged (own LDS traffic done, then the barrier by hand: the
            // compiler's barrier would also wait for the global loads in flight)
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            if (*staged > PAIR_STAGE / 2) flush_staged_pairs(stage, staged, PAIR_STAGE, flush_slot, out_pairs, cap, counter);
        }
        ks = pair_done ? 0 : ks + 1;
    };
    int t = 0;
    for (; t + 1 < T; t += 2) {
        slab(IC<0>{});
        slab(IC<1>{});
    }
    if (t < T) slab(IC<0>{});
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // reads, loads and writes of the tail have landed
    lds_barrier();
    flush_staged_pairs(stage, staged, PAIR_STAGE, flush_slot, out_pairs, cap, counter);
}

typedef PipeCfg<4, 2, 2, 4, 2> PipeLarge;  // 256 x 256 tile, waves of 128 x 64, two stages
typedef PipeCfg<2, 2, 4, 2, 3, 64, true> PipeMid;    // 256 x 128 tile, waves of 64 x 64, three stages; keys carry rows
typedef PipeCfg<1, 2, 8, 1, 3, 64, true> PipeSmall;  // 256 x 64 tile, waves of 32 x 64, three stages; keys carry rows
typedef PipeCfg<4, 2, 2, 4, 4, 32> PipeLarge32;  // 256 x 256 tile, slabs of 32 elements, four stages
// the same three tiles over E4M3 codes (slabs of 128 codes); all of their keys carry rows
typedef PipeCfg<4, 2, 2, 4, 2, 128, true, 1> F8Large;
typedef PipeCfg<2, 2, 4, 2, 3, 128, true, 1> F8Mid;
typedef PipeCfg<1, 2, 8, 1, 3, 128, true, 1> F8Small;
typedef PipeCfg<4, 2, 2, 4, 2, 128, true, 1, true> F8Large64;  // the same three tiles on 64-deep MFMAs
typedef PipeCfg<2, 2, 4, 2, 3, 128, true, 1, true> F8Mid64;
typedef PipeCfg<1, 2, 8, 1, 3, 128, true, 1, true> F8Small64;

// ----------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------
struct PipePlan {
    int cfg, bc, bq, tiles_per_slice, slices, nqt, qb;
    long grid;
};

// cfg: 1 = PipeLarge, 2 = PipeMid, 3 = PipeSmall, 4 = PipeLarge32, 5 = the wide kernel (same tile as 1)
static bool pipe_plan(const siso_cache *c, long n, int cfg, long want_wgs, PipePlan *p) {
    if (c->count < 1 || n < 1) return false;
    if (c->dtype == SISO_FP8) {  // slabs of 128 codes, at least two per tile
        if (c->dim % 128 != 0 || c->dim < 256) return false;
        if (cfg == 4 || cfg == 5) cfg = 1;
        if (cfg >= 6 && cfg <= 8) {  // the three tiles on 64-deep MFMAs (plans like configurations 1 to 3)
            const bool ok = pipe_plan(c, n, cfg - 5, want_wgs, p);
            p->cfg = cfg;
            return ok;
        }
    } else if (c->dtype != SISO_BF16 || c->dim % 64 != 0 || c->dim < 128) {
        return false;
    }
    if (cfg < 1 || cfg > 5) return false;
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
    if (c->plan_min_slices > 0) {  // a top-k lookup wants many slices: each contributes one row to its bound
        const long want_s = c->plan_min_slices < ct ? c->plan_min_slices : ct;
        const long t2 = ct / want_s > 1 ? ct / want_s : 1;
        if (tps > t2) tps = t2;
    }
    if (tps > ct) tps = ct;
    // query tiles per unit: 8 when there are that many (a centroid tile fetched into an XCD's L2 then
    // serves 8 workgroups, and 8 query tiles are about what stays resident in a 4 MB L2), fewer when the
    // batch is small; a unit should be full, so with few centroid tiles the slices get shorter until
    // there are 32/qb of them, and with very few tiles more query tiles share one
    int qb = c->opt_mfma_qblock > 0 ? c->opt_mfma_qblock : 8;
    if (qb != 1 && qb != 2 && qb != 4 && qb != 8 && qb != 16 && qb != 32) return false;
    if (c->opt_mfma_qblock <= 0) {
        // (any number from 1 to 32 will do for the kernels: a unit then uses qb * (32 / qb) of its 32 places)
        if (qb > nqt) qb = (int)nqt;
        if (c->opt_tiles_per_slice <= 0 && (ct + tps - 1) / tps < 32 / qb) tps = ct / (32 / qb) > 1 ? ct / (32 / qb) : 1;
        while (qb < 32 && qb * 2 <= nqt && (ct + tps - 1) / tps < 32 / qb) qb <<= 1;
        // blocks of query tiles of even size: 9 tiles as 5 + 4 rather than 8 + 1 (a block's places without a tile
        // stay empty: 9 tiles in blocks of 8 took as long as 11 tiles' worth of work)
        const long nqb = (nqt + qb - 1) / qb;
        qb = (int)((nqt + nqb - 1) / nqb);
    }
    // The groups of slices are dealt out to the XCDs in turn (pipe_map_block), and the 32 compute units of an XCD
    // take its workgroups (a slice x a query tile each, equally long) in rounds: a slice length that leaves the
    // last round of groups to a few XCDs, or the last round of workgroups to a few units, makes the rest wait
    // (3 query tiles over 1,024 centroid tiles: 11 groups of 6-tile slices put twice the work on three XCDs, 482 us;
    // 8 groups of 8-tile slices, 336 us).  Among the lengths up to the one chosen above, take the one with the
    // fewest tile periods on the busiest XCD, a round counted as its tiles plus half a tile for getting started.
    if (c->opt_tiles_per_slice <= 0 && c->plan_min_slices <= 0 && nqt > 1) {
        const long sb = 32 / qb;
        const long lo = tps / 4 > 2 ? tps / 4 : (tps < 2 ? tps : 2);
        auto periods = [&](long t) -> double {  // < 0: the other mapping (every XCD has a share of every group)
            const long sl = (ct + t - 1) / t, gr = (sl + sb - 1) / sb;
            if (gr <= 4) return -1.0;
            long busiest = 0;
            for (long x = 0; x < 8 && x < gr; ++x) {  // XCD x owns the groups x, x + 8, ...
                long mine = 0;
                for (long g = x; g < gr; g += 8) mine += (g + 1) * sb <= sl ? sb : sl - g * sb;
                if (mine > busiest) busiest = mine;
            }
            const long rounds = (busiest * nqt + 31) / 32;
            return (double)rounds * ((double)t + 0.5);
        };
        long best = tps;
        double least = periods(tps);
        if (least >= 0)
            for (long t = tps - 1; t >= lo; --t) {
                const double w = periods(t);
                if (w >= 0 && w < least * 0.99) {
                    least = w;
                    best = t;
                }
            }
        tps = best;
    }
    const long slices = (ct + tps - 1) / tps;
    if (nqt * slices > 2147483647L || slices > 1000000) return false;
    p->tiles_per_slice = (int)tps;
    p->slices = (int)slices;
    p->nqt = (int)nqt;
    p->qb = qb;
    p->grid = pipe_grid(slices, nqt, qb);
    if (p->grid > 2147483647L) return false;
    return true;
}

static bool mfma_plan(const siso_cache *c, long n, PipePlan *p) {
    int cfg = c->opt_mfma_config;
    if (cfg == 0 && c->dtype == SISO_FP8) cfg = n <= 64 ? 8 : n <= 128 ? 7 : 6;  // the 64-deep MFMAs
    if (cfg == 0) cfg = n <= 64 ? 3 : n <= 128 ? 2 : 5;
    // about two workgroups per compute unit when there is enough work
    return pipe_plan(c, n, cfg, 512, p);
}

static bool skinny_plan(const siso_cache *c, long n, PipePlan *p) {
    if (n > 64) return false;
    // exactly one workgroup per compute unit: every one streams an equal share of the centroids
    return pipe_plan(c, n, c->dtype == SISO_FP8 && c->opt_mfma_config != 3 ? 8 : 3, 256, p);
}

// Should the centroid loads of a launch carry the non-temporal hint?  With one tile of queries every centroid
// line is read by exactly one workgroup, once: marked as streaming, 384 MiB of centroids pass in 63 us instead
// of 72 (they no longer push each other through the caches).  A set that the 256 MB memory-side cache can hold
// most of is better left there for the next call (192 MiB: 30.0 us per pass unmarked, 32.7 marked; the two meet
// at 288 MiB, rows and codes alike); and with several query tiles the workgroups of an XCD share the lines in
// L2, where the mark makes them leave early (large batches over codes: 6 % slower marked; over bf16 rows, wide
// kernel: 1.5 %).
#define SISO_STREAM_BYTES (288l << 20)
static bool stream_hint(const siso_cache *c, const PipePlan &p) {
    if (c->opt_stream_hint > 0) return c->opt_stream_hint == 1;
    const long bytes = c->count * (long)c->dim * (c->dtype == SISO_FP8 ? 1 : 2);
    return p.nqt == 1 && bytes > SISO_STREAM_BYTES;
}

template <class Cfg, bool COLLECT, bool STREAM>
static int pipe_attr(siso_cache *c) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lookup_pipe<Cfg, COLLECT, STREAM>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, Cfg::LDS_BYTES);
        if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(k_lookup_pipe)");
        attr_done = true;
    }
    return SISO_OK;
}

template <class Cfg, bool STREAM>
static int launch_cfg2(siso_cache *c, const void *queries, long n, const PipePlan &p, u64 *keys) {
    const int rc = pipe_attr<Cfg, false, STREAM>(c);
    if (rc != SISO_OK) return rc;
    hipLaunchKernelGGL((k_lookup_pipe<Cfg, false, STREAM>), dim3((unsigned)p.grid), dim3(Cfg::NT), Cfg::LDS_BYTES,
                       c->stream, (const bf16_t *)queries, (const bf16_t *)c->cent, c->invn, n, c->count, c->dim,
                       p.tiles_per_slice, p.slices, p.nqt, p.qb, keys, (const float *)nullptr, (int *)nullptr,
                       (int *)nullptr, 0, c->board_to_clear);
    c->board_to_clear = nullptr;  // taken
    return siso_check_hip(c, hipGetLastError(), "k_lookup_pipe");
}
template <class Cfg>
static int launch_cfg(siso_cache *c, const void *queries, long n, const PipePlan &p, u64 *keys) {
    return stream_hint(c, p) ? launch_cfg2<Cfg, true>(c, queries, n, p, keys) : launch_cfg2<Cfg, false>(c, queries, n, p, keys);
}

template <class Cfg, bool STREAM>
static int launch_collect2(siso_cache *c, const void *queries, long n, const PipePlan &p, const float *tau, int *cand,
                           int *cnt, int cap) {
    const int rc = pipe_attr<Cfg, true, STREAM>(c);
    if (rc != SISO_OK) return rc;
    hipLaunchKernelGGL((k_lookup_pipe<Cfg, true, STREAM>), dim3((unsigned)p.grid), dim3(Cfg::NT), Cfg::LDS_BYTES,
                       c->stream, (const bf16_t *)queries, (const bf16_t *)c->cent, c->invn, n, c->count, c->dim,
                       p.tiles_per_slice, p.slices, p.nqt, p.qb, (u64 *)nullptr, tau, cand, cnt, cap, (u64 *)nullptr);
    return siso_check_hip(c, hipGetLastError(), "k_lookup_pipe (collect)");
}
template <class Cfg>
static int launch_collect(siso_cache *c, const void *queries, long n, const PipePlan &p, const float *tau, int *cand,
                          int *cnt, int cap) {
    return stream_hint(c, p) ? launch_collect2<Cfg, true>(c, queries, n, p, tau, cand, cnt, cap)
                             : launch_collect2<Cfg, false>(c, queries, n, p, tau, cand, cnt, cap);
}

// The wide kernel runs with several query tiles: its workgroups share the centroid lines in L2 either way.  A set
// that the memory-side cache holds is faster unmarked (96 MiB: 1.2 %, on every machine tried); over 2 GiB the two
// are within 1.7 % of each other, one ahead on one machine and the other on the next, and the marked loads move
// less through the fabric (35-43 GiB a launch against 48-118): marked there.
static bool stream_hint_wide(const siso_cache *c) {
    if (c->opt_stream_hint > 0) return c->opt_stream_hint == 1;
    return c->count * (long)c->dim * 2 > SISO_STREAM_BYTES;
}

template <bool STREAM>
static int launch_wide2(siso_cache *c, const void *queries, long n, const PipePlan &p, u64 *keys) {
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void *)k_lookup_wide<STREAM>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, WideCfg::LDS_BYTES);
        if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(k_lookup_wide)");
        attr_done = true;
    }
    hipLaunchKernelGGL((k_lookup_wide<STREAM>), dim3((unsigned)p.grid), dim3(WideCfg::NT), WideCfg::LDS_BYTES, c->stream,
                       (const bf16_t *)queries, (const bf16_t *)c->cent, c->invn, n, c->count, c->dim, p.tiles_per_slice,
                       p.slices, p.nqt, p.qb, keys);
    return siso_check_hip(c, hipGetLastError(), "k_lookup_wide");
}
static int launch_wide(siso_cache *c, const void *queries, long n, const PipePlan &p, u64 *keys) {
    return stream_hint_wide(c) ? launch_wide2<true>(c, queries, n, p, keys) : launch_wide2<false>(c, queries, n, p, keys);
}

static int pipe_launch(siso_cache *c, const void *queries, long n, const PipePlan &p, u64 *keys) {
    if (((uintptr_t)queries & 15) != 0) return siso_fail(c, SISO_EINVAL, "bf16 lookup: queries must be 16-byte aligned");
    if (c->dtype == SISO_FP8) {  // `queries` are codes here (the caller has quantised the batch)
        switch (p.cfg) {
            case 2: return launch_cfg<F8Mid>(c, queries, n, p, keys);
            case 3: return launch_cfg<F8Small>(c, queries, n, p, keys);
            case 6: return launch_cfg<F8Large64>(c, queries, n, p, keys);
            case 7: return launch_cfg<F8Mid64>(c, queries, n, p, keys);
            case 8: return launch_cfg<F8Small64>(c, queries, n, p, keys);
            default: return launch_cfg<F8Large>(c, queries, n, p, keys);
        }
    }
    switch (p.cfg) {
        case 1: return launch_cfg<PipeLarge>(c, queries, n, p, keys);
        case 2: return launch_cfg<PipeMid>(c, queries, n, p, keys);
        case 3: return launch_cfg<PipeSmall>(c, queries, n, p, keys);
        case 4: return launch_cfg<PipeLarge32>(c, queries, n, p, keys);
        default: return launch_wide(c, queries, n, p, keys);
    }
}

int siso_mfma_slices(const siso_cache *c, long n) {
    PipePlan p;
    return mfma_plan(c, n, &p) ? p.slices : 0;
}

// what the keys of a kernel carry
static int keys_carry_rows(const siso_cache *c, const PipePlan &p) {
    if (c->dtype == SISO_FP8) return SISO_KEY_ROWS;
    return (p.cfg == 2 && PipeMid::ROWS) || (p.cfg == 3 && PipeSmall::ROWS) ? SISO_KEY_ROWS : SISO_KEY_GROUPS4;
}

int siso_mfma_launch(siso_cache *c, const void *queries, long n, int slices, u64 *keys, int *row_keys) {
    PipePlan p;
    if (!mfma_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "mfma lookup: plan mismatch");
    *row_keys = keys_carry_rows(c, p);
    return pipe_launch(c, queries, n, p, keys);
}

int siso_skinny_slices(const siso_cache *c, long n) {
    PipePlan p;
    return skinny_plan(c, n, &p) ? p.slices : 0;
}

int siso_skinny_launch(siso_cache *c, const void *queries, long n, int slices, u64 *keys, int *row_keys) {
    PipePlan p;
    if (!skinny_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "skinny lookup: plan mismatch");
    *row_keys = keys_carry_rows(c, p);
    return pipe_launch(c, queries, n, p, keys);
}

// ----------------------------------------------------------------------------
// the two passes of a top-k lookup (the caller has set c->plan_min_slices)
// ----------------------------------------------------------------------------
int siso_topk_mfma_slices(const siso_cache *c, long n) {
    PipePlan p;
    return mfma_plan(c, n, &p) ? p.slices : 0;
}

int siso_topk_mfma_pass1(siso_cache *c, const void *queries, long n, int slices, u64 *keys, int *row_keys) {
    PipePlan p;
    if (!mfma_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "top-k lookup: plan mismatch");
    *row_keys = keys_carry_rows(c, p);
    return pipe_launch(c, queries, n, p, keys);
}

int siso_topk_mfma_collect(siso_cache *c, const void *queries, long n, int slices, const float *tau, int *cand,
                           int *cnt, int cap) {
    PipePlan p;
    if (!mfma_plan(c, n, &p) || p.slices != slices) return siso_fail(c, SISO_EINVAL, "top-k lookup: plan mismatch");
    if (((uintptr_t)queries & 15) != 0) return siso_fail(c, SISO_EINVAL, "top-k lookup: queries must be 16-byte aligned");
    if (c->dtype == SISO_FP8) {  // (`queries` are codes; the two passes run on the 64-deep kernels only)
        switch (p.cfg) {
            case 6: return launch_collect<F8Large64>(c, queries, n, p, tau, cand, cnt, cap);
            case 7: return launch_collect<F8Mid64>(c, queries, n, p, tau, cand, cnt, cap);
            case 8: return launch_collect<F8Small64>(c, queries, n, p, tau, cand, cnt, cap);
            default: return siso_fail(c, SISO_EINVAL, "top-k lookup: no collecting kernel for configuration %d", p.cfg);
        }
    }
    if (c->dtype != SISO_BF16) return siso_fail(c, SISO_EINVAL, "top-k lookup: bf16 and 8-bit caches only");
    switch (p.cfg) {
        case 2: return launch_collect<PipeMid>(c, queries, n, p, tau, cand, cnt, cap);
        case 3: return launch_collect<PipeSmall>(c, queries, n, p, tau, cand, cnt, cap);
        case 4: return launch_collect<PipeLarge32>(c, queries, n, p, tau, cand, cnt, cap);
        default: return launch_collect<PipeLarge>(c, queries, n, p, tau, cand, cnt, cap);  // also for the wide kernel's plan: same tiles
    }
}

// ----------------------------------------------------------------------------
// pair search (siso_merge) on the same kernel
// ----------------------------------------------------------------------------
int siso_pairs_mfma_supported(const siso_cache *c, long count) {
    if (c->opt_merge_config == 1) return 0;  // 1 = force the scalar kernel
    return c->dtype == SISO_BF16 && c->dim % 64 == 0 && c->dim >= 128 && count >= 2;
}

int siso_pairs_mfma_launch(siso_cache *c, const void *rows, const float *invn, long count, float threshold,
                           int *out_pairs, long cap, u64 *counter) {
    if (((uintptr_t)rows & 15) != 0) return siso_fail(c, SISO_EINVAL, "pair search: rows must be 16-byte aligned");
    // one stream of tile pairs per workgroup, one workgroup per compute unit
    const long T = (count + WideCfg::BC - 1) / WideCfg::BC;
    if (T > 1000000) return siso_fail(c, SISO_EINVAL, "pair search: too many tiles");
    int qb = 8;
    while (qb > 1 && qb > T) qb >>= 1;
    constexpr int room = 2 * WideCfg::BC * 4 + 2 * WideCfg::BQ * 4 + PAIR_STAGE * 8 + 16;  // inverse lengths, staged pairs
    static bool attr_done[2] = {false, false};
    if (c->opt_merge_config != 2) {  // 2 = the four-wave kernel below
        typedef PipeLarge Cfg;
        constexpr int lds = Cfg::NSTAGE * Cfg::STAGE + room;
        static_assert(lds <= 160 * 1024, "fits in LDS");
        if (!attr_done[0]) {
            hipError_t e = hipFuncSetAttribute((const void *)k_pairs_stream<Cfg>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(k_pairs_stream)");
            attr_done[0] = true;
        }
        hipLaunchKernelGGL((k_pairs_stream<Cfg>), dim3(256), dim3(Cfg::NT), lds, c->stream, (const bf16_t *)rows, invn, count,
                           c->dim, qb, threshold, out_pairs, cap, counter);
        return siso_check_hip(c, hipGetLastError(), "k_pairs_stream");
    }
    constexpr int lds = 2 * WideCfg::STAGE + room + WideCfg::NW * WideCfg::WC * WideCfg::WQ * 64 * 2;  // and the pair masks
    static_assert(lds <= 160 * 1024, "fits in LDS");
    if (!attr_done[1]) {
        hipError_t e = hipFuncSetAttribute((const void *)k_pairs_wide, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return siso_check_hip(c, e, "hipFuncSetAttribute(k_pairs_wide)");
        attr_done[1] = true;
    }
    hipLaunchKernelGGL(k_pairs_wide, dim3(256), dim3(WideCfg::NT), lds, c->stream, (const bf16_t *)rows, invn, count, c->dim, qb,
                       threshold, out_pairs, cap, counter);
    return siso_check_hip(c, hipGetLastError(), "k_pairs_wide");
}

// The dense contraction of DBDPC (Alg. 2): Gram matrix of the clustering keys on the matrix
// cores, turned into cosines (Eq. 5) in the epilogue and consumed on the spot:
//   MODE_DENSITY  kept x kept  : density terms exp(-d/d_n) summed per column in fp64 (Eq. 6),
//                                one bit per pair "cosine distance <= d_c (+ margin)", and a
//                                list of the pairs too close to d_c for fp32 to decide;
//   MODE_CAND     centres x pruned : per pruned token (a column) and group of 64 centres, the
//                                largest cosine of the group and one bit per centre that is
//                                within reach (alpha*d_c + margin) and can still be the
//                                nearest of its group (candidates for Eq. 8).
// The distance matrix itself is never written.
//
// Shape of the kernel (gfx950):
//  * one workgroup of 8 wavefronts per CU owns a (64*MI) x 256 output tile, MI = 4 or 2: 256x256
//    halves the L2 traffic per flop of 128x128 tiles (the L2 -> CU path is what limits this
//    contraction at a key width of 512), 128x256 is for launches that would otherwise leave
//    CUs without a tile; each wavefront computes (32*MI) x 64 of it as MI x 2
//    v_mfma_f32_32x32x16_bf16 accumulators (fp32 keys: as three bf16 planes, six passes);
//  * the key rows stream in 128-byte slices (whole cache lines: eight lanes fetch one row's
//    line) straight from global memory into a ring of LDS stages (global_load_lds_dwordx4: no
//    staging registers); waits on the ring are explicit (s_waitcnt vmcnt + s_barrier);
//  * both operands are rows of the same key matrix, so a lane takes 16 contiguous bytes of
//    "its" row per MFMA; the eight 16-byte chunks of a row slice are XOR-swizzled by the row
//    number so that 16 consecutive rows read conflict-free; the fragments of the next k-group
//    are read from LDS while the MFMAs of the current one run;
//  * the grid is persistent (the tile count depends on counts only the device knows) and
//    XCD-aware: each of the 8 XCDs (own L2) works on its own band of tile columns;
//  * density pass of a sample with more 256 x 256 tiles than workgroups: d_ij = d_ji, so only the
//    tiles on and above the diagonal are computed, and a tile above it also leaves the row sums,
//    the transposed bits and the flagged near-d_c pairs of its mirror image (template SYM).
#include <type_traits>

#include "pact_internal.h"

namespace pact {

enum { MODE_DENSITY = 0, MODE_CAND = 1 };

struct GramArgs {
    const char* keys;          // [total, dk]
    int32_t dk;
    const int32_t* idx_rows;   // sample-local token index of row position p (global offset base)
    const int32_t* idx_cols;
    const pact_report* rep;
    const float* rinv;         // [total] 1/|u| (0 for a zero vector)
    const char* zeros;         // >= 16 zero bytes (source of the slices past the key width)
    uint64_t* adj;             // [B][n_max][W]
    float* cbest;              // candidate pass: [B][W][n_max] largest cosine per (group of 64 centres, pruned token)
    double* rho_part;          // [B][W][n_max], one row per GRAM_RHO_ROWS kept rows
    uint32_t* near_list;       // [B][NEAR_CAP][2]
    int32_t* near_cnt;         // [B][2]: list slots taken, ordered pairs they stand for (8-byte aligned)
    uint32_t* stat;            // [B][stat_wgs * 8] per wavefront: bits of the most negative density exponent
                               // it saw (largest distance), or NULL when the statistic is not wanted
    int32_t stat_wgs;          // workgroup slots per sample in `stat`
    float margin;              // worst-case fp32 error of a cosine
    // Batches (mapped != 0): a one-dimensional grid of GRAM_MAX_WORKGROUPS workgroups, shared out
    // among the samples by size; workgroup i serves sample wg_map[i] >> 8 as its workgroup number
    // wg_map[i] & 255 of wg_count[sample] (0xFFFF: a spare workgroup).
    int32_t mapped;
    uint16_t wg_count[PACT_MAX_BATCH];
    uint16_t wg_map[GRAM_MAX_WORKGROUPS];
};

constexpr int TILE_C = 256;
constexpr int SLICE_BYTES = 128;           // bytes of each row per stage: 8 chunks of 16 B = one cache line
constexpr int LDS_BUDGET = 160 * 1024 - 4096;

template <int MI> struct Shape {
    static constexpr int TILE_R = 64 * MI;                              // 2 wavefront rows x MI x 32
    static constexpr int STAGE_BYTES = (TILE_R + TILE_C) * SLICE_BYTES; // A rows then B rows
    static constexpr int NSTAGE = (LDS_BUDGET / STAGE_BYTES) < 4 ? (LDS_BUDGET / STAGE_BYTES) : 4;
    static constexpr int AHEAD = NSTAGE - 1;                            // slices in flight besides the one being multiplied
    static constexpr int NB = (TILE_R + TILE_C) / 64;                   // 1 KB blocks (8 rows) each wavefront brings per stage
    static constexpr size_t LDS_BYTES = (size_t)NSTAGE * STAGE_BYTES + TILE_R * sizeof(float) + 4 * 64 * sizeof(double);
    static_assert(NSTAGE >= 2, "the ring needs a slot to fill while another is multiplied");
};

typedef __attribute__((address_space(3))) char lds_char;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4_t lds_u32x4;
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) u32x2_t lds_uint2;
typedef __attribute__((address_space(3))) double lds_f64;
constexpr int NEAR_BUF = 512;              // undecided pairs a wavefront buffers before reserving list slots (> 32)

// 16 bytes per lane, global -> LDS at (lds_base + lane * 16); asynchronous, counted by vmcnt.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_base) : "memory");
}
// The same with the address as a scalar base plus a 32-bit offset per lane (one add per fetch).
__device__ __forceinline__ void dma16_off(const char* base, uint32_t off, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(off), "s"(base), "s"(lds_base) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// v = value in lane `l` of a wavefront-wide register (value and lane are wave-uniform)
// Files the two halves of two ballots (m0: columns 0-31 of rows L and L+4, m1: columns 32-63)
// under lanes L and L+4 of `lo` / `hi`.  (The compiler cannot see into the asm to pad the
// distance a VALU-written scalar needs before another VALU instruction reads it, hence the s_nop.)
template <int L> __device__ __forceinline__ void file_ballots(uint32_t& lo, uint32_t& hi, uint64_t m0, uint64_t m1) {
    asm("s_nop 1\n\t"
        "v_writelane_b32 %0, %2, %6\n\t"
        "v_writelane_b32 %1, %4, %6\n\t"
        "v_writelane_b32 %0, %3, %7\n\t"
        "v_writelane_b32 %1, %5, %7"
        : "+v"(lo), "+v"(hi)
        : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)),
          "n"(L), "n"(L + 4));
}
// The same for two sets of ballots at once (m -> lo/hi, h -> lo2/hi2).
template <int L> __device__ __forceinline__ void file_ballots2(uint32_t& lo, uint32_t& hi, uint32_t& lo2, uint32_t& hi2,
                                                               uint64_t m0, uint64_t m1, uint64_t h0, uint64_t h1) {
    asm("s_nop 1\n\t"
        "v_writelane_b32 %0, %4, %12\n\t"
        "v_writelane_b32 %1, %6, %12\n\t"
        "v_writelane_b32 %0, %5, %13\n\t"
        "v_writelane_b32 %1, %7, %13\n\t"
        "v_writelane_b32 %2, %8, %12\n\t"
        "v_writelane_b32 %3, %10, %12\n\t"
        "v_writelane_b32 %2, %9, %13\n\t"
        "v_writelane_b32 %3, %11, %13"
        : "+v"(lo), "+v"(hi), "+v"(lo2), "+v"(hi2)
        : "s"((uint32_t)m0), "s"((uint32_t)(m0 >> 32)), "s"((uint32_t)m1), "s"((uint32_t)(m1 >> 32)),
          "s"((uint32_t)h0), "s"((uint32_t)(h0 >> 32)), "s"((uint32_t)h1), "s"((uint32_t)(h1 >> 32)),
          "n"(L), "n"(L + 4));
}
// body(std::integral_constant<int, 0>{}) ... body(std::integral_constant<int, N-1>{})
// value of the lane whose number differs by XOR (1, 2, 4, 8 or 16): a swizzle inside each
// group of 32 lanes, which needs no address register
template <int XOR> __device__ __forceinline__ double swizzle_xor(double v) {
    static_assert(XOR >= 1 && XOR < 32, "within 32 lanes");
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    if constexpr (XOR < 16) {
        // inside a row of 16 lanes the vector unit's own lane permutes do it (no trip through the LDS
        // crossbar): quad permutes for 1 and 2, a rotation by 8 for 8, and for 4 a shift by 4 either
        // way, each written to the banks of 4 lanes whose partner lies that way
        auto half = [](int w) __attribute__((always_inline)) {
            if constexpr (XOR == 1) return __builtin_amdgcn_update_dpp(w, w, 0xB1, 0xF, 0xF, false);
            else if constexpr (XOR == 2) return __builtin_amdgcn_update_dpp(w, w, 0x4E, 0xF, 0xF, false);
            else if constexpr (XOR == 8) return __builtin_amdgcn_update_dpp(w, w, 0x128, 0xF, 0xF, false);
            else {
                static_assert(XOR == 4, "1, 2, 4 or 8");
                const int t = __builtin_amdgcn_update_dpp(w, w, 0x104, 0xF, 0x5, false);    // row_shl:4 -> banks 0, 2
                return __builtin_amdgcn_update_dpp(t, w, 0x114, 0xF, 0xA, false);           // row_shr:4 -> banks 1, 3
            }
        };
        const uint32_t lo = (uint32_t)half((int)(uint32_t)u), hi = (uint32_t)half((int)(uint32_t)(u >> 32));
        return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
    }
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)u, (XOR << 10) | 0x1f);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_swizzle((int)(uint32_t)(u >> 32), (XOR << 10) | 0x1f);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
template <int N, int I = 0, class F> __device__ __forceinline__ void static_for(F&& body) {
    if constexpr (I < N) {
        body(std::integral_constant<int, I>{});
        static_for<N, I + 1>(body);
    }
}

template <int DT> struct Mfma;
template <> struct Mfma<PACT_BF16> {
    __device__ static __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                    __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<PACT_F32X3> : Mfma<PACT_BF16> {};

// Density pass with t x t square tiles on g workgroups: do mirrored tiles (upper triangle only,
// longer epilogue) save at least one turn in eight of a workgroup's tile loop?
__host__ __device__ __forceinline__ bool mirrored_tiles_pay(int t, int g) {
    const long full = (long)t * t, tri = (long)t * (t + 1) / 2;
    return ((tri + g - 1) / g) * 9 < ((full + g - 1) / g) * 8;
}

template <int DT, int MODE, int MI, bool STAT, bool SYM>
__global__ __launch_bounds__(512, 2) void gram_kernel(Batch bt, GramArgs ga) {
    typedef Shape<MI> SH;
    constexpr int TILE_R = SH::TILE_R, STAGE_BYTES = SH::STAGE_BYTES, NSTAGE = SH::NSTAGE;
    constexpr int AHEAD = SH::AHEAD, NB = SH::NB, WROWS = 32 * MI;
    extern __shared__ uint4 s_ring[];                         // NSTAGE stages, TILE_R floats, 256 doubles
    // Which sample, which of its workgroups, and how many it has.  Batches: read from the map the
    // host made.  Workgroups are dealt to the 8 XCDs round-robin in launch order (XCD = workgroup
    // number mod 8) and every XCD has its own L2; the map gives a sample workgroups of one XCD
    // where it can, so that the sample's keys (a few MB) stay in that L2 instead of passing
    // through all eight, and it gives large samples more workgroups than small ones.
    int b = blockIdx.y, wg = blockIdx.x, G = gridDim.x;
    if (ga.mapped) {
        const uint32_t e = ga.wg_map[blockIdx.x];
        if (e == 0xFFFFu) return;
        b = (int)(e >> 8);
        wg = (int)(e & 255u);
        G = ga.wg_count[b];
    }
    if (STAT && wg == 0)                                      // slots no workgroup of this sample writes
        for (int k = threadIdx.x; k < (ga.stat_wgs - G) * 8; k += 512) ga.stat[((size_t)b * ga.stat_wgs + G) * 8 + k] = 0u;
    const Seg sg = bt.s[b];
    const int q_kept = clamp_count(ga.rep[b].n_kept, sg.n);
    // density pass: kept x kept; candidate pass: rows are the centres, columns the pruned tokens
    // (what is wanted there is per pruned token, and a lane holds 16 rows of one column)
    const int nA = (MODE == MODE_DENSITY) ? q_kept : clamp_count(ga.rep[b].n_centers, q_kept);
    const int nB = (MODE == MODE_DENSITY) ? q_kept : clamp_count(ga.rep[b].n_pruned, sg.n - q_kept);
    if (nA <= 0 || nB <= 0) {
        if (STAT && (threadIdx.x & 63) == 0)
            ga.stat[((size_t)b * ga.stat_wgs + wg) * 8 + (threadIdx.x >> 6)] = 0u;
        return;
    }
    const int tilesR = (nA + TILE_R - 1) / TILE_R;
    const int tilesC = (nB + TILE_C - 1) / TILE_C;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
    const int wr = wave >> 2, wc = wave & 3;                      // 2 x 4 wavefronts of WROWS x 64

    lds_char* ring = (lds_char*)s_ring;
    const uint32_t ring_base = (uint32_t)(uintptr_t)ring;
    float* sRinv = (float*)((char*)s_ring + NSTAGE * STAGE_BYTES);   // [TILE_R]
    lds_f64* sRho = (lds_f64*)(ring + NSTAGE * STAGE_BYTES + TILE_R * sizeof(float));   // [4][64]

    // A row is dk bf16 values; fp32 keys arrive as three such planes per token (hi, mid, lo:
    // x = hi + mid + lo to 24 bits), each padded to whole 16-byte chunks.  Their product is then
    // six passes over the key width, u.v = sum over the plane pairs below of plane_a(u).plane_b(v)
    // (what is left out - mid.lo, lo.mid, lo.lo - is below 2^-23 |u||v|), smallest terms first:
    // every fp32 rounding of the accumulator is relative to its size at that moment, so the
    // five passes of small terms cost next to nothing in accuracy and the hi.hi pass at the end
    // the same as a plain bf16 product.
    constexpr bool SPLIT = DT == PACT_F32X3;
    constexpr bool SHARE_RING = SPLIT && NSTAGE == 2;   // see the order of the slices below
    const int row_bytes = SPLIT ? ((ga.dk + 7) & ~7) * 2 : ga.dk * Elem<PACT_BF16>::BYTES;   // of one plane
    const int tok_bytes = SPLIT ? 3 * row_bytes : row_bytes;
    const int spp = (row_bytes + SLICE_BYTES - 1) / SLICE_BYTES;                             // slices per plane
    const int nSlices = SPLIT ? 6 * spp : spp;
    const char* __restrict__ keys = ga.keys + (size_t)sg.base * tok_bytes;
    const int32_t* __restrict__ idxR = ga.idx_rows + sg.base;
    const int32_t* __restrict__ idxC = ga.idx_cols + sg.base;
    const float* __restrict__ rinv = ga.rinv + sg.base;
    uint64_t* adj = ga.adj + (size_t)b * bt.n_max * bt.W;

    // density constants: arg = cos * a - a = -(d / d_n) * log2(e); each of the two reciprocal norms
    // carries sqrt(a), so that the factor of a pair is the same product whichever token is the
    // row (pair (i, j) and pair (j, i) then get the same fp32 value, bit for bit)
    const float a_ = 1.4426950408889634f / sg.d_n;
    const float sa_ = (MODE == MODE_DENSITY) ? sqrtf(a_) : 1.0f;
    const float thr_cos = (MODE == MODE_DENSITY) ? (1.0f - sg.d_c) : (1.0f - sg.alpha * sg.d_c);
    const float t_lo = (MODE == MODE_DENSITY) ? -(sg.d_c + ga.margin) * a_ : thr_cos - ga.margin;
    const float t_hi = -(sg.d_c - ga.margin) * a_;

    // DMA roles: a stage is (TILE_R + 256) / 8 blocks of 1 KB (8 rows x 8 chunks), the A rows
    // first; wavefront w brings blocks w*NB .. w*NB+NB-1.  Lane l of a block: row 8*blk + l/8,
    // physical chunk l&7, which holds logical chunk (l&7) ^ ((row >> 1) & 7).
    const uint32_t dma_lds0 = ring_base + (uint32_t)(wave * NB * 1024);

    // Tile order.  Workgroups are dealt to the 8 XCDs round-robin (XCD = workgroup id mod 8) and
    // every XCD has its own 4 MB L2.  Full matrix: each XCD takes a patch of the tile grid, half
    // of the tile rows by a quarter of the tile columns, so that the keys it touches (a row and a
    // column operand of the patch: 3 MB for 4000 kept tokens of 1 KB) stay in its L2; walking whole
    // tile columns instead made every XCD touch all rows (4.6 MB; the density pass of one image
    // 1.2 us longer).  Triangle (below): a contiguous eighth of the tile sequence per XCD.
    // Symmetry (density pass, square tiles): d_ij = d_ji, so the tiles above the diagonal can
    // stand for their mirror images as well (their epilogue then also leaves row sums and the
    // transposed bits).  That epilogue is longer, and with a tile or less per workgroup the
    // kernel lasts as long as its slowest tile whatever their number: mirrored tiles are used
    // when they save at least one turn in eight of the workgroups' tile loop.
    const int xcd = wg & 7;
    const long nFull = (long)tilesR * tilesC;
    const long nTri = (long)tilesR * (tilesR + 1) / 2;
    bool sym = false;
    if constexpr (SYM) sym = mirrored_tiles_pay(tilesR, G);
    const long nTiles = sym ? nTri : nFull;
    const bool banded = !ga.mapped && nTiles >= 8 && (G & 7) == 0;        // (a sample kept on one XCD: one band)
    const bool patch = banded && !sym && (tilesR & 1) == 0 && (tilesC & 3) == 0;   // (patches of equal size only)
    const int pr0 = (xcd >> 2) * tilesR / 2, pnr = ((xcd >> 2) + 1) * tilesR / 2 - pr0;   // the XCD's patch
    const int pc0 = (xcd & 3) * tilesC / 4, pnc = ((xcd & 3) + 1) * tilesC / 4 - pc0;
    const int l_lo = patch ? 0 : banded ? (int)(xcd * nTiles / 8) : 0;
    const int l_hi = patch ? pnr * pnc : banded ? (int)((xcd + 1) * nTiles / 8) : (int)nTiles;
    const int t_first = l_lo + (banded ? (wg >> 3) : wg);
    const int t_step = banded ? (G >> 3) : G;

    float far = 0.0f;              // most negative density exponent seen = largest distance (density pass)
    for (int tl = t_first; tl < l_hi; tl += t_step) {
        // Per-lane constants of a tile.  (The build with mirrored tiles has no register to spare
        // in its epilogue: there they are derived anew for every tile from a laundered thread
        // number, so that they do not occupy registers from one tile to the next.)
        int tid_t = tid;
        if constexpr (SYM) asm volatile("" : "+v"(tid_t));
        const int lane = tid_t & 63;
        const int l32_ = lane & 31, hh_ = lane >> 5;
        const int dma_row0 = wave * NB * 8 + (lane >> 3);          // DMA: stage row of this lane in block k: + 8 * k
        // fragment addressing: lane (l32, hh) reads chunk 2g+hh of row (its wave's row block) + l32
        const int swz = (l32_ >> 1) & 7;
        const uint32_t fragA0 = (uint32_t)((wr * WROWS + l32_) * SLICE_BYTES);
        const uint32_t fragB0 = (uint32_t)((TILE_R + wc * 64 + l32_) * SLICE_BYTES);

        int tr = tl % tilesR, tc = tl / tilesR;
        if (patch) {
            tr = pr0 + tl % pnr;
            tc = pc0 + tl / pnr;
        }
        if (sym) {
            // the tiles above the diagonal, column by column: tile tl is (tr, tc) with tr < tc,
            // tl = tc (tc - 1) / 2 + tr; then the tiles on the diagonal, whose epilogue is the
            // shorter one (the last turn of a workgroup's tile loop is then a short one)
            const int nOff = tilesR * (tilesR - 1) / 2;
            if (tl < nOff) {
                tc = (int)((sqrtf(8.0f * (float)tl + 1.0f) + 1.0f) * 0.5f);
                while ((tc + 1) * tc / 2 <= tl) ++tc;
                while (tc * (tc - 1) / 2 > tl) --tc;
                tr = tl - tc * (tc - 1) / 2;
            } else {
                tr = tc = tl - nOff;
            }
        }
        const int rowBase = tr * TILE_R;
        const int colBase = tc * TILE_C;
        const bool mirror = SYM && sym && tr != tc;  // this tile also stands for tile (tc, tr)

        // byte offsets of this lane's 16 bytes in the first slice of its NB DMA rows; rows past the
        // end are clamped to the last one (their products are discarded in the epilogue)
        uint32_t ro[NB];
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int r = dma_row0 + 8 * k;
            const int tok = (r >= TILE_R) ? idxC[min(colBase + r - TILE_R, nB - 1)] : idxR[min(rowBase + r, nA - 1)];
            // (with the lane's chunk: the swizzle term depends on the row only through
            //  (row >> 1) & 7, and rows advance by 8 per block)
            ro[k] = (uint32_t)tok * (uint32_t)tok_bytes + (uint32_t)(((lane & 7) ^ ((r >> 1) & 7)) * 16);
        }
        if (tid_t < TILE_R) sRinv[tid_t] = rinv[idxR[min(rowBase + tid_t, nA - 1)]] * sa_;
        float rj_pre[2];                                    // 1/|u_j| of this lane's two columns (used in the epilogue)
#pragma unroll
        for (int j = 0; j < 2; ++j) rj_pre[j] = rinv[idxC[min(colBase + wc * 64 + j * 32 + l32_, nB - 1)]];

        // Order of the slices.  bf16 keys: along the key width.  fp32 keys (three planes): the five
        // pairs of small terms first, then (hi,hi) along the key width (see above).  With two ring
        // stages (256 x 256 tiles, where a wavefront fetches rows of one operand only) the small
        // pairs of one slice of the key width follow each other so that each step changes one
        // operand only - (hi,lo) (hi,mid) (mid,mid) (mid,hi) (lo,hi) - and the other half of the
        // stage is reused instead of fetched again: the two halves of the ring then alternate
        // independently (eight instead of twelve plane slices per slice of the key width).
        constexpr bool SHARE = SHARE_RING;
        static_assert(!SHARE || NB * 8 * 4 == TILE_R, "four wavefronts fetch the row operand, four the column operand");
        int next_pass = 0, next_ks = 0;          // of the next slice to fetch (slices are fetched in order)
        int slotA = 1, slotB = 1;                // SHARE: ring slot that holds the newest row / column operand
        auto issue = [&](int s) __attribute__((always_inline)) {      // slice s -> ring slot s % NSTAGE
            const int pass = SPLIT ? next_pass : 0;   // SHARE: position in the group of five small pairs, 5 = (hi,hi)
            const int ks = SPLIT ? next_ks : s;
            uint32_t planeA, planeB;
            bool fetchA = true, fetchB = true;
            if constexpr (SHARE) {
                planeA = (0x250u >> (2 * pass)) & 3;  planeB = (0x016u >> (2 * pass)) & 3;
                fetchA = (0x35u >> pass) & 1;         fetchB = (0x2Bu >> pass) & 1;
                if (pass == 5) { ++next_ks; }
                else if (++next_pass == 5) { next_pass = 0; if (++next_ks == spp) { next_ks = 0; next_pass = 5; } }
                slotA ^= fetchA ? 1 : 0;
                slotB ^= fetchB ? 1 : 0;
            } else {
                // (hi,lo) (lo,hi) (mid,mid) (hi,mid) (mid,hi) (hi,hi), two bits per pass
                planeA = (0x118u >> (2 * pass)) & 3;  planeB = (0x052u >> (2 * pass)) & 3;
                if (SPLIT && ++next_ks == spp) { next_ks = 0; ++next_pass; }
            }
            const uint32_t offA = (uint32_t)(ks * SLICE_BYTES) + (SPLIT ? planeA * (uint32_t)row_bytes : 0u);
            const uint32_t offB = (uint32_t)(ks * SLICE_BYTES) + (SPLIT ? planeB * (uint32_t)row_bytes : 0u);
            const uint32_t ldsA = dma_lds0 + (uint32_t)((SHARE ? slotA : s % NSTAGE) * STAGE_BYTES);
            const uint32_t ldsB = dma_lds0 + (uint32_t)((SHARE ? slotB : s % NSTAGE) * STAGE_BYTES);
            if ((ks + 1) * SLICE_BYTES <= row_bytes) {
                // a whole slice: scalar base + (row offset + chunk) + slice offset, one add per block.
                // (These instructions sit between the barrier and the first MFMA of every
                //  wavefront, i.e. the matrix cores idle meanwhile: they are kept few.)
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    const bool colRows = wave * NB * 8 + 8 * k >= TILE_R;          // (wave-uniform)
                    if (colRows ? fetchB : fetchA)
                        dma16_off(keys, ro[k] + (colRows ? offB : offA), (colRows ? ldsB : ldsA) + k * 1024);
                }
            } else {
#pragma unroll
                for (int k = 0; k < NB; ++k) {
                    const bool colRows = wave * NB * 8 + 8 * k >= TILE_R;
                    const int chunk = (lane & 7) ^ (((dma_row0 + 8 * k) >> 1) & 7);
                    const bool ok = ks * SLICE_BYTES + chunk * 16 < row_bytes;     // past the key width: zeros
                    const char* src = ok ? keys + (ro[k] + (colRows ? offB : offA)) : ga.zeros;
                    if (colRows ? fetchB : fetchA) dma16(src, (colRows ? ldsB : ldsA) + k * 1024);
                }
            }
        };
        f32x16_t acc[MI][2];
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

#pragma unroll
        for (int s = 0; s < AHEAD; ++s)
            if (s < nSlices) issue(s);

        for (int s = 0; s < nSlices; ++s) {
            // slice s has landed once at most the younger slices' loads are outstanding
            if (s + AHEAD - 1 < nSlices) wait_vmcnt<NB * (AHEAD - 1)>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();      // ... for every wavefront; and slot (s-1)%NSTAGE is free

            // the fragments of k-group g+1 are read from LDS while the MFMAs of group g run
            // (slotA / slotB still name the slots of this slice: the next fetch comes further down)
            const lds_char* stA = ring + (SHARE ? slotA : s % NSTAGE) * STAGE_BYTES;
            const lds_char* stB = ring + (SHARE ? slotB : s % NSTAGE) * STAGE_BYTES;
            u32x4_t fa[2][MI], fb[2][2];
            auto load_frags = [&](int g, int buf) __attribute__((always_inline)) {
                const uint32_t co = (uint32_t)(((2 * g + hh_) ^ swz) << 4);
#pragma unroll
                for (int i = 0; i < MI; ++i) fa[buf][i] = *(const lds_u32x4*)(stA + fragA0 + i * 32 * SLICE_BYTES + co);
#pragma unroll
                for (int j = 0; j < 2; ++j) fb[buf][j] = *(const lds_u32x4*)(stB + fragB0 + j * 32 * SLICE_BYTES + co);
            };
            constexpr int MF = 1;                               // MFMA instructions per fragment pair
            load_frags(0, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, MI + 2, 0);
            // (the next fetches are issued while the first fragments are on their way from the LDS:
            //  nothing else can fill the time between the barrier and the first MFMA)
            if (s + AHEAD < nSlices) issue(s + AHEAD);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (g + 1 < 4) load_frags(g + 1, (g + 1) & 1);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) Mfma<DT>::run(fa[g & 1][i], fb[g & 1][j], acc[i][j]);
                // issue order: the LDS reads of the next k-group go out one by one between the
                // first MFMAs of this one (the scheduler would otherwise serialise read -> wait ->
                // multiply on one set of fragment registers)
                if (g + 1 < 4) {
#pragma unroll
                    for (int k = 0; k < MI + 2; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, MF, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x008, MF * (2 * MI - (MI + 2)), 0);
                } else {
                    __builtin_amdgcn_sched_group_barrier(0x008, MF * 2 * MI, 0);
                }
            }
        }
        // LDS the epilogue may use for its buffers: the ring stage that the last slice did not
        // occupy; where the two halves of the ring alternate independently the last slice may
        // occupy halves of both, so there every wavefront finishes its reads first.
        const int freeStage = SHARE_RING ? 0 : (nSlices % NSTAGE);
        if constexpr (SHARE_RING) __builtin_amdgcn_s_barrier();

        // ------------------------------------------------------------------ epilogue
        // acc[i][j][r] holds row  rowBase + wr*WROWS + i*32 + 8*(r/4) + 4*hh + (r%4)
        //              and column colBase + wc*64 + j*32 + l32.
        // (lane coordinates are laundered through an empty asm so that the per-element index
        //  arithmetic below is not hoisted out of the tile loop into long-lived registers)
        int l32 = l32_, hh = hh_;
        asm volatile("" : "+v"(l32), "+v"(hh));
        const int colW = colBase + wc * 64;                 // first column of this wave, multiple of 64
        const int wordIdx = colW >> 6;
        const int rowW = rowBase + wr * WROWS;
        float rj[2];
        int colP[2];
        uint64_t laneOk[2];                                 // lanes whose column exists
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            colP[j] = colW + j * 32 + l32;
            rj[j] = rj_pre[j] * sa_;
            laneOk[j] = __ballot(colP[j] < nB);
        }
        double rho[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
        // per-wavefront buffer of undecided pairs, in a ring slot no wavefront reads any more
        lds_uint2* nearBuf = (lds_uint2*)(ring + freeStage * STAGE_BYTES + wave * (NEAR_BUF * 8));
        int nearN = 0;
        // mirrored tiles: the wavefronts' row sums (128 rows x 64 columns each), behind the pair buffers
        lds_f64* rowBuf = (lds_f64*)(ring + freeStage * STAGE_BYTES + 8 * (NEAR_BUF * 8));
        auto flush_near = [&]() __attribute__((always_inline)) {
            int base_slot = 0;
            // (one 64-bit atomic: slots in the low word, ordered pairs in the high word)
            if (lane == 0)
                base_slot = (int)(uint32_t)atomicAdd((unsigned long long*)&ga.near_cnt[2 * b],
                                                     (unsigned long long)nearN | ((unsigned long long)(mirror ? 2 * nearN : nearN) << 32));
            base_slot = __shfl(base_slot, 0, 64);
            for (int k = lane; k < nearN; k += 64) {
                const int slot = base_slot + k;
                if (slot < NEAR_CAP) {
                    const u32x2_t e = nearBuf[k];
                    *(u32x2_t*)(ga.near_list + ((size_t)b * NEAR_CAP + slot) * 2) = e;
                }
            }
            nearN = 0;
        };
        // (the barriers of the slice loop also ordered the sRinv writes before these reads)
        if constexpr (MODE == MODE_CAND) {
            // A lane holds 2 x 16 of the 64 centres of a group for each of its two pruned tokens,
            // the lane 32 further on the other 2 x 16: maximum and bits are assembled in the lane
            // and completed with one exchange.  A bit is set for a centre within reach whose
            // cosine is at most 2 * margin below the group's largest: no other centre of the
            // group can be the nearest in exact arithmetic.  Layout [group][pruned token], so that
            // the 32 lanes of a half-wave store contiguously.
            uint64_t* cw = adj + (size_t)q_kept * bt.W;                   // [Wc][nB] words, in the unused bitmap rows
            float* cb = ga.cbest + (size_t)b * bt.W * bt.n_max;
            const float two_m = 2.0f * ga.margin;
#pragma unroll
            for (int gi = 0; gi < MI / 2; ++gi) {
                const int rowG = rowW + gi * 64;                           // first centre of the group
                if (rowG >= nA) continue;
                float rs[2][16];
#pragma unroll
                for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        rs[i2][r] = sRinv[wr * WROWS + gi * 64 + i2 * 32 + 8 * (r >> 2) + 4 * hh + (r & 3)];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    float lb = -INFINITY;
#pragma unroll
                    for (int i2 = 0; i2 < 2; ++i2)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const bool pad = rowG + i2 * 32 + 8 * (r >> 2) + 4 * hh + (r & 3) >= nA;
                            const float v = pad ? -INFINITY : acc[2 * gi + i2][j][r] * rs[i2][r] * rj[j];
                            acc[2 * gi + i2][j][r] = v;
                            lb = fmaxf(lb, v);
                        }
                    lb = fmaxf(lb, __shfl_xor(lb, 32, 64));
                    const float cut = fmaxf(lb - two_m, t_lo);
                    uint32_t w32[2];
#pragma unroll
                    for (int i2 = 0; i2 < 2; ++i2) {
                        uint32_t bits = 0u;
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            bits |= (acc[2 * gi + i2][j][r] >= cut) ? (1u << (8 * (r >> 2) + (r & 3))) : 0u;
                        bits <<= 4 * hh;
                        w32[i2] = bits | (uint32_t)__shfl_xor((int)bits, 32, 64);
                    }
                    if (hh == j && colP[j] < nB) {
                        cb[(size_t)(rowG >> 6) * bt.n_max + colP[j]] = lb;
                        if (lb >= t_lo) cw[(size_t)(rowG >> 6) * nB + colP[j]] = ((uint64_t)w32[1] << 32) | w32[0];
                    }
                }
            }
        } else {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            float rs[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) rs[r] = sRinv[wr * WROWS + i * 32 + 8 * (r >> 2) + 4 * hh + (r & 3)];
            const int rowI = rowW + i * 32;                 // first row of this 32-row block
            // phase A1: cosines (scaled for the density exponent), left in place of the accumulators
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const bool pad = rowI + 8 * (r >> 2) + 4 * hh + (r & 3) >= nA;   // padded row: no term, no bit
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const float v = fmaf(acc[i][j][r], rs[r] * rj[j], -a_);
                    acc[i][j][r] = pad ? -INFINITY : v;
                }
            }
            if (MODE == MODE_DENSITY) {
                // d_ii = 0 exactly: only the blocks on the diagonal hold such elements
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    if (rowI == colW + j * 32) {
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (8 * (r >> 2) + 4 * hh + (r & 3) == l32 && rowI + l32 < nA) acc[i][j][r] = 0.0f;
                    }
                // phase A2: density terms
                if (mirror) {
                    // ... which also belong to the densities of this tile's rows: sum them over
                    // the wavefront's 64 columns.  Each lane has 4 rows x 2 columns at a time; the 32
                    // lanes of a half-wave halve their row sets twice (a lane sends the sums of the
                    // rows it gives up and adds what it receives for those it keeps) and are left
                    // with one row each, eight neighbouring lanes with parts of the same one.
                    const bool ok0 = colP[0] < nB, ok1 = colP[1] < nB;      // clamped columns count nowhere
                    static_for<4>([&](auto r4_tag) __attribute__((always_inline)) {   // four rows at a time: registers are tight
                        constexpr int r4 = 4 * decltype(r4_tag)::value;
                        double d[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const double e0 = (double)__builtin_amdgcn_exp2f(acc[i][0][r4 + r]);
                            const double e1 = (double)__builtin_amdgcn_exp2f(acc[i][1][r4 + r]);
                            rho[0][r & 1] += e0;
                            rho[1][r & 1] += e1;
                            d[r] = (ok0 ? e0 : 0.0) + (ok1 ? e1 : 0.0);
                        }
                        {
                            const bool up = (l32 & 16) != 0;
#pragma unroll
                            for (int k = 0; k < 2; ++k) {
                                const double keep = up ? d[k + 2] : d[k];
                                const double send = up ? d[k] : d[k + 2];
                                d[k] = keep + swizzle_xor<16>(send);
                            }
                        }
                        {
                            const bool up = (l32 & 8) != 0;
                            const double keep = up ? d[1] : d[0];
                            const double send = up ? d[0] : d[1];
                            d[0] = keep + swizzle_xor<8>(send);
                        }
                        d[0] += swizzle_xor<4>(d[0]);
                        d[0] += swizzle_xor<2>(d[0]);
                        d[0] += swizzle_xor<1>(d[0]);
                        // rows r4 .. r4+3 of this lane are rows 2 r4 + 4 hh + (0..3) of the block
                        if ((l32 & 7) == 0) rowBuf[wave * 128 + i * 32 + 2 * r4 + 4 * hh + (l32 >> 3)] = d[0];
                        if (r4 == 4) __builtin_amdgcn_sched_barrier(0);     // two groups at a time may overlap their exchanges
                    });
                } else {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
#pragma unroll
                    for (int j = 0; j < 2; ++j) rho[j][r & 1] += (double)__builtin_amdgcn_exp2f(acc[i][j][r]);
                    if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // bound the live ranges: registers are tight
                }
                }
            }
            // phase B: one bit per pair; most 32 x 64 blocks have none set: test the block's maximum first
            float mx = fmaxf(acc[i][0][0], acc[i][1][0]);
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(acc[i][0][r], acc[i][1][r]));
            if (STAT) {
                // the block's smallest exponent (largest distance); padded rows hold -inf and are
                // left out (padded columns repeat a real column: harmless)
                if (rowI + 32 <= nA) {
                    float mn = fminf(acc[i][0][0], acc[i][1][0]);
#pragma unroll
                    for (int r = 1; r < 16; ++r) mn = fminf(mn, fminf(acc[i][0][r], acc[i][1][r]));
                    far = fminf(far, mn);
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const bool pad = rowI + 8 * (r >> 2) + 4 * hh + (r & 3) >= nA;
                        far = fminf(far, pad ? 0.0f : fminf(acc[i][0][r], acc[i][1][r]));
                    }
                }
            }
            if (__ballot(mx >= t_lo) == 0) continue;
            // Ballots put the 64 columns of two rows (hh = 0 / 1) into a scalar pair; v_writelane
            // files each half under the lane of its row, so that lane k < 32 ends up holding the
            // 64-bit bitmap word of row rowI + k.  (Scalar instructions are the scarce resource
            // here: the CU's four SIMDs share one scalar unit.)
            // The same is done with the ballots against the upper edge of the undecided band, so
            // that the band itself (pairs too close to d_c for fp32) falls out per row afterwards.
            // Straight-line code per element is kept to compares and lane writes: this part is
            // unrolled 16 * MI times, and blocks that reach it are the minority, so its
            // instructions are rarely in the instruction cache when they are needed.
            uint32_t wlo = 0, whi = 0, hlo = 0, hhi = 0;
            static_for<16>([&](auto r_tag) __attribute__((always_inline)) {
                constexpr int r = decltype(r_tag)::value;
                constexpr int k0 = 8 * (r >> 2) + (r & 3);            // row of the lanes with hh = 0; hh = 1: k0 + 4
                const uint64_t m0 = __ballot(acc[i][0][r] >= t_lo);
                const uint64_t m1 = __ballot(acc[i][1][r] >= t_lo);
                if (MODE == MODE_DENSITY) {
                    const uint64_t h0 = __ballot(acc[i][0][r] >= t_hi);
                    const uint64_t h1 = __ballot(acc[i][1][r] >= t_hi);
                    file_ballots2<k0>(wlo, whi, hlo, hhi, m0, m1, h0, h1);
                } else {
                    file_ballots<k0>(wlo, whi, m0, m1);
                }
            });
            // the 32 words of this block, one store instruction (the bitmap was cleared beforehand;
            // columns past the last one come from a clamped row: mask them)
            wlo &= (uint32_t)laneOk[0];
            whi &= (uint32_t)laneOk[1];
            if (lane < 32 && (wlo | whi) != 0)
                adj[(size_t)(rowI + lane) * bt.W + wordIdx] = ((uint64_t)whi << 32) | wlo;
            if (MODE == MODE_DENSITY && mirror) {
                // the same bits for the mirror image: 32 rows of this block are 32 columns (half a
                // bitmap word) of the rows that are this tile's columns; assembled in the lane
                // from its 16 rows and completed by the lane 32 further on
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    uint32_t bits = 0u;
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        bits |= (acc[i][j][r] >= t_lo) ? (1u << (8 * (r >> 2) + (r & 3))) : 0u;
                    bits <<= 4 * hh;
                    bits |= (uint32_t)__shfl_xor((int)bits, 32, 64);
                    if (hh == j && colP[j] < nB && bits != 0u)
                        ((uint32_t*)adj)[((size_t)colP[j] * bt.W + (rowI >> 6)) * 2 + ((rowI >> 5) & 1)] = bits;
                }
            }
            if (MODE == MODE_DENSITY) {
                // Undecided pairs: queue them for the fp64 check.  They collect in this wavefront's
                // LDS buffer, every lane adding one pair of its row per turn; one atomic reserves
                // list slots for a whole buffer (an atomic per pair would cost a memory round trip).
                uint64_t band = ((uint64_t)(whi & ~hhi) << 32) | (wlo & ~hlo);   // zero in lanes 32..63
                uint64_t has;
                while ((has = __ballot(band != 0)) != 0) {
                    if (band != 0) {
                        const int c = __builtin_ctzll(band);
                        band &= band - 1;
                        nearBuf[nearN + __popcll(has & ((1ull << lane) - 1ull))] =
                            u32x2_t{(uint32_t)(rowI + lane) | (mirror ? NEAR_MIRROR : 0u), (uint32_t)(colW + c)};
                    }
                    nearN += __popcll(has);
                    if (nearN > NEAR_BUF - 32) flush_near();
                }
            }
        }
        }
        if (MODE == MODE_DENSITY && nearN > 0) flush_near();

        if (MODE == MODE_DENSITY) {
            // column sums over this wave's rows: combine the two half-waves; one row of partials
            // covers GRAM_RHO_ROWS = 128 kept rows, i.e. one wavefront row (MI = 4) or both (MI = 2)
            static_assert(GRAM_RHO_ROWS == 128, "the density partials are per 128 kept rows");
            double tot[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const double part = rho[j][0] + rho[j][1];
                tot[j] = part + __shfl_xor(part, 32, 64);
            }
            if (MI == 2) {
                if (wr == 1 && hh == 0) { sRho[wc * 64 + l32] = tot[0]; sRho[wc * 64 + 32 + l32] = tot[1]; }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                if (wr == 0 && hh == 0) { tot[0] += sRho[wc * 64 + l32]; tot[1] += sRho[wc * 64 + 32 + l32]; }
            }
            const int rt = (MI == 4) ? (rowBase / GRAM_RHO_ROWS) + wr : rowBase / GRAM_RHO_ROWS;
            double* out = ga.rho_part + ((size_t)b * bt.W + rt) * bt.n_max;
            const bool writer = hh == 0 && (MI == 4 ? rowW < nA : wr == 0);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                if (writer && colP[j] < nB) out[colP[j]] = tot[j];
        }
        if (MODE == MODE_DENSITY && mirror) {
            // row sums: two wavefronts side by side cover the 128 columns of one row of partials
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            const int half = tid_t >> 8, pair = (tid_t >> 7) & 1, row = tid_t & 127;
            const double v = rowBuf[(half * 4 + pair * 2) * 128 + row] + rowBuf[(half * 4 + pair * 2 + 1) * 128 + row];
            const int gRow = rowBase + half * 128 + row;
            if (gRow < nA && colBase + pair * 128 < nB)
                ga.rho_part[((size_t)b * bt.W + colBase / GRAM_RHO_ROWS + pair) * bt.n_max + gRow] = v;
        }
        if (tl + t_step < l_hi) {
            // the ring and sRinv are rewritten by the next tile: every wavefront must be done with
            // them (and the slice loop's vmcnt arithmetic assumes nothing older is outstanding)
            wait_vmcnt<0>();
            __syncthreads();
        }
    }
    if (STAT) {
        // one word per wavefront, no atomics (thousands of them on one address would take longer
        // than the kernel); the kernel that finishes the densities takes the minimum
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) far = fminf(far, __shfl_xor(far, sft, 64));
        if (lane == 0) ga.stat[((size_t)b * ga.stat_wgs + wg) * 8 + wave] = far < 0.0f ? __float_as_uint(far) : 0u;
    }
}

// One sample: a workgroup per tile, at most one per CU, a multiple of the 8 XCDs (see the tile order).
static int gram_grid_x(const Batch& bt, long tiles) {
    long grid_x = tiles;
    static_assert(GRAM_MAX_WORKGROUPS == 256, "one workgroup per CU, 256 CUs");
    if (grid_x > GRAM_MAX_WORKGROUPS) grid_x = GRAM_MAX_WORKGROUPS;
    if (grid_x >= 8) grid_x &= ~7L;
    return (int)grid_x;
}

// Batches: the chip's 256 workgroup slots are shared out among the samples by the number of
// tiles each is expected to have (tiles[b] >= 1): the fewest turns R of a workgroup's tile loop
// such that ceil(tiles[b] / R) workgroups per sample fit, spare slots to the samples with the
// most tiles per workgroup.  Each sample then gets slots of one XCD where it can (slot i belongs
// to XCD i mod 8), the largest samples first.  The counts are estimates (the real ones are on the
// device): a sample with more tiles than expected just takes more turns.
// Fills ga.wg_map / ga.wg_count, returns the largest count.
static int build_wg_map(int B, const long* tiles, GramArgs& ga) {
    constexpr int S = GRAM_MAX_WORKGROUPS;
    int g[PACT_MAX_BATCH], order[PACT_MAX_BATCH];
    long most_tiles = 1;
    for (int b = 0; b < B; ++b) most_tiles = tiles[b] > most_tiles ? tiles[b] : most_tiles;
    long R = 1;
    for (;; ++R) {                            // (R = most_tiles needs one workgroup per sample, B <= 64 < S)
        long need = 0;
        for (int b = 0; b < B; ++b) need += (tiles[b] + R - 1) / R;
        if (need <= S || R >= most_tiles) break;
    }
    int used = 0;
    for (int b = 0; b < B; ++b) { g[b] = (int)((tiles[b] + R - 1) / R); if (g[b] < 1) g[b] = 1; used += g[b]; }
    while (used < S) {
        int best = -1;
        for (int b = 0; b < B; ++b)
            if (g[b] < tiles[b] && (best < 0 || (double)tiles[b] / g[b] > (double)tiles[best] / g[best])) best = b;
        if (best < 0) break;
        ++g[best]; ++used;
    }
    for (int b = 0; b < B; ++b) order[b] = b;
    for (int i = 1; i < B; ++i)              // by workgroup count, largest first (insertion sort, B <= 64)
        for (int j = i; j > 0 && g[order[j]] > g[order[j - 1]]; --j) { const int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t; }
    int freeSlots[8];
    for (int x = 0; x < 8; ++x) freeSlots[x] = S / 8;
    for (int i = 0; i < S; ++i) ga.wg_map[i] = 0xFFFFu;
    int most = 0;
    for (int k = 0; k < B; ++k) {
        const int b = order[k];
        ga.wg_count[b] = (uint16_t)g[b];
        if (g[b] > most) most = g[b];
        int left = g[b], rank = 0;
        while (left > 0) {
            int x = 0;
            for (int y = 1; y < 8; ++y) if (freeSlots[y] > freeSlots[x]) x = y;
            const int take = left < freeSlots[x] ? left : freeSlots[x];
            for (int t = 0; t < take; ++t) {
                const int slot = (S / 8 - freeSlots[x]) + t;       // this XCD's next unused slot
                ga.wg_map[slot * 8 + x] = (uint16_t)((b << 8) | rank++);
            }
            freeSlots[x] -= take;
            left -= take;
        }
    }
    return most;
}

template <int MODE, int MI, bool STAT, bool SYM>
static int launch_gram_shape(const Batch& bt, const GramArgs& ga_in, pact_dtype k_dt, hipStream_t st,
                             const char* name, int* grid_out) {
    typedef Shape<MI> SH;
    const int tilesR = (bt.n_max + SH::TILE_R - 1) / SH::TILE_R, tilesC = (bt.n_max + TILE_C - 1) / TILE_C;
    GramArgs ga = ga_in;
    int grid_x = gram_grid_x(bt, (long)tilesR * tilesC);
    dim3 grid(grid_x, 1);
    ga.mapped = bt.B > 1;
    if (ga.mapped) {
        // tiles a sample is expected to have: kept tokens n - floor(lambda n); density pass
        // kept x kept (square tiles: the triangle); candidate pass about kept / 2 centres x pruned
        long tiles[PACT_MAX_BATCH];
        for (int b = 0; b < bt.B; ++b) {
            const long n = bt.s[b].n, q = n - (long)floorf(bt.s[b].lambda * (float)n);
            const long rows = (MODE == MODE_DENSITY) ? q : (q + 1) / 2, cols = (MODE == MODE_DENSITY) ? q : n - q;
            const long tr = (rows + SH::TILE_R - 1) / SH::TILE_R, tc = (cols + TILE_C - 1) / TILE_C;
            tiles[b] = (MODE == MODE_DENSITY && SYM) ? tr * (tr + 1) / 2 : tr * tc;
            if (tiles[b] < 1) tiles[b] = 1;
        }
        grid_x = build_wg_map(bt.B, tiles, ga);                // (from here on: the largest count of a sample)
        grid = dim3(GRAM_MAX_WORKGROUPS, 1);
    }
    ga.stat_wgs = grid_x;
    if (grid_out) *grid_out = grid_x;
    const size_t lds = SH::LDS_BYTES;
    static bool raised[2] = {false, false};
    const int di = k_dt == PACT_BF16 ? 1 : 0;
    const void* fn = (k_dt == PACT_BF16) ? (const void*)gram_kernel<PACT_BF16, MODE, MI, STAT, SYM>
                                         : (const void*)gram_kernel<PACT_F32X3, MODE, MI, STAT, SYM>;
    if (!raised[di]) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return PACT_ERR_HIP;
        raised[di] = true;
    }
    if (k_dt == PACT_BF16)
        PACT_LAUNCH_SHMEM(name, (gram_kernel<PACT_BF16, MODE, MI, STAT, SYM>), grid, dim3(512), lds, st, bt, ga);
    else
        PACT_LAUNCH_SHMEM(name, (gram_kernel<PACT_F32X3, MODE, MI, STAT, SYM>), grid, dim3(512), lds, st, bt, ga);
    return PACT_OK;
}

// 256 x 256 tiles when there are enough of them to occupy the chip, else 128 x 256.
// mirrored: the kernel build that can let the tiles above the diagonal stand for those below
// (it decides per sample, from the count of kept tokens it finds, whether to do so).
template <int MODE>
static int launch_gram(const Batch& bt, const GramArgs& ga, pact_dtype k_dt, hipStream_t st,
                       const char* name, long tiles256, bool mirrored, int* grid_out) {
    if (!ga.keys || !ga.idx_rows || !ga.idx_cols || !ga.rep || !ga.rinv || !ga.zeros || !ga.adj || ga.dk < 1)
        return PACT_ERR_NULL;                     // (an argument block that was not filled in completely)
    // the kernel addresses a sample's key rows with 32-bit byte offsets
    const uint64_t tok_bytes = (k_dt == PACT_F32) ? 3ull * (((uint64_t)ga.dk + 7) & ~7ull) * 2 : (uint64_t)ga.dk * 2;
    if ((uint64_t)bt.n_max * tok_bytes > 0xFFFFFFFFull) return PACT_ERR_SHAPE;
    const bool big = tiles256 * bt.B >= 256;
    if constexpr (MODE == MODE_DENSITY) {
        if (ga.stat) {                            // with the key-distance statistic
            if (big && mirrored) return launch_gram_shape<MODE, 4, true, true>(bt, ga, k_dt, st, name, grid_out);
            if (big) return launch_gram_shape<MODE, 4, true, false>(bt, ga, k_dt, st, name, grid_out);
            return launch_gram_shape<MODE, 2, true, false>(bt, ga, k_dt, st, name, grid_out);
        }
        if (big && mirrored) return launch_gram_shape<MODE, 4, false, true>(bt, ga, k_dt, st, name, grid_out);
    }
    if (big) return launch_gram_shape<MODE, 4, false, false>(bt, ga, k_dt, st, name, grid_out);
    return launch_gram_shape<MODE, 2, false, false>(bt, ga, k_dt, st, name, grid_out);
}

int launch_gram_density(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                        const int32_t* idx, pact_report* rep, bool want_stat, int* stat_words, hipStream_t st) {
    GramArgs ga = {};
    // (fp32 keys: their three bf16 planes)
    ga.keys = (k_dt == PACT_F32) ? (const char*)w.ksplit : (const char*)keys;
    ga.dk = dk; ga.idx_rows = idx; ga.idx_cols = idx; ga.rep = rep;
    ga.rinv = w.rinv; ga.zeros = (const char*)w.zeros; ga.adj = w.adj; ga.cbest = nullptr; ga.rho_part = w.rho_part;
    ga.near_list = w.near_list; ga.near_cnt = w.near_cnt; ga.stat = want_stat ? w.stat : nullptr; ga.margin = (float)cos_margin(dk);
    const long t1 = (bt.n_max + 255) / 256;
    // The count of kept tokens is known on the device only; what the percentile will leave
    // (n - floor(lambda n), more on ties) tells whether mirrored tiles are likely to pay for
    // some sample.  The kernel decides again from the real count, so a wrong guess costs time only.
    // (In a batch every sample has its own number of workgroups: the build that can mirror is
    //  used there whenever the tiles are square.)
    bool mirrored = bt.B > 1;
    const int gx = gram_grid_x(bt, t1 * t1);
    for (int b = 0; b < bt.B; ++b) {
        const int q_est = bt.s[b].n - (int)floorf(bt.s[b].lambda * (float)bt.s[b].n);
        mirrored = mirrored || mirrored_tiles_pay((q_est + 255) / 256, gx);
    }
    int grid_x = 0;
    const int rc = launch_gram<MODE_DENSITY>(bt, ga, k_dt, st, "gram_density", t1 * t1, mirrored, &grid_x);
    if (stat_words) *stat_words = want_stat ? grid_x * 8 : 0;
    return rc;
}

int launch_gram_candidates(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                           const int32_t* pruned_idx, const int32_t* center_idx, pact_report* rep,
                           hipStream_t st) {
    GramArgs ga = {};
    ga.keys = (k_dt == PACT_F32) ? (const char*)w.ksplit : (const char*)keys;
    ga.dk = dk; ga.idx_rows = center_idx; ga.idx_cols = pruned_idx;
    ga.rep = rep; ga.rinv = w.rinv; ga.zeros = (const char*)w.zeros; ga.adj = w.adj; ga.cbest = w.cbest;
    ga.rho_part = nullptr;
    ga.near_list = nullptr; ga.near_cnt = nullptr; ga.stat = nullptr; ga.margin = (float)cos_margin(dk);
    // rows: the centres, columns: the pruned tokens; neither count is known on the host, a
    // typical split (half pruned, a third of the rest centres) sizes the choice
    const long tr = (bt.n_max / 6 + 255) / 256, tc = (bt.n_max / 2 + 255) / 256;
    return launch_gram<MODE_CAND>(bt, ga, k_dt, st, "gram_candidates", tr * tc, false, nullptr);
}

int plan_gram_workgroups(const int32_t* tiles, int32_t batch, uint16_t* wg_map, uint16_t* wg_count) {
    if (!tiles || !wg_map || !wg_count) return PACT_ERR_NULL;
    if (batch < 1 || batch > PACT_MAX_BATCH) return PACT_ERR_SHAPE;
    GramArgs ga = {};
    long t[PACT_MAX_BATCH];
    for (int b = 0; b < batch; ++b) {
        if (tiles[b] < 1) return PACT_ERR_SHAPE;
        t[b] = tiles[b];
    }
    build_wg_map(batch, t, ga);
    for (int i = 0; i < GRAM_MAX_WORKGROUPS; ++i) wg_map[i] = ga.wg_map[i];
    for (int b = 0; b < batch; ++b) wg_count[b] = ga.wg_count[b];
    return PACT_OK;
}


}  // namespace pact

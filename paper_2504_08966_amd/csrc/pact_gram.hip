// The dense contraction of DBDPC (Alg. 2): Gram matrix of the clustering keys on the matrix
// cores, turned into cosines (Eq. 5) in the epilogue and consumed on the spot:
//   MODE_DENSITY  kept x kept  : density terms exp(-d/d_n) summed per column in fp64 (Eq. 6),
//                                one bit per pair "cosine distance <= d_c (+ margin)", and a
//                                list of the pairs too close to d_c for fp32 to decide;
//   MODE_CAND     pruned x centres : one bit per pair "distance < alpha*d_c (+ margin)"
//                                (candidates for Eq. 8).
// The distance matrix itself is never written.
//
// Shape of the kernel (gfx950):
//  * one workgroup of 8 wavefronts per CU owns a 256x256 output tile (L2 traffic per flop is
//    half that of 128x128 tiles, and the L2 -> CU path is what limits this contraction at a
//    key width of 512); each wavefront computes 128x64 of it as 4x2 v_mfma_f32_32x32x16_bf16
//    (or 32x32x2_f32) accumulators;
//  * the key rows stream in 64-byte slices straight from global memory into a ring of LDS
//    stages (global_load_lds_dwordx4: no staging registers), three slices ahead of the MFMAs;
//    waits on the ring are explicit (s_waitcnt vmcnt + s_barrier);
//  * both operands are rows of the same key matrix, so a lane takes 16 contiguous bytes of
//    "its" row per MFMA; the four 16-byte chunks of a row slice are XOR-swizzled by the row
//    number so that 16 consecutive rows read conflict-free;
//  * the grid is persistent (the tile count depends on counts only the device knows) and
//    XCD-aware: each of the 8 XCDs (own L2) works on its own band of tile columns.
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
    double* rho_part;          // [B][W][n_max], one row per GRAM_RHO_ROWS kept rows
    uint32_t* near_list;       // [B][NEAR_CAP][2]
    int32_t* near_cnt;         // [B]
    float margin;              // worst-case fp32 error of a cosine
};

constexpr int TILE = 256;
constexpr int SLICE_BYTES = 64;            // bytes of each row per stage: 4 chunks of 16 B
constexpr int NSTAGE = 4;                  // LDS ring: 3 slices in flight + 1 being multiplied
constexpr int AHEAD = NSTAGE - 1;
constexpr int STAGE_BYTES = 2 * TILE * SLICE_BYTES;   // A rows then B rows: 32 KB

typedef __attribute__((address_space(3))) char lds_char;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4_t lds_u32x4;
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) u32x2_t lds_uint2;
constexpr int NEAR_BUF = 512;              // undecided pairs a wavefront buffers before reserving list slots

// 16 bytes per lane, global -> LDS at (lds_base + lane * 16); asynchronous, counted by vmcnt.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :: "v"(gptr), "s"(lds_base) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int DT> struct Mfma;
template <> struct Mfma<PACT_BF16> {
    __device__ static __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                    __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<PACT_F32> {
    __device__ static __forceinline__ void run(const u32x4_t& a, const u32x4_t& b, f32x16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

template <int DT, int MODE>
__global__ __launch_bounds__(512, 2) void gram_kernel(Batch bt, GramArgs ga) {
    extern __shared__ uint4 s_ring[];                         // NSTAGE x 32 KB, then 256 floats
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int q_kept = clamp_count(ga.rep[b].n_kept, sg.n);
    const int nA = (MODE == MODE_DENSITY) ? q_kept : clamp_count(ga.rep[b].n_pruned, sg.n - q_kept);
    const int nB = (MODE == MODE_DENSITY) ? q_kept : clamp_count(ga.rep[b].n_centers, q_kept);
    const int row_off = (MODE == MODE_DENSITY) ? 0 : q_kept;   // candidate rows follow the kept rows
    if (nA <= 0 || nB <= 0) return;
    const int tilesR = (nA + TILE - 1) / TILE;
    const int tilesC = (nB + TILE - 1) / TILE;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
    const int wr = wave >> 2, wc = wave & 3;                      // 2 x 4 wavefronts of 128 x 64
    const int l32_ = lane & 31, hh_ = lane >> 5;

    lds_char* ring = (lds_char*)s_ring;
    const uint32_t ring_base = (uint32_t)(uintptr_t)ring;
    float* sRinv = (float*)((char*)s_ring + NSTAGE * STAGE_BYTES);   // [TILE]

    const int row_bytes = ga.dk * Elem<DT>::BYTES;
    const int nSlices = (row_bytes + SLICE_BYTES - 1) / SLICE_BYTES;
    const char* __restrict__ keys = ga.keys + (size_t)sg.base * row_bytes;
    const int32_t* __restrict__ idxR = ga.idx_rows + sg.base;
    const int32_t* __restrict__ idxC = ga.idx_cols + sg.base;
    const float* __restrict__ rinv = ga.rinv + sg.base;
    uint64_t* adj = ga.adj + (size_t)b * bt.n_max * bt.W;

    // density constants: arg = cos * a - a = -(d / d_n) * log2(e)
    const float a_ = 1.4426950408889634f / sg.d_n;
    const float thr_cos = (MODE == MODE_DENSITY) ? (1.0f - sg.d_c) : (1.0f - sg.alpha * sg.d_c);
    const float t_lo = (MODE == MODE_DENSITY) ? -(sg.d_c + ga.margin) * a_ : thr_cos - ga.margin;
    const float t_hi = -(sg.d_c - ga.margin) * a_;

    // DMA roles: a stage is 32 blocks of 1 KB (16 rows x 4 chunks); wavefronts 0-3 bring the
    // A rows, 4-7 the B rows, 4 blocks each.  Lane l of a block: row 16*blk + l/4, physical
    // chunk l&3, which holds logical chunk (l&3) ^ ((row >> 2) & 3).
    const int dma_is_b = wave >> 2;
    const int dma_row0 = (wave & 3) * 64 + (lane >> 2);       // + 16 * k, k = 0..3
    const int dma_chunk = (lane & 3) ^ ((lane >> 4) & 3);     // logical chunk this lane fetches
    const uint32_t dma_lds0 = ring_base + (uint32_t)(dma_is_b * TILE * SLICE_BYTES + (wave & 3) * 4096);

    // Tile order.  Workgroups are dealt to the 8 XCDs round-robin (XCD = workgroup id mod 8) and
    // every XCD has its own L2, so each XCD works on its own band of tile columns: its key rows
    // for those columns stay in its L2 while the row tiles stream through.
    const int xcd = blockIdx.x & 7;
    const bool banded = tilesC >= 8 && (gridDim.x & 7) == 0;
    const int c_lo = banded ? (int)((long)xcd * tilesC / 8) : 0;
    const int bw = banded ? (int)((long)(xcd + 1) * tilesC / 8) - c_lo : tilesC;
    const int myTiles = banded ? tilesR * bw : tilesR * tilesC;
    const int t_first = banded ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
    const int t_step = banded ? (int)(gridDim.x >> 3) : (int)gridDim.x;

    for (int tl = t_first; tl < myTiles; tl += t_step) {
        const int rowBase = (tl / bw) * TILE, colBase = (c_lo + tl % bw) * TILE;

        // byte offsets of this lane's 4 DMA rows; rows past the end are clamped to the last one
        // (their products are discarded in the epilogue)
        uint32_t ro[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int r = dma_row0 + 16 * k;
            const int tok = dma_is_b ? idxC[min(colBase + r, nB - 1)] : idxR[min(rowBase + r, nA - 1)];
            ro[k] = (uint32_t)tok * (uint32_t)row_bytes;
        }
        if (tid < TILE) sRinv[tid] = rinv[idxR[min(rowBase + tid, nA - 1)]];
        float rj_pre[2];                                    // 1/|u_j| of this lane's two columns (used in the epilogue)
#pragma unroll
        for (int j = 0; j < 2; ++j) rj_pre[j] = rinv[idxC[min(colBase + wc * 64 + j * 32 + l32_, nB - 1)]];

        auto issue = [&](int s) __attribute__((always_inline)) {      // slice s -> ring slot s % NSTAGE
            const int byte0 = s * SLICE_BYTES + dma_chunk * 16;
            const bool ok = byte0 < row_bytes;                         // past the key width: zeros
            const uint32_t slot = dma_lds0 + (uint32_t)((s % NSTAGE) * STAGE_BYTES);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const char* src = ok ? keys + (ro[k] + (uint32_t)byte0) : ga.zeros;
                dma16(src, slot + k * 1024);
            }
        };

        f32x16_t acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

#pragma unroll
        for (int s = 0; s < AHEAD; ++s)
            if (s < nSlices) issue(s);

        for (int s = 0; s < nSlices; ++s) {
            // slice s has landed once at most the younger slices' loads are outstanding
            if (s + AHEAD - 1 < nSlices) wait_vmcnt<4 * (AHEAD - 1)>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();      // ... for every wavefront; and slot (s-1)%NSTAGE is free
            if (s + AHEAD < nSlices) issue(s + AHEAD);

            const lds_char* stA = ring + (s % NSTAGE) * STAGE_BYTES;
            const lds_char* stB = stA + TILE * SLICE_BYTES;
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                const int chunk = 2 * g + hh_;
                u32x4_t fa[4], fb[2];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int r = wr * 128 + i * 32 + l32_;
                    fa[i] = *(const lds_u32x4*)(stA + r * SLICE_BYTES + ((chunk ^ ((r >> 2) & 3)) << 4));
                }
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const int c = wc * 64 + j * 32 + l32_;
                    fb[j] = *(const lds_u32x4*)(stB + c * SLICE_BYTES + ((chunk ^ ((c >> 2) & 3)) << 4));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) Mfma<DT>::run(fa[i], fb[j], acc[i][j]);
            }
        }

        // ------------------------------------------------------------------ epilogue
        // acc[i][j][r] holds row  rowBase + wr*128 + i*32 + 8*(r/4) + 4*hh + (r%4)
        //              and column colBase + wc*64 + j*32 + l32.
        // (lane coordinates are laundered through an empty asm so that the per-element index
        //  arithmetic below is not hoisted out of the tile loop into long-lived registers)
        int l32 = l32_, hh = hh_;
        asm volatile("" : "+v"(l32), "+v"(hh));
        const int colW = colBase + wc * 64;                 // first column of this wave, multiple of 64
        const int wordIdx = colW >> 6;
        float rj[2];
        int colP[2];
        uint64_t laneOk[2];                                 // lanes whose column exists
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            colP[j] = colW + j * 32 + l32;
            rj[j] = (MODE == MODE_DENSITY) ? rj_pre[j] * a_ : rj_pre[j];
            laneOk[j] = __ballot(colP[j] < nB);
        }
        double rho[2][2] = {{0.0, 0.0}, {0.0, 0.0}};
        // per-wavefront buffer of undecided pairs, in a ring slot no wavefront reads any more
        lds_uint2* nearBuf = (lds_uint2*)(ring + (nSlices % NSTAGE) * STAGE_BYTES + wave * (NEAR_BUF * 8));
        int nearN = 0;
        auto flush_near = [&]() __attribute__((always_inline)) {
            int base_slot = 0;
            if (lane == 0) base_slot = atomicAdd(&ga.near_cnt[b], nearN);
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
        // rows past nA and the diagonal (d_ii = 0 exactly) need a fix-up; only few wave blocks
        // contain either, the others run the plain variant
        auto epilogue = [&](auto general_tag) __attribute__((always_inline)) {
            constexpr bool GENERAL = decltype(general_tag)::value;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float rs[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) rs[r] = sRinv[wr * 128 + i * 32 + 8 * (r >> 2) + 4 * hh + (r & 3)];
                // phase A: straight-line arithmetic, values left in place of the accumulators
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rowP = rowBase + wr * 128 + i * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        if (MODE == MODE_DENSITY) {
                            const float t = acc[i][j][r] * rs[r];
                            float arg = fmaf(t, rj[j], -a_);
                            if (GENERAL) {
                                if (rowP >= nA) arg = -INFINITY;        // padded row: exp2 -> 0, no bit
                                if (rowP == colP[j]) arg = 0.0f;        // d_ii = 0 exactly
                            }
                            rho[j][r & 1] += (double)__builtin_amdgcn_exp2f(arg);
                            acc[i][j][r] = arg;
                        } else {
                            float c = acc[i][j][r] * rs[r] * rj[j];
                            if (GENERAL && rowP >= nA) c = -INFINITY;
                            acc[i][j][r] = c;
                        }
                    }
                    if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // bound the live ranges: registers are tight
                }
                __builtin_amdgcn_sched_barrier(0);      // keep the row blocks apart: registers are tight
                // phase B: one bit per pair; almost every 2 x 64-pair group has none set
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint64_t m0 = __ballot(acc[i][0][r] >= t_lo) & laneOk[0];
                    const uint64_t m1 = __ballot(acc[i][1][r] >= t_lo) & laneOk[1];
                    if ((m0 | m1) == 0) continue;
                    // lanes 0-31 of a ballot: row with hh = 0; lanes 32-63: the row 4 below it
                    const uint64_t w0 = (m0 & 0xFFFFFFFFull) | (m1 << 32);
                    const uint64_t w1 = (m0 >> 32) | (m1 & 0xFFFFFFFF00000000ull);
                    const int rowP0 = rowBase + wr * 128 + i * 32 + 8 * (r >> 2) + (r & 3);
                    if (w0 != 0 && lane == 0) adj[(size_t)(row_off + rowP0) * bt.W + wordIdx] = w0;
                    if (w1 != 0 && lane == 0) adj[(size_t)(row_off + rowP0 + 4) * bt.W + wordIdx] = w1;
                    if (MODE == MODE_DENSITY) {
                        const uint64_t mS0 = __ballot(acc[i][0][r] >= t_hi), mS1 = __ballot(acc[i][1][r] >= t_hi);
                        const uint64_t s0 = (mS0 & 0xFFFFFFFFull) | (mS1 << 32);
                        const uint64_t s1 = (mS0 >> 32) | (mS1 & 0xFFFFFFFF00000000ull);
                        const uint64_t n0 = w0 & ~s0, n1 = w1 & ~s1;
                        if ((n0 | n1) != 0) {
                            // too close to d_c for fp32: queue the pairs for the fp64 check.  They
                            // collect in this wavefront's LDS buffer; one atomic reserves list slots
                            // for a whole buffer (an atomic per event would cost a memory round trip).
                            const uint64_t mine = hh ? n1 : n0;
                            const bool f0 = (mine >> l32) & 1ull, f1 = (mine >> (32 + l32)) & 1ull;
                            const uint64_t b0 = __ballot(f0), b1 = __ballot(f1);
                            const uint64_t below = (1ull << lane) - 1ull;
                            const int rowP = rowP0 + 4 * hh;
                            if (f0) nearBuf[nearN + __popcll(b0 & below)] = u32x2_t{(uint32_t)rowP, (uint32_t)colP[0]};
                            if (f1) nearBuf[nearN + __popcll(b0) + __popcll(b1 & below)] = u32x2_t{(uint32_t)rowP, (uint32_t)colP[1]};
                            nearN += __popcll(b0) + __popcll(b1);
                            if (nearN > NEAR_BUF - 128) flush_near();
                        }
                    }
                }
            }
        };
        // (the barriers of the slice loop also ordered the sRinv writes before these reads)
        // One variant only: two copies of this block (with and without the fix-ups) made the
        // register allocator spill inside it.
        const int rowW = rowBase + wr * 128;
        epilogue(std::true_type{});
        if (MODE == MODE_DENSITY && nearN > 0) flush_near();

        if (MODE == MODE_DENSITY) {
            // column sums over this wave's 128 rows: combine the two half-waves, one store per column
            const int rt = (rowBase / GRAM_RHO_ROWS) + wr;
            double* out = ga.rho_part + ((size_t)b * bt.W + rt) * bt.n_max;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const double part = rho[j][0] + rho[j][1];
                const double tot = part + __shfl_xor(part, 32, 64);
                if (hh == 0 && colP[j] < nB && rowW < nA) out[colP[j]] = tot;
            }
        }
        // the ring and sRinv are rewritten by the next tile: every wavefront must be done with them
        wait_vmcnt<0>();
        __syncthreads();
    }
}

template <int MODE>
static int launch_gram(const Batch& bt, const GramArgs& ga, pact_dtype k_dt, hipStream_t st,
                       const char* name) {
    const int tiles1 = (bt.n_max + TILE - 1) / TILE;
    int grid_x = tiles1 * tiles1;
    const int cap = (bt.B >= 8) ? 32 : (bt.B >= 2 ? 128 : 256);   // one workgroup per CU, 256 CUs
    if (grid_x > cap) grid_x = cap;
    if (grid_x >= 8) grid_x &= ~7;                // a multiple of the 8 XCDs (see the tile order)
    dim3 grid(grid_x, bt.B);
    const size_t lds = (size_t)NSTAGE * STAGE_BYTES + TILE * sizeof(float);
    static bool raised[2][2] = {{false, false}, {false, false}};
    const int di = k_dt == PACT_BF16 ? 1 : 0;
    const void* fn = (k_dt == PACT_BF16) ? (const void*)gram_kernel<PACT_BF16, MODE>
                                         : (const void*)gram_kernel<PACT_F32, MODE>;
    if (!raised[di][MODE]) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return PACT_ERR_HIP;
        raised[di][MODE] = true;
    }
    if (k_dt == PACT_BF16)
        PACT_LAUNCH_SHMEM(name, (gram_kernel<PACT_BF16, MODE>), grid, dim3(512), lds, st, bt, ga);
    else
        PACT_LAUNCH_SHMEM(name, (gram_kernel<PACT_F32, MODE>), grid, dim3(512), lds, st, bt, ga);
    return PACT_OK;
}

int launch_gram_density(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                        const int32_t* idx, pact_report* rep, hipStream_t st) {
    GramArgs ga;
    ga.keys = (const char*)keys; ga.dk = dk; ga.idx_rows = idx; ga.idx_cols = idx; ga.rep = rep;
    ga.rinv = w.rinv; ga.zeros = (const char*)w.zeros; ga.adj = w.adj; ga.rho_part = w.rho_part;
    ga.near_list = w.near_list; ga.near_cnt = w.near_cnt; ga.margin = (float)cos_margin(dk);
    return launch_gram<MODE_DENSITY>(bt, ga, k_dt, st, "gram_density");
}

int launch_gram_candidates(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                           const int32_t* pruned_idx, const int32_t* center_idx, pact_report* rep,
                           hipStream_t st) {
    GramArgs ga;
    ga.keys = (const char*)keys; ga.dk = dk; ga.idx_rows = pruned_idx; ga.idx_cols = center_idx;
    ga.rep = rep; ga.rinv = w.rinv; ga.zeros = (const char*)w.zeros; ga.adj = w.adj; ga.rho_part = nullptr;
    ga.near_list = nullptr; ga.near_cnt = nullptr; ga.margin = (float)cos_margin(dk);
    return launch_gram<MODE_CAND>(bt, ga, k_dt, st, "gram_candidates");
}

}  // namespace pact

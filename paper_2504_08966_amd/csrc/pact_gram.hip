// The dense contraction of DBDPC (Alg. 2): Gram matrix of the clustering keys on the matrix
// cores, turned into cosines (Eq. 5) in the epilogue and consumed on the spot:
//   MODE_DENSITY  kept x kept  : density terms exp(-d/d_n) summed per column in fp64 (Eq. 6),
//                                one bit per pair "cosine distance <= d_c (+ margin)", and a
//                                list of the pairs too close to d_c for fp32 to decide;
//   MODE_CAND     pruned x centres : one bit per pair "distance < alpha*d_c (+ margin)"
//                                (candidates for Eq. 8).
// The distance matrix itself is never written.
//
// Tiling: a workgroup (4 wavefronts, 2x2) owns a 128x128 output tile and walks the whole key
// width in 128-byte slices through a double-buffered LDS tile pair; every wavefront computes a
// 64x64 block as 2x2 v_mfma_f32_32x32x16_bf16 (or 32x32x2_f32) accumulators.  Rows of both
// operands are rows of the same key matrix, so each lane simply takes 16 contiguous bytes of
// "its" row per MFMA group; the 16-byte chunks of a row are XOR-swizzled by the row number so
// that the 32 rows a half-wave reads at once fall in different LDS banks.  The grid is
// persistent (tile index strides by gridDim.x) because the tile count depends on counts that
// only the device knows.
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
    uint64_t* adj;             // [B][n_max][W]
    double* rho_part;          // [B][W][n_max]
    uint32_t* near_list;       // [B][NEAR_CAP][2]
    int32_t* near_cnt;         // [B]
    float margin;              // worst-case fp32 error of a cosine
};

constexpr int TILE = 128;
constexpr int KSLICE_BYTES = 128;          // bytes of each row per LDS slice (8 chunks of 16 B)
constexpr int CHUNKS = KSLICE_BYTES / 16;  // 8

template <int DT> struct Mfma;
template <> struct Mfma<PACT_BF16> {
    __device__ static __forceinline__ void run(const uint4& a, const uint4& b, f32x16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                    __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mfma<PACT_F32> {
    __device__ static __forceinline__ void run(const uint4& a, const uint4& b, f32x16_t& c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

template <int DT, int MODE>
__global__ __launch_bounds__(256, 2) void gram_kernel(Batch bt, GramArgs ga) {
    __shared__ uint4 sA[2][TILE][CHUNKS];
    __shared__ uint4 sB[2][TILE][CHUNKS];
    __shared__ float2 sRow[TILE];     // per tile row: (1/|u_i|, additive term)

    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int q_kept = clamp_count(ga.rep[b].n_kept, sg.n);
    const int nA = (MODE == MODE_DENSITY) ? q_kept : clamp_count(ga.rep[b].n_pruned, sg.n - q_kept);
    const int nB = (MODE == MODE_DENSITY) ? q_kept : clamp_count(ga.rep[b].n_centers, q_kept);
    const int row_off = (MODE == MODE_DENSITY) ? 0 : q_kept;   // candidate rows follow the kept rows
    if (nA <= 0 || nB <= 0) return;
    const int tilesR = (nA + TILE - 1) / TILE;
    const int tilesC = (nB + TILE - 1) / TILE;
    const int nTiles = tilesR * tilesC;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wr = wave >> 1, wc = wave & 1;
    const int l32 = lane & 31, hh = lane >> 5;

    const size_t row_bytes = (size_t)ga.dk * Elem<DT>::BYTES;
    const int nSlices = (int)((row_bytes + KSLICE_BYTES - 1) / KSLICE_BYTES);
    const int row_bytes_i = (int)row_bytes;                   // a row's tail slice is zero-filled
    const char* __restrict__ keys = ga.keys + (size_t)sg.base * row_bytes;
    const int32_t* idxR = ga.idx_rows + sg.base;
    const int32_t* idxC = ga.idx_cols + sg.base;
    const float* rinv = ga.rinv + sg.base;
    uint64_t* adj = ga.adj + (size_t)b * bt.n_max * bt.W;

    // density constants: arg = cos * a - a = -(d / d_n) * log2(e)
    const float a_ = 1.4426950408889634f / sg.d_n;
    const float thr_cos = (MODE == MODE_DENSITY) ? (1.0f - sg.d_c) : (1.0f - sg.alpha * sg.d_c);
    const float t_lo = (MODE == MODE_DENSITY) ? -(sg.d_c + ga.margin) * a_ : thr_cos - ga.margin;
    const float t_hi = -(sg.d_c - ga.margin) * a_;

    // this thread's 4 load slots: slot u covers tile row (tid>>3) + 32u, chunk tid&7
    const int ld_row = tid >> 3;
    const int ld_chunk = tid & 7;

    // Tile order.  Workgroups are dealt to the 8 XCDs round-robin (XCD = workgroup id mod 8) and
    // every XCD has its own L2, so each XCD works on its own band of tile columns: its key rows
    // for those columns stay in its L2 while the row tiles stream through.
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int nslot = (gridDim.x + 7 - xcd) >> 3;      // workgroups of this launch on this XCD
    const bool banded = tilesC >= 8 && (gridDim.x & 7) == 0;
    const int c_lo = banded ? (int)((long)xcd * tilesC / 8) : 0;
    const int bw = banded ? (int)((long)(xcd + 1) * tilesC / 8) - c_lo : tilesC;
    const int myTiles = banded ? tilesR * bw : nTiles;
    const int t_first = banded ? slot : (int)blockIdx.x;
    const int t_step = banded ? nslot : (int)gridDim.x;

    for (int tl = t_first; tl < myTiles; tl += t_step) {
        const int tr = tl / bw, tc = c_lo + tl % bw;
        const int rowBase = tr * TILE, colBase = tc * TILE;

        // Rows past the end are clamped to the last valid row: their products are discarded in
        // the epilogue (row terms via sRow, columns via the column mask), so no zero fill.
        uint32_t oa[4], ob[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = ld_row + 32 * u;
            const int ra = min(rowBase + r, nA - 1), rb = min(colBase + r, nB - 1);
            oa[u] = (uint32_t)idxR[ra] * (uint32_t)row_bytes_i + ld_chunk * 16;
            ob[u] = (uint32_t)idxC[rb] * (uint32_t)row_bytes_i + ld_chunk * 16;
        }
        if (tid < TILE) {
            const int ra = rowBase + tid;
            float2 v;
            if (MODE == MODE_DENSITY) {
                v.x = (ra < nA) ? rinv[idxR[ra]] : 0.0f;
                v.y = (ra < nA) ? -a_ : -INFINITY;       // padded rows contribute exp2(-inf) = 0
            } else {
                v.x = (ra < nA) ? rinv[idxR[ra]] : __uint_as_float(0x7FC00000u);   // NaN never passes >=
                v.y = 0.0f;
            }
            sRow[tid] = v;
        }

        f32x16_t acc[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

        uint4 ra_[4], rb_[4];
        {
            // the key width need not fill the last 128-byte slice: chunks past it count as zero
            const bool in0 = ld_chunk * 16 < row_bytes_i;
            const uint32_t back = in0 ? 0u : (uint32_t)(ld_chunk * 16);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ra_[u] = *(const uint4*)(keys + (oa[u] - back));
                rb_[u] = *(const uint4*)(keys + (ob[u] - back));
                if (!in0) { ra_[u] = make_uint4(0, 0, 0, 0); rb_[u] = make_uint4(0, 0, 0, 0); }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = ld_row + 32 * u;
            sA[0][r][ld_chunk ^ (r & 7)] = ra_[u];
            sB[0][r][ld_chunk ^ (r & 7)] = rb_[u];
        }
        __syncthreads();

        for (int ks = 0; ks < nSlices; ++ks) {
            const int buf = ks & 1;
            if (ks + 1 < nSlices) {
                const int off = (ks + 1) * KSLICE_BYTES;
                const bool in1 = off + ld_chunk * 16 < row_bytes_i;
                const uint32_t o1 = in1 ? (uint32_t)off : 0u;
                const uint32_t back = in1 ? 0u : (uint32_t)(ld_chunk * 16);
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    ra_[u] = *(const uint4*)(keys + (oa[u] + o1 - back));
                    rb_[u] = *(const uint4*)(keys + (ob[u] + o1 - back));
                    if (!in1) { ra_[u] = make_uint4(0, 0, 0, 0); rb_[u] = make_uint4(0, 0, 0, 0); }
                }
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int chunk = 2 * g + hh;
                uint4 fa[2], fb[2];
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const int r = wr * 64 + s * 32 + l32;
                    const int c = wc * 64 + s * 32 + l32;
                    fa[s] = sA[buf][r][chunk ^ (r & 7)];
                    fb[s] = sB[buf][c][chunk ^ (c & 7)];
                }
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j) Mfma<DT>::run(fa[i], fb[j], acc[i][j]);
            }
            if (ks + 1 < nSlices) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int r = ld_row + 32 * u;
                    sA[buf ^ 1][r][ld_chunk ^ (r & 7)] = ra_[u];
                    sB[buf ^ 1][r][ld_chunk ^ (r & 7)] = rb_[u];
                }
            }
            __syncthreads();
        }

        // ------------------------------------------------------------------ epilogue
        // acc[i][j][r] holds row  rowBase + wr*64 + i*32 + 8*(r/4) + 4*hh + (r%4)
        //              and column colBase + wc*64 + j*32 + l32.
        const int colW = colBase + wc * 64;                 // first column of this wave, multiple of 64
        const int wordIdx = colW >> 6;
        const int validCols = min(max(nB - colW, 0), 64);
        const uint64_t colMask = validCols >= 64 ? ~0ull : ((1ull << validCols) - 1ull);
        float rj[2];
        int colP[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            colP[j] = colW + j * 32 + l32;
            rj[j] = (colP[j] < nB) ? rinv[idxC[colP[j]]] : 0.0f;
            if (MODE == MODE_DENSITY) rj[j] *= a_;
        }
        const bool diagWave = (MODE == MODE_DENSITY) && (rowBase + wr * 64 == colW);
        double rho[2] = {0.0, 0.0};

#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rowL = wr * 64 + i * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
                const float2 rv = sRow[rowL];
                const int rowP = rowBase + rowL;
                uint64_t mMaybe[2], mSure[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (MODE == MODE_DENSITY) {
                        const float t = acc[i][j][r] * rv.x;
                        float arg = fmaf(t, rj[j], rv.y);
                        if (diagWave && rowP == colP[j]) arg = 0.0f;     // d_ii = 0 exactly
                        rho[j] += (double)__builtin_amdgcn_exp2f(arg);
                        mMaybe[j] = __ballot(arg >= t_lo);
                        mSure[j] = __ballot(arg >= t_hi);
                    } else {
                        const float c = acc[i][j][r] * rv.x * rj[j];
                        mMaybe[j] = __ballot(c >= t_lo);
                        mSure[j] = 0;
                    }
                }
                // lanes 0-31 of a ballot: row with hh = 0; lanes 32-63: the row 4 below it
                const uint64_t w0 = ((mMaybe[0] & 0xFFFFFFFFull) | (mMaybe[1] << 32)) & colMask;
                const uint64_t w1 = ((mMaybe[0] >> 32) | (mMaybe[1] & 0xFFFFFFFF00000000ull)) & colMask;
                const int rowP0 = rowBase + wr * 64 + i * 32 + 8 * (r >> 2) + (r & 3);
                if (w0 != 0 && lane == 0) adj[(size_t)(row_off + rowP0) * bt.W + wordIdx] = w0;
                if (w1 != 0 && lane == 0) adj[(size_t)(row_off + rowP0 + 4) * bt.W + wordIdx] = w1;
                if (MODE == MODE_DENSITY) {
                    const uint64_t s0 = ((mSure[0] & 0xFFFFFFFFull) | (mSure[1] << 32));
                    const uint64_t s1 = ((mSure[0] >> 32) | (mSure[1] & 0xFFFFFFFF00000000ull));
                    const uint64_t n0 = w0 & ~s0, n1 = w1 & ~s1;
                    if ((n0 | n1) != 0) {
                        // one atomic per wavefront reserves the slots of all its near pairs
                        const uint64_t mine = hh ? n1 : n0;
                        const bool f0 = (mine >> l32) & 1ull, f1 = (mine >> (32 + l32)) & 1ull;
                        const uint64_t b0 = __ballot(f0), b1 = __ballot(f1);
                        const int total = __popcll(b0) + __popcll(b1);
                        int base_slot = 0;
                        if (lane == 0) base_slot = atomicAdd(&ga.near_cnt[b], total);
                        base_slot = __shfl(base_slot, 0, 64);
                        const uint64_t below = (1ull << lane) - 1ull;
                        if (f0) {
                            const int slot = base_slot + __popcll(b0 & below);
                            if (slot < NEAR_CAP) {
                                uint32_t* e = ga.near_list + ((size_t)b * NEAR_CAP + slot) * 2;
                                e[0] = (uint32_t)rowP; e[1] = (uint32_t)colP[0];
                            }
                        }
                        if (f1) {
                            const int slot = base_slot + __popcll(b0) + __popcll(b1 & below);
                            if (slot < NEAR_CAP) {
                                uint32_t* e = ga.near_list + ((size_t)b * NEAR_CAP + slot) * 2;
                                e[0] = (uint32_t)rowP; e[1] = (uint32_t)colP[1];
                            }
                        }
                    }
                }
            }
        }
        if (MODE == MODE_DENSITY) {
            // column sums over this wave's 64 rows: combine the two half-waves, one store per column
            const int rt64 = (rowBase >> 6) + wr;
            double* out = ga.rho_part + ((size_t)b * bt.W + rt64) * bt.n_max;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const double tot = rho[j] + __shfl_xor(rho[j], 32, 64);
                if (hh == 0 && colP[j] < nB && rowBase + wr * 64 < nA) out[colP[j]] = tot;
            }
        }
        // sRow and the LDS tiles are rewritten at the top of the next tile: all waves must be
        // done reading them
        __syncthreads();
    }
}

template <int MODE>
static int launch_gram(const Batch& bt, const GramArgs& ga, pact_dtype k_dt, hipStream_t st,
                       const char* name) {
    const int tiles1 = (bt.n_max + TILE - 1) / TILE;
    int grid_x = tiles1 * tiles1;
    const int cap = (bt.B >= 8) ? 128 : 512;      // two workgroups per CU resident, 256 CUs
    if (grid_x > cap) grid_x = cap;
    if (grid_x >= 8) grid_x &= ~7;                // a multiple of the 8 XCDs (see the tile order)
    dim3 grid(grid_x, bt.B);
    if (k_dt == PACT_BF16)
        PACT_LAUNCH(name, (gram_kernel<PACT_BF16, MODE>), grid, dim3(256), st, bt, ga);
    else
        PACT_LAUNCH(name, (gram_kernel<PACT_F32, MODE>), grid, dim3(256), st, bt, ga);
    return PACT_OK;
}

int launch_gram_density(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                        const int32_t* idx, pact_report* rep, hipStream_t st) {
    GramArgs ga;
    ga.keys = (const char*)keys; ga.dk = dk; ga.idx_rows = idx; ga.idx_cols = idx; ga.rep = rep;
    ga.rinv = w.rinv; ga.adj = w.adj; ga.rho_part = w.rho_part; ga.near_list = w.near_list;
    ga.near_cnt = w.near_cnt; ga.margin = (float)cos_margin(dk);
    return launch_gram<MODE_DENSITY>(bt, ga, k_dt, st, "gram_density");
}

int launch_gram_candidates(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                           const int32_t* pruned_idx, const int32_t* center_idx, pact_report* rep,
                           hipStream_t st) {
    GramArgs ga;
    ga.keys = (const char*)keys; ga.dk = dk; ga.idx_rows = pruned_idx; ga.idx_cols = center_idx;
    ga.rep = rep; ga.rinv = w.rinv; ga.adj = w.adj; ga.rho_part = nullptr; ga.near_list = nullptr;
    ga.near_cnt = nullptr; ga.margin = (float)cos_margin(dk);
    return launch_gram<MODE_CAND>(bt, ga, k_dt, st, "gram_candidates");
}

}  // namespace pact

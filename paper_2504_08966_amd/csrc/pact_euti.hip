// EUTI (Alg. 1): global query (Eq. 1), importance score (Eq. 2), percentile split (Eq. 3/4),
// plus the per-token preparation of the clustering keys (norms, cleared bitmap rows).
// All arithmetic of the score is fp64 (the stage is bound by reading H from HBM, the ALU work
// is free), rounded once to fp32; the split then compares fp32 bit patterns exactly.
#include "pact_internal.h"

namespace pact {

// ------------------------------------------------------------------------------------------
// First kernel of a call.  Three independent jobs share one launch:
//   blocks [nQ, nQ + nKeyBlocks)      : one wavefront per token: squared key norm (fp64),
//                                       reciprocal norm (fp32), cleared bitmap row, and the
//                                       per-token initial state (status, cluster id, counts);
//   blocks [0, nQ)                    : Eq. 1 pass 1, column sums of one row chunk of Q; rows wider than
//                                       1024 columns are shared out in groups of 1024 columns
//                                       (nQ = QG_CHUNKS x groups, or 0 without a query pass).
// grid (nKeyBlocks + nQ, B), block 256.
struct PrepArgs {
    const char* keys; int32_t dk;
    const char* q; int32_t qcols;            // q == nullptr: no query pass
    double* nn; float* rinv; uint64_t* adj; double* qg_part;
    uint32_t* status; int32_t* ident; int32_t* near_cnt; int32_t* tie_cnt;
    pact_report* rep; int32_t* cluster_id; int32_t* cluster_counts;
    const int32_t* n_idx_dev; uint32_t* zeros;
    uint16_t* ksplit;                        // fp32 keys only: [total][3][dk rounded up to 8] bf16 parts for the Gram passes
    int32_t mode; int32_t n_key_blocks; int32_t n_q_blocks;
};

template <int KDT, int QDT>
__global__ __launch_bounds__(256) void prep_kernel(Batch bt, PrepArgs a) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int n_q_blocks = a.n_q_blocks;             // the query chunks come first: they are the longer job
    if ((int)blockIdx.x >= n_q_blocks) {
        const int kblk = blockIdx.x - n_q_blocks;
        if (kblk == 0 && b == 0 && threadIdx.x < 64) a.zeros[threadIdx.x] = 0u;
        if (kblk == 0 && threadIdx.x == 0) {
            a.near_cnt[2 * b] = 0; a.near_cnt[2 * b + 1] = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) a.tie_cnt[4 * b + k] = 0;
            pact_report* rp = a.rep + b;
            const int mode = a.mode;
            if (mode == INIT_REDUCE || mode == INIT_DBDPC_ALL || mode == INIT_DBDPC_SUBSET) {
                if (mode != INIT_REDUCE) {
                    const int k = (mode == INIT_DBDPC_ALL) ? sg.n : min(max(*a.n_idx_dev, 0), sg.n);
                    rp->n_kept = k;
                    rp->n_pruned = (mode == INIT_DBDPC_ALL) ? 0 : sg.n - k;
                }
                rp->n_centers = 0; rp->rounds = 0; rp->dc_checked_pairs = 0; rp->dc_near_ties = 0;
                rp->refine_overflow = 0; rp->n_reincorporated = 0; rp->n_dropped = 0;
                rp->zero_norm_seen = 0;     // counted by the assignment kernels, which run later
                rp->max_key_distance = 0.0f;
                rp->rho_rechecked = 0; rp->rho_near_ties = 0;
                // (a clustering call on a subset follows a split, whose two counters it adds to)
                if (mode != INIT_DBDPC_SUBSET) { rp->score_near_ties = 0; rp->nonfinite_seen = 0; }
                rp->reserved[0] = 0;
            }
            if (mode == INIT_REINC) { rp->n_reincorporated = 0; rp->n_dropped = 0; }
        }
        const int i = kblk * 4 + (threadIdx.x >> 6);
        if (i >= sg.n) return;
        const size_t g = (size_t)sg.base + i;
        const char* row = a.keys + g * (size_t)a.dk * Elem<KDT>::BYTES;
        const double v = wave_dot64<KDT>(row, row, a.dk, lane);
        if constexpr (KDT == PACT_F32) {
            // x = hi + mid + lo, each the bf16 nearest to what the parts before it leave (the
            // differences are exact in fp32); together they carry the 24 bits of x
            const int dkp = (a.dk + 7) & ~7;                   // plane pitch: whole 16-byte chunks, zero-padded
            uint16_t* sp = a.ksplit + g * (size_t)(3 * dkp);
            for (int e = lane * 4; e < dkp; e += 256) {
                const float4 x4 = (e < a.dk) ? *(const float4*)(row + (size_t)e * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
                const float x[4] = {x4.x, x4.y, x4.z, x4.w};
                uint32_t part[3][4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float r = x[i];
#pragma unroll
                    for (int pl = 0; pl < 3; ++pl) {
                        part[pl][i] = f32_to_bf16_rne(r);
                        r -= __uint_as_float(part[pl][i] << 16);
                    }
                }
#pragma unroll
                for (int pl = 0; pl < 3; ++pl)
                    *(uint2*)(sp + (size_t)pl * dkp + e) =
                        make_uint2(part[pl][0] | (part[pl][1] << 16), part[pl][2] | (part[pl][3] << 16));
            }
        }
        // The bitmap is used over (kept tokens) x (kept tokens).  In a full reduction that is
        // n - m rows and columns unless scores tie at the threshold (Eq. 3 / 4); the split
        // clears the rest itself in that case.
        uint64_t* arow = a.adj + ((size_t)b * bt.n_max + i) * bt.W;
        const int side = (a.mode == INIT_REDUCE) ? sg.n - prune_rank(sg.lambda, sg.n) : sg.n;
        const int Wn = (i < side) ? (side + 63) >> 6 : 0;
        for (int k = lane; k < Wn; k += 64) arow[k] = 0ull;
        if (lane == 0) {
            a.nn[g] = v;
            a.rinv[g] = v > 0.0 ? (float)(1.0 / sqrt(v)) : 0.0f;
            if (a.mode == INIT_REDUCE || a.mode == INIT_DBDPC_ALL || a.mode == INIT_DBDPC_SUBSET) {
                a.status[(size_t)b * bt.n_max + i] = ST_UNKNOWN;
                a.ident[g] = i;
                a.cluster_id[g] = -1;
                if (a.cluster_counts) a.cluster_counts[g] = 0;
            }
        }
        return;
    }
    // ---- Eq. 1, pass 1
    const int chunk = blockIdx.x % QG_CHUNKS, cgroup = blockIdx.x / QG_CHUNKS;
    const int rows_per = (sg.n + QG_CHUNKS - 1) / QG_CHUNKS;
    const int r0 = chunk * rows_per;
    const int r1 = min(sg.n, r0 + rows_per);
    const size_t row_bytes = (size_t)a.qcols * Elem<QDT>::BYTES;
    double* out = a.qg_part + ((size_t)b * QG_CHUNKS + chunk) * a.qcols;
    // Four columns per thread.  Rows of at most 512 (256) columns leave half (three quarters) of
    // the threads without columns: they take every second (fourth) row of the chunk instead, and
    // the row groups' sums meet in LDS.
    const int RG = a.qcols <= 256 ? 4 : a.qcols <= 512 ? 2 : 1;
    const int tpg = 256 / RG;
    const int rg = threadIdx.x / tpg, ct = threadIdx.x % tpg;
    __shared__ double s_part[192 * 4];
    auto sum_rows = [&](int c, double (&acc)[4]) __attribute__((always_inline)) {
        const char* base = a.q + (size_t)sg.base * row_bytes + (size_t)c * Elem<QDT>::BYTES;
        for (int r = r0 + rg; r < r1; r += 8 * RG) {
            float f[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const bool ok = r + u * RG < r1;
                const char* p = base + (size_t)(ok ? r + u * RG : r0) * row_bytes;
                if (QDT == PACT_BF16) {
                    const uint2 v = *(const uint2*)p;
                    f[u][0] = __uint_as_float(v.x << 16); f[u][1] = __uint_as_float(v.x & 0xFFFF0000u);
                    f[u][2] = __uint_as_float(v.y << 16); f[u][3] = __uint_as_float(v.y & 0xFFFF0000u);
                } else {
                    const float4 v = *(const float4*)p;
                    f[u][0] = v.x; f[u][1] = v.y; f[u][2] = v.z; f[u][3] = v.w;
                }
                if (!ok) { f[u][0] = f[u][1] = f[u][2] = f[u][3] = 0.0f; }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[i] += (double)f[u][i];
        }
    };
    if (RG == 1) {
        const int c = cgroup * 1024 + threadIdx.x * 4;
        if (c < a.qcols) {
            double acc[4] = {0.0, 0.0, 0.0, 0.0};
            sum_rows(c, acc);
#pragma unroll
            for (int i = 0; i < 4; ++i) out[c + i] = acc[i];
        }
        return;
    }
    const int c = ct * 4;
    const bool act = c < a.qcols;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    if (act) sum_rows(c, acc);
    if (act && rg > 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) s_part[((rg - 1) * tpg + ct) * 4 + i] = acc[i];
    }
    __syncthreads();
    if (act && rg == 0) {
        for (int g = 1; g < RG; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += s_part[((g - 1) * tpg + ct) * 4 + i];
#pragma unroll
        for (int i = 0; i < 4; ++i) out[c + i] = acc[i];
    }
}

// |h_g|_2 in fp64 by one wavefront (8 independent 16-byte loads in flight per lane).
template <int HDT>
__device__ __forceinline__ void hnorm_row(const char* __restrict__ hidden, int h, size_t g, int lane,
                                          double* __restrict__ hnorm, bool stream) {
    const char* hp = hidden + g * (size_t)h * Elem<HDT>::BYTES;
    constexpr int HE = Elem<HDT>::EPL;
    double ss[4] = {0.0, 0.0, 0.0, 0.0};
    for (int e0 = lane * HE; e0 < h; e0 += 8 * 64 * HE) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int e = e0 + u * 64 * HE;
            v[u] = (e >= h) ? make_uint4(0, 0, 0, 0)
                 : stream ? load_once16(hp + (size_t)e * Elem<HDT>::BYTES)
                          : *(const uint4*)(hp + (size_t)e * Elem<HDT>::BYTES);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            double x[8];
            Elem<HDT>::widen(v[u], x);
#pragma unroll
            for (int k = 0; k < HE; ++k) ss[u & 3] = fma(x[k], x[k], ss[u & 3]);
        }
    }
    const double sst = wave_sum_f64((ss[0] + ss[1]) + (ss[2] + ss[3]));
    if (lane == 0) hnorm[g] = sqrt(sst);
}
// The norms are split over two launches: tokens below hnorm_split(n, share) go with the global
// query, the others with the logits (share in 256ths; a multiple of the 16 tokens of a block).
__host__ __device__ __forceinline__ int hnorm_split(int n, int share) {
    const int s = (((n * share) >> 8) + SCORE_TOK_PER_WG - 1) & ~(SCORE_TOK_PER_WG - 1);
    return s < n ? s : n;
}

// Eq. 1, pass 2, and the hidden-state norms of Eq. 2, two independent jobs in one launch (the
// first is a handful of blocks; the second streams H, the stage's one large read, which needs
// neither the global query nor the logits and so need not wait for them):
//   blocks [0, nq_blocks): the global query - the chunk partials summed in a fixed order and
//       divided by n (64 columns x 16 slices of the chunk range per block), or, when the caller
//       supplied the global query ([B, qcols]), its widening to fp64 (1024 columns per block);
//   the other blocks: |h_i|_2 in fp64, one wavefront per token, 16 tokens per block.
// grid (nq_blocks + ceil(n_max/16), B), block 1024.
// Where column c of the global query goes.  The logits kernel for grouped-query heads wants it
// laid out as its lanes read it (see there): element k of 16-byte chunk cc of query head
// kvh * rep + r at ((r * epl + k) * n_kv + kvh) * lph + cc; rep == 0: as it is.
struct QgLayout {
    int rep, n_kv, d_h, lph, epl;
    __device__ __forceinline__ int at(int c) const {
        if (rep == 0) return c;
        const int j = c / d_h, e = c - j * d_h;
        return (((j % rep) * epl + (e % epl)) * n_kv + j / rep) * lph + e / epl;
    }
};

template <int HDT, int QDT>
__global__ __launch_bounds__(1024) void qglobal_hnorm_kernel(Batch bt, int qcols, int q_per_token, int nq_blocks,
                                                             QgLayout lay,
                                                             const double* __restrict__ qg_part,
                                                             const char* __restrict__ q_given,
                                                             double* __restrict__ qg,
                                                             const char* __restrict__ hidden, int h,
                                                             double* __restrict__ hnorm, int hshare, int stream) {
    __shared__ double s_p[16][64];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    if ((int)blockIdx.x < nq_blocks) {
        if (q_per_token) {
            const int cl = threadIdx.x & 63, slice = threadIdx.x >> 6;
            const int c = blockIdx.x * 64 + cl;
            constexpr int PER = QG_CHUNKS / 16;
            double acc = 0.0;
            if (c < qcols) {
                const double* in = qg_part + ((size_t)b * QG_CHUNKS + slice * PER) * qcols + c;
                double v[PER];
#pragma unroll
                for (int k = 0; k < PER; ++k) v[k] = in[(size_t)k * qcols];
#pragma unroll
                for (int k = 0; k < PER; ++k) acc += v[k];
            }
            s_p[slice][cl] = acc;
            __syncthreads();
            if (slice == 0 && c < qcols) {
                double t = 0.0;
#pragma unroll
                for (int k = 0; k < 16; ++k) t += s_p[k][cl];
                qg[(size_t)b * qcols + lay.at(c)] = t / (double)sg.n;
            }
        } else {
            const int c = blockIdx.x * 1024 + threadIdx.x;
            if (c < qcols) {
                const char* p = q_given + ((size_t)b * qcols + c) * Elem<QDT>::BYTES;
                float f;
                if (QDT == PACT_BF16) f = __uint_as_float((uint32_t)(*(const uint16_t*)p) << 16);
                else f = *(const float*)p;
                qg[(size_t)b * qcols + lay.at(c)] = (double)f;
            }
        }
        return;
    }
    const int i = (blockIdx.x - nq_blocks) * SCORE_TOK_PER_WG + (threadIdx.x >> 6);
    if (i >= hnorm_split(sg.n, hshare)) return;
    hnorm_row<HDT>(hidden, h, (size_t)sg.base + i, threadIdx.x & 63, hnorm, stream != 0);
}

constexpr int LOGITS_MAX_REP = 8;        // query heads per key head that the grouped fast path handles
constexpr int LOGITS_QG_LDS = 4096;      // columns of the global query that its LDS copy holds
// key row of at most 1 KB, a power-of-two number of whole 16-byte chunks per head
__host__ __device__ inline bool logits_shaped(int n_kv, int d_h, int elem_bytes) {
    const int lph = d_h * elem_bytes / 16;
    return (size_t)n_kv * d_h * elem_bytes <= 1024 && lph * 16 == d_h * elem_bytes && lph >= 1 && (lph & (lph - 1)) == 0;
}
__host__ __device__ inline bool logits_grouped(int n_kv, int n_q, int d_h, int elem_bytes) {
    const int rep = n_q / n_kv;
    return rep > 1 && rep <= LOGITS_MAX_REP && logits_shaped(n_kv, d_h, elem_bytes) && n_q * d_h <= LOGITS_QG_LDS;
}

// ------------------------------------------------------------------------------------------
// Eq. 2, pass 1: one wavefront per token computes the n_q logits k_i^(g(j)) . Qg^(j); the
// workgroup (SCORE_TOK_PER_WG tokens) then leaves one online-softmax partial (max, sum of exp)
// per head.  grid (ceil(n_max/16), B), block 1024.
template <int KDT, int HDT, bool GROUPED>
__global__ __launch_bounds__(1024) void score_logits_kernel(Batch bt, const char* __restrict__ keys, int n_kv, int d_h,
                                                            int n_q, const double* __restrict__ qg,
                                                            double* __restrict__ logits,
                                                            double* __restrict__ sm_part, int n_logit_blocks,
                                                            const char* __restrict__ hidden, int h,
                                                            double* __restrict__ hnorm, int hshare, int stream) {
    __shared__ double s_l[SCORE_TOK_PER_WG][PACT_MAX_QHEADS];
    __shared__ double s_qg[GROUPED ? LOGITS_QG_LDS : 1];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if ((int)blockIdx.x >= n_logit_blocks) {
        // the rest of the hidden-state norms (independent of the logits; rides in this launch)
        const int i = hnorm_split(sg.n, hshare) + ((int)blockIdx.x - n_logit_blocks) * SCORE_TOK_PER_WG + wave;
        if (i < sg.n) hnorm_row<HDT>(hidden, h, (size_t)sg.base + i, lane, hnorm, stream != 0);
        return;
    }
    const int t0 = blockIdx.x * SCORE_TOK_PER_WG;
    if (t0 >= sg.n) return;
    const int qcols = n_q * d_h;
    const int rep = n_q / n_kv;
    const double* qgb = qg + (size_t)b * qcols;
    const size_t krow = (size_t)n_kv * d_h * Elem<KDT>::BYTES;

    // Fast paths (the usual shapes: key row of at most 1 KB, a power-of-two number of 16-byte
    // chunks per head): the whole key row is one load per lane and a head's logit is a reduction
    // over the few lanes that hold it.  `fast`: one query head per key head.  GROUPED (its own
    // build; the host checks logits_grouped()): up to LOGITS_MAX_REP query heads per key head
    // (grouped-query attention); a lane then forms the partial logits of all query heads of its
    // key head, against a copy of the global query in LDS.
    const int lph = (int)((size_t)d_h * Elem<KDT>::BYTES / 16);      // lanes (chunks) per head
    const bool fast = rep == 1 && logits_shaped(n_kv, d_h, Elem<KDT>::BYTES);
    const int i = t0 + wave;
    if constexpr (GROUPED) {
        // The copy is laid out so that the lanes of a wavefront read neighbouring words: element k
        // of chunk cc of query head kvh * rep + r sits at ((r * EPL + k) * n_kv + kvh) * lph + cc,
        // i.e. at (r * EPL + k) * (lanes that hold the key row) + (the lane that needs it).
        constexpr int EPL = Elem<KDT>::EPL;
        const int klanes = n_kv * lph;
        for (int c = threadIdx.x; c < qcols; c += 1024) s_qg[c] = qgb[c];      // (left in this order by the kernel before)
        __syncthreads();
        if (i < sg.n) {
            const size_t g = (size_t)sg.base + i;
            const bool klane = lane < klanes;
            const int kvh = lane / lph;
            double acc[LOGITS_MAX_REP];
#pragma unroll
            for (int r = 0; r < LOGITS_MAX_REP; ++r) acc[r] = 0.0;
            if (klane) {
                const uint4 kv = *(const uint4*)(keys + g * krow + (size_t)lane * 16);
                double x[8];
                Elem<KDT>::widen(kv, x);
#pragma unroll
                for (int r = 0; r < LOGITS_MAX_REP; ++r)
                    if (r < rep) {
#pragma unroll
                        for (int k = 0; k < EPL; ++k) acc[r] = fma(x[k], s_qg[(r * EPL + k) * klanes + lane], acc[r]);
                    }
            }
#pragma unroll
            for (int r = 0; r < LOGITS_MAX_REP; ++r)
                if (r < rep) acc[r] = group_sum_f64(acc[r], lph);
            if (klane && (lane & (lph - 1)) == 0) {
#pragma unroll
                for (int r = 0; r < LOGITS_MAX_REP; ++r)
                    if (r < rep) {
                        logits[g * n_q + kvh * rep + r] = acc[r];
                        s_l[wave][kvh * rep + r] = acc[r];
                    }
            }
        }
    } else if (i < sg.n) {
        const size_t g = (size_t)sg.base + i;
        const char* kp = keys + g * krow;
        if (fast) {
            // lane l holds elements [l * EPL, (l + 1) * EPL) of the row, i.e. of head l / lph
            const bool klane = (size_t)lane * 16 < krow;
            double acc = 0.0;
            if (klane) {
                const uint4 kv = *(const uint4*)(kp + (size_t)lane * 16);
                double x[8];
                Elem<KDT>::widen(kv, x);
                const double* qq = qgb + lane * Elem<KDT>::EPL;
#pragma unroll
                for (int k = 0; k < Elem<KDT>::EPL; ++k) acc = fma(x[k], qq[k], acc);
            }
            acc = group_sum_f64(acc, lph);
            if (klane && (lane & (lph - 1)) == 0) {
                const int j = lane / lph;
                logits[g * n_q + j] = acc;
                s_l[wave][j] = acc;
            }
        } else {
            // per-head logits, one head after the other
            for (int j = 0; j < n_q; ++j) {
                const int kvh = j / rep;
                double acc = 0.0;
                for (int e = lane * Elem<KDT>::EPL; e < d_h; e += 64 * Elem<KDT>::EPL) {
                    const uint4 v = *(const uint4*)(kp + (size_t)(kvh * d_h + e) * Elem<KDT>::BYTES);
                    double x[8];
                    Elem<KDT>::widen(v, x);
                    const double* qq = qgb + j * d_h + e;
#pragma unroll
                    for (int k = 0; k < Elem<KDT>::EPL; ++k) acc = fma(x[k], qq[k], acc);
                }
                acc = wave_sum_f64(acc);
                if (lane == 0) {
                    logits[g * n_q + j] = acc;
                    s_l[wave][j] = acc;
                }
            }
        }
    }
    __syncthreads();
    // the workgroup's softmax partial per head: thread (head j, token t) = 16 * j + t takes one
    // exponential, the 16 lanes of a head combine (SCORE_TOK_PER_WG * PACT_MAX_QHEADS threads at most)
    static_assert(SCORE_TOK_PER_WG == 16 && SCORE_TOK_PER_WG * PACT_MAX_QHEADS <= 1024, "one thread per (token, head)");
    {
        const int j = threadIdx.x >> 4, t = threadIdx.x & 15;
        const int cnt = min(SCORE_TOK_PER_WG, sg.n - t0);
        if (j < n_q) {                                             // (whole groups of 16 lanes take the branch)
            const double v = t < cnt ? s_l[t][j] : -INFINITY;
            double m = v;
            m = group_max_f64<16>(m);
            double e = t < cnt ? exp(v - m) : 0.0;
            e = group_sum_f64(e, 16);
            if (t == 0) {
                const int smwg = (bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
                double* out = sm_part + (((size_t)b * smwg + blockIdx.x) * n_q + j) * 2;
                out[0] = m;
                out[1] = e;
            }
        }
    }
}

// (max, normaliser) of one head from the workgroup partials, by one wavefront: every lane
// loads its (max, sum) pairs 8 at a time, then the usual two-step combine.
__device__ __forceinline__ void combine_softmax_partials(const double* part, int nwg, int stride, int lane,
                                                         double& M, double& Z) {
    // the first 512 pairs stay in registers between the two steps (one fetch, not two)
    double2 v0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int w = lane + 64 * u;
        v0[u] = (w < nwg) ? *(const double2*)(part + (size_t)w * stride) : make_double2(-INFINITY, 0.0);
    }
    double m = -INFINITY;
#pragma unroll
    for (int u = 0; u < 8; ++u) m = fmax(m, v0[u].x);
    for (int w0 = lane + 512; w0 < nwg; w0 += 512) {
        double2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int w = w0 + 64 * u;
            v[u] = (w < nwg) ? *(const double2*)(part + (size_t)w * stride) : make_double2(-INFINITY, 0.0);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) m = fmax(m, v[u].x);
    }
    m = wave_max_f64(m);
    double z = 0.0;
#pragma unroll
    for (int u = 0; u < 8; ++u) z += (v0[u].y != 0.0) ? v0[u].y * exp(v0[u].x - m) : 0.0;
    for (int w0 = lane + 512; w0 < nwg; w0 += 512) {
        double2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int w = w0 + 64 * u;
            v[u] = (w < nwg) ? *(const double2*)(part + (size_t)w * stride) : make_double2(-INFINITY, 0.0);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) z += (v[u].y != 0.0) ? v[u].y * exp(v[u].x - m) : 0.0;
    }
    M = m;
    Z = wave_sum_f64(z);
}

// ------------------------------------------------------------------------------------------
// Eq. 2, pass 2 for many query heads, first half: (max, normaliser) of every head, once per sample
// (left to every workgroup of the kernel below, the n_q * n / 16 exponentials of the combine are
// most of that kernel's time from a dozen heads on).  mz: [B][n_q][2].  grid (n_q, B), block 64.
__global__ __launch_bounds__(64) void softmax_combine_kernel(Batch bt, int n_q, const double* __restrict__ sm_part,
                                                             double* __restrict__ mz) {
    const int b = blockIdx.y, j = blockIdx.x;
    const Seg sg = bt.s[b];
    if (sg.n <= 0) return;
    const int smwg = (bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    const int nwg = (sg.n + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    double m, z;
    combine_softmax_partials(sm_part + ((size_t)b * smwg * n_q + j) * 2, nwg, n_q * 2, threadIdx.x, m, z);
    if (threadIdx.x == 0) { mz[((size_t)b * n_q + j) * 2] = m; mz[((size_t)b * n_q + j) * 2 + 1] = z; }
}

// Eq. 2, pass 2: (max, normaliser) per head - combined here from the partials, or read from mz -
// then s_i = |h_i| * (1/n_q) sum_j exp(l_ij - M_j) / Z_j.
// A workgroup finishes TOK tokens with TOK * PARTS threads: thread (token, part) takes the heads
// part, part + PARTS, ... of its token (and its wavefront the heads wave, wave + TOK * PARTS / 64,
// ... of the combine); the parts of a token meet in LDS and are added in the order of their numbers.
// grid (ceil(n_max/TOK), B), block TOK * PARTS.
template <int TOK, int PARTS>
__global__ __launch_bounds__(TOK * PARTS) void score_final_kernel(Batch bt, int n_q,
                                                                  const double* __restrict__ logits,
                                                                  const double* __restrict__ hnorm,
                                                                  const double* __restrict__ sm_part,
                                                                  const double* __restrict__ mz,
                                                                  float* __restrict__ scores) {
    __shared__ double s_M[PACT_MAX_QHEADS], s_Z[PACT_MAX_QHEADS];
    __shared__ double s_acc[PARTS > 1 ? PARTS - 1 : 1][TOK];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    if (blockIdx.x * TOK >= sg.n) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int tok = threadIdx.x % TOK, part = threadIdx.x / TOK;
    const int smwg = (bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    const int nwg = (sg.n + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    // this thread's token: its norm and first logits are requested before the partials are
    // combined (they do not depend on them)
    const int i = blockIdx.x * TOK + tok;
    const size_t g = (size_t)sg.base + min(i, sg.n - 1);
    const double hn = hnorm[g];
    double lg[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) lg[u] = (part + u * PARTS < n_q) ? logits[g * n_q + part + u * PARTS] : 0.0;
    if (mz) {
        if ((int)threadIdx.x < n_q) {
            s_M[threadIdx.x] = mz[((size_t)b * n_q + threadIdx.x) * 2];
            s_Z[threadIdx.x] = mz[((size_t)b * n_q + threadIdx.x) * 2 + 1];
        }
    } else {
        for (int j = wave; j < n_q; j += TOK * PARTS / 64) {
            double m, z;
            combine_softmax_partials(sm_part + ((size_t)b * smwg * n_q + j) * 2, nwg, n_q * 2, lane, m, z);
            if (lane == 0) { s_M[j] = m; s_Z[j] = z; }
        }
    }
    __syncthreads();
    // the two ablations of Eq. 2: without the norm; norm only (softmax term -> 1/n)
    const bool norm_only = (sg.flags & PACT_FLAG_SCORE_NORM_ONLY) != 0;
    double acc = 0.0;
    if (!norm_only && i < sg.n) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (part + u * PARTS < n_q) acc += exp(lg[u] - s_M[part + u * PARTS]) / s_Z[part + u * PARTS];
        for (int j = part + 4 * PARTS; j < n_q; j += PARTS) acc += exp(logits[g * n_q + j] - s_M[j]) / s_Z[j];
    }
    if (PARTS > 1) {
        if (part > 0) s_acc[part - 1][tok] = acc;
        __syncthreads();
        if (part > 0) return;
#pragma unroll
        for (int k = 0; k + 1 < PARTS; ++k) acc += s_acc[k][tok];
    }
    if (i >= sg.n) return;
    const double p = norm_only ? 1.0 / (double)sg.n : acc / (double)n_q;
    scores[g] = (float)((sg.flags & PACT_FLAG_SCORE_NO_NORM) ? p : hn * p);
}

// ------------------------------------------------------------------------------------------
// Eq. 3/4, one workgroup of 1024 per sample, on the finished fp32 scores:
//   (a) the scores become order-preserving integer keys in LDS;
//   (b) exact radix select of the (m+1)-th smallest key, m = min(floor(lambda n), n-1);
//   (c) ordered compaction into the kept / pruned index lists.
// (Finishing the scores here as well - one launch fewer - was slower: one compute unit then
// evaluates all n * n_q fp64 exponentials.)
// Dynamic LDS: n_max * 4 bytes.
__device__ __forceinline__ uint32_t ordered_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(1024) void score_prune_kernel(Batch bt, const float* __restrict__ scores,
                                                           uint64_t* __restrict__ adj,
                                                           int32_t* __restrict__ kept_idx,
                                                           int32_t* __restrict__ pruned_idx,
                                                           pact_report* __restrict__ rep) {
    extern __shared__ uint32_t s_key[];
    __shared__ int s_hist[256 * 16];
    __shared__ int s_bin[256];
    __shared__ int s_sel[2][2];
    __shared__ int s_wtot[16];
    __shared__ int s_odd[2];             // scores next to the threshold without being equal to it; non-finite scores
    __shared__ uint32_t s_mm[2][16], s_cand[64];
    __shared__ int s_ncand;
    const int b = blockIdx.x;
    const Seg sg = bt.s[b];
    const int n = sg.n;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const float* s = scores + sg.base;

    // this thread's first keys stay in registers for the select (its passes then issue their
    // histogram updates back to back instead of waiting for an LDS read before each)
    constexpr int KREG = 8;
    uint32_t kreg[KREG];
    {
        float sv[KREG];
#pragma unroll
        for (int u = 0; u < KREG; ++u) sv[u] = (tid + 1024 * u < n) ? s[tid + 1024 * u] : 0.0f;   // all in flight
#pragma unroll
        for (int u = 0; u < KREG; ++u) {
            kreg[u] = ordered_key(sv[u]);
            if (tid + 1024 * u < n) s_key[tid + 1024 * u] = kreg[u];
        }
        for (int i = tid + 1024 * KREG; i < n; i += 1024) s_key[i] = ordered_key(s[i]);
        __syncthreads();
    }

    const int m_rank = prune_rank(sg.lambda, n);
    int k = m_rank;
    uint32_t prefix = 0, mask = 0;
    // Selection in one histogram where that works: the keys of a sample share their leading bits
    // (scores of one image lie within a few binades), so the 4096 bins are laid over the range the
    // keys actually span, [smallest, largest]; the bin that holds rank k then has a handful of keys,
    // and one wavefront finds the wanted one among them by counting.  More than 64 keys in that bin
    // (ties, non-finite values that stretch the range): the radix select below does the whole job.
    bool selected = false;
    {
        uint32_t kmin = 0xFFFFFFFFu, kmax = 0u;
#pragma unroll
        for (int r = 0; r < KREG; ++r)
            if (tid + 1024 * r < n) { kmin = min(kmin, kreg[r]); kmax = max(kmax, kreg[r]); }
        for (int i = tid + 1024 * KREG; i < n; i += 1024) { const uint32_t u = s_key[i]; kmin = min(kmin, u); kmax = max(kmax, u); }
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, sft, 64));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, sft, 64));
        }
        if (lane == 0) { s_mm[0][wave] = kmin; s_mm[1][wave] = kmax; }
        for (int i = tid; i < 256 * 16; i += 1024) s_hist[i] = 0;
        if (tid == 0) s_ncand = 0;
        __syncthreads();
        kmin = s_mm[0][lane & 15];
        kmax = s_mm[1][lane & 15];
#pragma unroll
        for (int sft = 8; sft >= 1; sft >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, sft, 64));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, sft, 64));
        }
        const uint32_t range = kmax - kmin;
        const int nbits = range ? 32 - __builtin_clz(range) : 0;
        const int bshift = nbits > 12 ? nbits - 12 : 0;                  // (key - kmin) >> bshift < 4096
#pragma unroll
        for (int r = 0; r < KREG; ++r)
            if (tid + 1024 * r < n) atomicAdd(&s_hist[(kreg[r] - kmin) >> bshift], 1);
        for (int i = tid + 1024 * KREG; i < n; i += 1024) atomicAdd(&s_hist[(s_key[i] - kmin) >> bshift], 1);
        __syncthreads();
        // exclusive scan over the bins, four per thread
        const int c0 = s_hist[4 * tid], c1 = s_hist[4 * tid + 1], c2 = s_hist[4 * tid + 2], c3 = s_hist[4 * tid + 3];
        const int loc = c0 + c1 + c2 + c3;
        const int inc = wave_scan_incl_i32(loc);
        if (lane == 63) s_wtot[wave] = inc;
        __syncthreads();
        int e = inc - loc;
        for (int w = 0; w < wave; ++w) e += s_wtot[w];
        {
            const int c[4] = {c0, c1, c2, c3};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (k >= e && k < e + c[t]) { s_sel[0][0] = 4 * tid + t; s_sel[0][1] = k - e; s_sel[1][0] = c[t]; }
                e += c[t];
            }
        }
        __syncthreads();
        const int sel = s_sel[0][0], kk = s_sel[0][1], ncand = s_sel[1][0];
        if (ncand <= 64) {                                                   // (uniform)
#pragma unroll
            for (int r = 0; r < KREG; ++r)
                if (tid + 1024 * r < n && (int)((kreg[r] - kmin) >> bshift) == sel) s_cand[atomicAdd(&s_ncand, 1)] = kreg[r];
            for (int i = tid + 1024 * KREG; i < n; i += 1024) {
                const uint32_t u = s_key[i];
                if ((int)((u - kmin) >> bshift) == sel) s_cand[atomicAdd(&s_ncand, 1)] = u;
            }
            __syncthreads();
            if (wave == 0) {
                const uint32_t v = lane < ncand ? s_cand[lane] : 0xFFFFFFFFu;
                int below = 0, equal = 0;
                for (int j = 0; j < ncand; ++j) {
                    const uint32_t u = s_cand[j];
                    below += u < v;
                    equal += u == v;
                }
                if (lane < ncand && below <= kk && kk < below + equal) s_mm[0][0] = v;   // (the same value from every lane that qualifies)
            }
            __syncthreads();
            prefix = s_mm[0][0];
            selected = true;
        }
        __syncthreads();                   // (s_hist, s_sel and s_wtot are used again below)
    }
    if (!selected) {
    // Radix select, 8 bits per pass from the top.  Scores of one image share their leading bits,
    // so a plain histogram would serialise thousands of atomics on a handful of LDS words: every
    // bin has 16 copies (one per lane & 15, in 16 different banks), summed after the pass.
    for (int i = tid; i < 256 * 16; i += 1024) s_hist[i] = 0;
    __syncthreads();
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
#pragma unroll
        for (int r = 0; r < KREG; ++r) {
            const uint32_t u = kreg[r];
            if (tid + 1024 * r < n && (u & mask) == prefix)
                atomicAdd(&s_hist[(((u >> shift) & 255) << 4) + (lane & 15)], 1);
        }
        for (int i = tid + 1024 * KREG; i < n; i += 1024) {
            const uint32_t u = s_key[i];
            if ((u & mask) == prefix) atomicAdd(&s_hist[(((u >> shift) & 255) << 4) + (lane & 15)], 1);
        }
        __syncthreads();
        if (tid < 256) {                   // sum the 16 copies of a bin and leave them cleared for the next pass
            int t = 0;
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                const int a = (tid << 4) + ((c + tid) & 15);   // (rotated: spreads the banks)
                t += s_hist[a];
                s_hist[a] = 0;
            }
            s_bin[tid] = t;
        }
        __syncthreads();
        if (tid < 64) {
            const int c0 = s_bin[4 * tid], c1 = s_bin[4 * tid + 1];
            const int c2 = s_bin[4 * tid + 2], c3 = s_bin[4 * tid + 3];
            const int loc = c0 + c1 + c2 + c3;
            const int inc = wave_scan_incl_i32(loc);
            int e = inc - loc;   // keys with a smaller digit
            const int c[4] = {c0, c1, c2, c3};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (k >= e && k < e + c[t]) { s_sel[pass & 1][0] = 4 * tid + t; s_sel[pass & 1][1] = k - e; }
                e += c[t];
            }
        }
        __syncthreads();                   // (s_sel alternates, so no barrier is needed after reading it)
        prefix |= (uint32_t)s_sel[pass & 1][0] << shift;
        mask |= 255u << shift;
        k = s_sel[pass & 1][1];
    }
    }
    const uint32_t tau = prefix;

    // Ordered split (Eq. 3 / 4): wavefront w owns a contiguous range of tokens; a ballot per 64
    // tokens gives each its place, so both index lists are written in coalesced runs.
    const int per_wave = ((n + 15) / 16 + 63) / 64 * 64;
    const int i0 = min(n, wave * per_wave), i1 = min(n, i0 + per_wave);
    int cnt = 0;
    for (int i = i0; i < i1; i += 64) {
        const int t = i + lane;
        cnt += __popcll(__ballot(t < i1 && s_key[t] >= tau));
    }
    if (lane == 0) s_wtot[wave] = cnt;
    if (tid == 0) { s_odd[0] = 0; s_odd[1] = 0; }
    __syncthreads();
    // the threshold as a score again (inverse of ordered_key), for the two counters of the report
    const float tau_f = __uint_as_float((tau & 0x80000000u) ? (tau & 0x7FFFFFFFu) : ~tau);
    const double tau_band = 1e-6 * fabs((double)tau_f);
    int n_near = 0, n_bad = 0;
    int kp = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
        if (w < wave) kp += s_wtot[w];
        total += s_wtot[w];
    }
    int32_t* ko = kept_idx + sg.base;
    int32_t* po = pruned_idx + sg.base;
    for (int i = i0; i < i1; i += 64) {
        const int t = i + lane;
        const bool in = t < i1;
        const uint32_t key = in ? s_key[t] : tau;
        const bool keep = in && key >= tau;
        const uint64_t m = __ballot(keep);
        const int below = __popcll(m & ((1ull << lane) - 1ull));
        if (keep) ko[kp + below] = t;
        else if (in) po[t - (kp + below)] = t;
        kp += __popcll(m);
        const float f = __uint_as_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
        n_near += __popcll(__ballot(key != tau && fabs((double)f - (double)tau_f) <= tau_band));
        n_bad += __popcll(__ballot(in && !isfinite(f)));
    }
    if (lane == 0 && (n_near | n_bad)) { atomicAdd(&s_odd[0], n_near); atomicAdd(&s_odd[1], n_bad); }
    __syncthreads();
    if (tid == 0) {
        rep[b].n_kept = total;
        rep[b].n_pruned = n - total;
        rep[b].score_near_ties = s_odd[0];
        rep[b].nonfinite_seen = s_odd[1];
    }
    // Scores tied at the threshold: more tokens are kept than the n - m whose bitmap rows and
    // words were cleared along with the key norms; clear what the clustering will use.
    if (adj && total > n - m_rank) {
        uint64_t* rows = adj + (size_t)b * bt.n_max * bt.W;
        const int Wq = (total + 63) >> 6;
        for (int r = wave; r < total; r += 16)
            for (int w = lane; w < Wq; w += 64) rows[(size_t)r * bt.W + w] = 0ull;
    }
}

// ------------------------------------------------------------------------------------------
static hipError_t raise_lds_limit(const void* fn, size_t bytes) {
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int KDT>
static int launch_prep_q(const Batch& bt, const PrepArgs& a, pact_dtype q_dt, dim3 grid, hipStream_t st) {
    if (q_dt == PACT_BF16)
        PACT_LAUNCH("prep", (prep_kernel<KDT, PACT_BF16>), grid, dim3(256), st, bt, a);
    else
        PACT_LAUNCH("prep", (prep_kernel<KDT, PACT_F32>), grid, dim3(256), st, bt, a);
    return PACT_OK;
}

int launch_prep(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                const void* q, pact_dtype q_dt, int32_t qcols, pact_report* rep, int32_t* cluster_id,
                int32_t* cluster_counts, int mode, const int32_t* n_idx_dev, hipStream_t st) {
    PrepArgs a;
    a.keys = (const char*)keys; a.dk = dk;
    a.q = (const char*)q; a.qcols = qcols;
    a.nn = w.nn; a.rinv = w.rinv; a.adj = w.adj; a.qg_part = w.qg_part;
    a.status = w.status; a.ident = w.ident; a.near_cnt = w.near_cnt; a.tie_cnt = w.tie_cnt;
    a.rep = rep; a.cluster_id = cluster_id; a.cluster_counts = cluster_counts; a.n_idx_dev = n_idx_dev;
    a.zeros = w.zeros; a.ksplit = w.ksplit;
    a.mode = mode; a.n_key_blocks = keys ? (bt.n_max + 3) / 4 : 0;
    a.n_q_blocks = q ? QG_CHUNKS * ((qcols + 1023) / 1024) : 0;
    dim3 grid(a.n_key_blocks + a.n_q_blocks, bt.B);
    return (k_dt == PACT_BF16) ? launch_prep_q<PACT_BF16>(bt, a, q_dt, grid, st)
                               : launch_prep_q<PACT_F32>(bt, a, q_dt, grid, st);
}

// Share (in 256ths) of the hidden-state norms that go with the global query; the rest goes with
// the logits.  For one image the norms are best left in one launch (split, the two launches
// together took 1.5 us longer); for large batches, whose logits launch is long enough to hide
// part of the read behind its arithmetic, a 144 : 112 split was 8 us (1.5%) faster on 8 x 6272.
static int hnorm_share(const Batch& bt) { return bt.total >= 20000 ? 144 : 256; }

template <int HDT>
static int launch_qglobal_hnorm(const Batch& bt, const Ws& w, const ScoreIn& in, hipStream_t st) {
    const int qcols = in.n_q * in.d_h;
    const int nq_blocks = in.q_per_token ? (qcols + 63) / 64 : (qcols + 1023) / 1024;
    const int share = hnorm_share(bt);
    const int stream = hidden_streams(bt.total, in.h, Elem<HDT>::BYTES) ? 1 : 0;
    dim3 grid(nq_blocks + (hnorm_split(bt.n_max, share) + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG, bt.B);
    const int kbytes = in.k_dt == PACT_BF16 ? 2 : 4;
    QgLayout lay = {0, in.n_kv, in.d_h, in.d_h * kbytes / 16, 16 / kbytes};
    if (logits_grouped(in.n_kv, in.n_q, in.d_h, kbytes)) lay.rep = in.n_q / in.n_kv;
    if (in.q_dt == PACT_BF16)
        PACT_LAUNCH("qglobal_hnorm", (qglobal_hnorm_kernel<HDT, PACT_BF16>), grid, dim3(1024), st, bt, qcols,
                    in.q_per_token ? 1 : 0, nq_blocks, lay, w.qg_part, (const char*)in.q, w.qg, (const char*)in.hidden,
                    in.h, w.hnorm, share, stream);
    else
        PACT_LAUNCH("qglobal_hnorm", (qglobal_hnorm_kernel<HDT, PACT_F32>), grid, dim3(1024), st, bt, qcols,
                    in.q_per_token ? 1 : 0, nq_blocks, lay, w.qg_part, (const char*)in.q, w.qg, (const char*)in.hidden,
                    in.h, w.hnorm, share, stream);
    return PACT_OK;
}

template <int HDT>
static int launch_logits_hnorm(const Batch& bt, const Ws& w, const ScoreIn& in, hipStream_t st) {
    const int n_logit_blocks = (bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    const int share = hnorm_share(bt);
    const int stream = hidden_streams(bt.total, in.h, Elem<HDT>::BYTES) ? 1 : 0;
    // tokens past the split: n - split(n) <= n - floor(n * share / 256), which grows with n
    const int rest = bt.n_max - ((bt.n_max * share) >> 8);
    dim3 grid(n_logit_blocks + (rest + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG, bt.B);
    const bool grouped = logits_grouped(in.n_kv, in.n_q, in.d_h, in.k_dt == PACT_BF16 ? 2 : 4);
#define PACT_LOGITS(KDT, G)                                                                                          \
    PACT_LAUNCH("score_logits", (score_logits_kernel<KDT, HDT, G>), grid, dim3(1024), st, bt,                        \
                (const char*)in.keys_pre, in.n_kv, in.d_h, in.n_q, w.qg, w.logits, w.sm_part, n_logit_blocks,        \
                (const char*)in.hidden, in.h, w.hnorm, share, stream)
    if (in.k_dt == PACT_BF16) { if (grouped) PACT_LOGITS(PACT_BF16, true); else PACT_LOGITS(PACT_BF16, false); }
    else { if (grouped) PACT_LOGITS(PACT_F32, true); else PACT_LOGITS(PACT_F32, false); }
#undef PACT_LOGITS
    return PACT_OK;
}

// Scores for every sample.  The per-token query pass (Eq. 1 pass 1) must already have run
// (launch_prep with q != nullptr) when in.q_per_token is set.
int launch_score(const Batch& bt, const Ws& w, const ScoreIn& in, hipStream_t st) {
    int rc = (in.h_dt == PACT_BF16) ? launch_qglobal_hnorm<PACT_BF16>(bt, w, in, st)
                                    : launch_qglobal_hnorm<PACT_F32>(bt, w, in, st);
    if (rc) return rc;
    return (in.h_dt == PACT_BF16) ? launch_logits_hnorm<PACT_BF16>(bt, w, in, st)
                                  : launch_logits_hnorm<PACT_F32>(bt, w, in, st);
}

int launch_score_only(const Batch& bt, const Ws& w, int n_q, float* scores, hipStream_t st) {
    // Many query heads: the combine once per sample in a launch of its own (its result in the
    // array of the query's chunk sums, which the global query has replaced by now), and sixteen
    // threads per token.
    if (n_q > 8) {
        double* mz = w.qg_part;
        PACT_LAUNCH("softmax_combine", softmax_combine_kernel, dim3(n_q, bt.B), dim3(64), st, bt, n_q, w.sm_part, mz);
        PACT_LAUNCH("score_final", (score_final_kernel<64, 16>), dim3((bt.n_max + 63) / 64, bt.B), dim3(1024), st, bt,
                    n_q, w.logits, w.hnorm, w.sm_part, (const double*)mz, scores);
    } else {
        PACT_LAUNCH("score_final", (score_final_kernel<256, 1>), dim3((bt.n_max + 255) / 256, bt.B), dim3(256), st, bt,
                    n_q, w.logits, w.hnorm, w.sm_part, (const double*)nullptr, scores);
    }
    return PACT_OK;
}

// Splits the finished scores of every sample (Eq. 3 / 4).
// adj: the samples' neighbour bitmaps as launch_prep(INIT_REDUCE) left them, or nullptr when no
// clustering follows.
int launch_score_prune(const Batch& bt, const float* scores, uint64_t* adj, int32_t* kept_idx,
                       int32_t* pruned_idx, pact_report* rep, hipStream_t st) {
    const size_t lds = (size_t)((bt.n_max + 63) / 64 * 64) * sizeof(uint32_t);
    static size_t raised = 0;
    if (lds > 48 * 1024 && lds > raised) {
        if (raise_lds_limit((const void*)score_prune_kernel, lds) != hipSuccess) return PACT_ERR_HIP;
        raised = lds;
    }
    PACT_LAUNCH_SHMEM("score_prune", score_prune_kernel, dim3(bt.B), dim3(1024), lds, st, bt, scores, adj,
                      kept_idx, pruned_idx, rep);
    return PACT_OK;
}

}  // namespace pact

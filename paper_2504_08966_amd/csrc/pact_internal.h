// Internal declarations shared by the HIP sources of libpact (gfx950 only).
// Paper notation: n tokens, q kept tokens ("p-space" = position of a kept token in the
// ascending kept list), C centres, d_c cutoff, d_n density normaliser, alpha recovery factor.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "pact.h"
#include "pact_measure.h"

namespace pact {

// ---------------------------------------------------------------------------------------
// Batch descriptor: passed BY VALUE as a kernel argument (no device copy to manage).
struct Seg {
    int32_t base;     // first row of this sample in every token-indexed tensor
    int32_t n;        // tokens in this sample
    float lambda, d_c, d_n, alpha;
    int32_t fallback_T;
    uint32_t flags;
};
struct Batch {
    int32_t B;        // samples in this launch (<= PACT_MAX_BATCH)
    int32_t n_max;    // max tokens of one sample; pitch of per-sample workspace arrays
    int32_t W;        // 64-bit words per bitmap row = ceil(n_max / 64)
    int32_t total;    // tokens over all samples
    Seg s[PACT_MAX_BATCH];
};

// ---------------------------------------------------------------------------------------
// Workspace layout.  Offsets in bytes from the 256-aligned workspace base.
constexpr int QG_CHUNKS = 512;        // row chunks of the global-query column sum
constexpr int SCORE_TOK_PER_WG = 16;  // tokens (= wavefronts) per workgroup in the logits kernel
constexpr int PRED_CAP = 64;          // 16-bit slots per kept token: slot 0 = count, then up to 63 preceding neighbours
constexpr int GRAM_RHO_ROWS = 128;    // kept rows summed into one row of the density partials
constexpr int GRAM_MAX_WORKGROUPS = 256; // workgroups of 8 wavefronts per sample in a Gram pass (one per CU)
constexpr int NEAR_CAP = 1 << 16;     // near-threshold pairs kept for fp64 re-evaluation, per sample
constexpr uint32_t NEAR_MIRROR = 0x80000000u;   // flag in a listed pair's row: the pair (col, row) is meant as well
constexpr uint32_t ST_UNKNOWN = 0, ST_CENTER = 1, ST_NOT = 2;
constexpr int RHO_RECHECK_MAX = PACT_MAX_RHO_RECHECK;   // tokens per sample whose density is evaluated again in fp64
constexpr int RHO_RECHECK_CHUNK = 64;                   // kept tokens per partial sum of such an evaluation
// Clusters of at least MERGE_BIG rows are merged first (a cluster of 30 rows takes several times
// as long as one of 2, and started in the last turn it alone would be the end of the kernel).
// The first MERGE_SLOTS members of a cluster are noted as they join it (one 128-byte line per
// cluster), so that the merge of a full reduction needs no pass that builds member lists.
constexpr int MERGE_BIG = 12, MERGE_SLOTS = 32;
constexpr int RESOLVE_LDS_TOKENS = 8192;   // samples up to this size keep the work lists of the centre rounds in LDS
constexpr int32_t OVERFLOW_NEAR_LIST = 1, OVERFLOW_RHO_RECHECK = 2;   // bits of pact_report.refine_overflow

struct WsLayout {
    size_t qg_part, qg, logits, hnorm, sm_part;        // score
    size_t nn, rinv;                                   // key norms, per token (global row index)
    size_t ident;                                      // identity index list (idx == NULL)
    size_t adj;                                        // [B][n_max][W] u64: rows < q adjacency; from row q on: candidate words [Wc][n_pruned]
    size_t cbest;                                      // [B][W][n_max] f32: largest cosine per (group of 64 centres, pruned token)
    size_t rho_part;                                   // [B][W][n_max] f64
    size_t rho, rank, status, cnum, cmask;             // per sample, pitch n_max (cmask: W)
    size_t preds, heads;                               // [B][n_max][PRED_CAP] u16, [B][n_max] 4 x u16 (count + first 3)
    size_t ksplit;                                     // [total][3][dk rounded up to 8] bf16: fp32 clustering keys as three bf16 parts
    size_t near_list, near_cnt, stat;                  // refine list, counter; [B][workgroups * 8] most negative density exponent seen
    size_t tie_list, tie_cnt;                          // [B][RHO_RECHECK_MAX] kept positions whose density is re-evaluated; [B][4]: count, ticket
    size_t rho_fix;                                    // [B][min(RHO_RECHECK_MAX, n_max)][ceil(n_max / RHO_RECHECK_CHUNK)][2] f64 partial sums of those
    size_t offsets, members, big;                      // merge CSR (global row index); ids of the large clusters
    size_t slots;                                      // [total][MERGE_SLOTS] i32: first members of each cluster, in the order they joined
    size_t worklist;                                   // [B][2][n_max] 8-byte entries: the centre rounds' work lists of samples too large for the LDS
    size_t zeros;                                      // 256 zero bytes
    size_t total;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
__host__ __device__ inline int64_t rho_fix_tokens(int64_t n_max) { return n_max < RHO_RECHECK_MAX ? n_max : RHO_RECHECK_MAX; }
__host__ __device__ inline int64_t rho_fix_chunks(int64_t n_max) { return (n_max + RHO_RECHECK_CHUNK - 1) / RHO_RECHECK_CHUNK; }

// dk: width of the clustering keys (0 for calls that run no Gram pass); k_dt: their type (only
// fp32 keys have a three-part bf16 copy)
inline WsLayout make_layout(int64_t n_max, int64_t B, int64_t total, int64_t qcols, int64_t n_q, int64_t dk,
                            int k_dt) {
    WsLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const int64_t W = (n_max + 63) / 64;
    const int64_t smwg = (n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    L.qg_part = take(sizeof(double) * B * QG_CHUNKS * qcols);
    L.qg = take(sizeof(double) * B * qcols);
    L.logits = take(sizeof(double) * total * n_q);
    L.hnorm = take(sizeof(double) * total);
    L.sm_part = take(sizeof(double) * B * smwg * n_q * 2);
    L.nn = take(sizeof(double) * total);
    L.rinv = take(sizeof(float) * total);
    L.ident = take(sizeof(int32_t) * total);
    L.adj = take(sizeof(uint64_t) * B * n_max * W);
    L.cbest = take(sizeof(float) * B * W * n_max);
    L.rho_part = take(sizeof(double) * B * W * n_max);
    L.rho = take(sizeof(double) * B * n_max);
    L.rank = take(sizeof(int32_t) * B * n_max);
    L.status = take(sizeof(uint32_t) * B * n_max);
    L.cnum = take(sizeof(int32_t) * B * n_max);
    L.cmask = take(sizeof(uint64_t) * B * W);
    L.preds = take(sizeof(uint16_t) * B * n_max * PRED_CAP);
    L.heads = take(sizeof(uint16_t) * 4 * B * n_max);
    L.near_list = take(sizeof(uint32_t) * 2 * B * NEAR_CAP);
    L.near_cnt = take(sizeof(int32_t) * 2 * B);   // per sample: list slots taken, ordered pairs they stand for
    L.stat = take(sizeof(uint32_t) * B * GRAM_MAX_WORKGROUPS * 8);   // one word per wavefront of the density pass
    L.tie_list = take(sizeof(int32_t) * B * RHO_RECHECK_MAX);
    L.tie_cnt = take(sizeof(int32_t) * 4 * B);
    L.rho_fix = take(sizeof(double) * 2 * B * rho_fix_tokens(n_max) * rho_fix_chunks(n_max));
    L.offsets = take(sizeof(int32_t) * (total + B));
    L.members = take(sizeof(int32_t) * total);
    L.big = take(sizeof(int32_t) * total);
    L.slots = take(sizeof(int32_t) * total * MERGE_SLOTS);
    L.worklist = take(n_max > RESOLVE_LDS_TOKENS ? 16 * B * n_max : 0);
    L.zeros = take(256);
    L.ksplit = take(k_dt == PACT_F32 ? sizeof(uint16_t) * 3 * total * ((dk + 7) / 8 * 8) : 0);   // planes padded to whole 16-byte chunks
    L.total = off;
    return L;
}

// Resolved device pointers for one call.
struct Ws {
    double* qg_part; double* qg; double* logits; double* hnorm; double* sm_part;
    double* nn; float* rinv; int32_t* ident;
    uint64_t* adj; float* cbest; double* rho_part; double* rho; int32_t* rank; uint32_t* status;
    int32_t* cnum; uint64_t* cmask; uint16_t* preds; uint2* heads; uint32_t* near_list; int32_t* near_cnt; uint32_t* stat;
    int32_t* tie_list; int32_t* tie_cnt; double* rho_fix;
    int32_t* offsets; int32_t* members; int32_t* big; int32_t* slots; uint2* worklist; uint32_t* zeros; uint16_t* ksplit;
};

inline Ws resolve(void* base, const WsLayout& L) {
    char* p = (char*)base;
    Ws w;
    w.qg_part = (double*)(p + L.qg_part); w.qg = (double*)(p + L.qg);
    w.logits = (double*)(p + L.logits); w.hnorm = (double*)(p + L.hnorm);
    w.sm_part = (double*)(p + L.sm_part);
    w.nn = (double*)(p + L.nn); w.rinv = (float*)(p + L.rinv); w.ident = (int32_t*)(p + L.ident);
    w.adj = (uint64_t*)(p + L.adj); w.cbest = (float*)(p + L.cbest); w.rho_part = (double*)(p + L.rho_part);
    w.rho = (double*)(p + L.rho); w.rank = (int32_t*)(p + L.rank);
    w.status = (uint32_t*)(p + L.status); w.cnum = (int32_t*)(p + L.cnum);
    w.preds = (uint16_t*)(p + L.preds); w.heads = (uint2*)(p + L.heads);
    w.cmask = (uint64_t*)(p + L.cmask); w.near_list = (uint32_t*)(p + L.near_list);
    w.near_cnt = (int32_t*)(p + L.near_cnt); w.stat = (uint32_t*)(p + L.stat);
    w.tie_list = (int32_t*)(p + L.tie_list); w.tie_cnt = (int32_t*)(p + L.tie_cnt);
    w.rho_fix = (double*)(p + L.rho_fix);
    w.offsets = (int32_t*)(p + L.offsets); w.big = (int32_t*)(p + L.big);
    w.members = (int32_t*)(p + L.members); w.slots = (int32_t*)(p + L.slots); w.worklist = (uint2*)(p + L.worklist); w.zeros = (uint32_t*)(p + L.zeros);
    w.ksplit = (uint16_t*)(p + L.ksplit);
    return w;
}

// ---------------------------------------------------------------------------------------
// Kernel launch bookkeeping (optional per-kernel events).
void prof_begin(const char* name, hipStream_t s);
void prof_end(hipStream_t s);

#define PACT_LAUNCH(name, kernel, grid, block, stream, ...)                        \
    do {                                                                           \
        ::pact::prof_begin(name, stream);                                          \
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);           \
        ::pact::prof_end(stream);                                                  \
        if (hipGetLastError() != hipSuccess) return PACT_ERR_HIP;                  \
    } while (0)

#define PACT_LAUNCH_SHMEM(name, kernel, grid, block, shmem, stream, ...)          \
    do {                                                                           \
        ::pact::prof_begin(name, stream);                                          \
        hipLaunchKernelGGL(kernel, grid, block, shmem, stream, __VA_ARGS__);       \
        ::pact::prof_end(stream);                                                  \
        if (hipGetLastError() != hipSuccess) return PACT_ERR_HIP;                  \
    } while (0)

// ---------------------------------------------------------------------------------------
// Stage launchers (host).  Each enqueues on `st` and returns a pact_status.
struct ScoreIn {
    const void* hidden; pact_dtype h_dt; int32_t h;
    const void* keys_pre; pact_dtype k_dt; int32_t n_kv, d_h;
    const void* q; pact_dtype q_dt; int32_t q_per_token; int32_t n_q;   // q_per_token: 1 = [total, ..], 0 = [B, ..]
};

// First kernel of every call: key norms, cleared bitmap rows, per-token initial state and
// (q != nullptr) the first pass of Eq. 1.
int launch_prep(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                const void* q, pact_dtype q_dt, int32_t qcols, pact_report* rep, int32_t* cluster_id,
                int32_t* cluster_counts, int mode, const int32_t* n_idx_dev, hipStream_t st);
int launch_score(const Batch& bt, const Ws& w, const ScoreIn& in, hipStream_t st);
int launch_score_only(const Batch& bt, const Ws& w, int n_q, float* scores, hipStream_t st);
int launch_score_prune(const Batch& bt, const float* scores, uint64_t* adj, int32_t* kept_idx,
                       int32_t* pruned_idx, pact_report* rep, hipStream_t st);
// want_stat: also record the largest key distance; *stat_words = words per sample the kernel
// wrote to w.stat (0 if not wanted), to be handed to launch_centres.
int launch_gram_density(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                        const int32_t* idx, pact_report* rep, bool want_stat, int* stat_words, hipStream_t st);
// (diagnostic) the map of workgroup slots to samples that the Gram passes of a batch use
int plan_gram_workgroups(const int32_t* tiles, int32_t batch, uint16_t* wg_map, uint16_t* wg_count);
int launch_centres(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                   const int32_t* idx, int32_t* center_idx, int32_t* cluster_id,
                   int32_t* cluster_counts, pact_report* rep, double* rho_opt, int32_t* rank_opt,
                   int stat_words, bool assign_now, hipStream_t st);
int launch_reincorporate(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                         const int32_t* pruned_idx, const int32_t* center_idx, int32_t* cluster_id,
                         int32_t* cluster_counts, pact_report* rep, bool count_totals,
                         const int32_t* kept_idx, hipStream_t st);
int launch_merge(const Batch& bt, const Ws& w, const void* hidden, pact_dtype h_dt, int32_t h,
                 const int32_t* cluster_id, const int32_t* center_idx, pact_report* rep,
                 void* merged, pact_dtype out_dt, int32_t* cluster_counts, bool recount,
                 hipStream_t st);

int launch_handoff(const Batch& bt, const int32_t* center_idx, const int32_t* cluster_counts,
                   const pact_report* rep, const int32_t* positions, int32_t* positions_out,
                   float* log_weight, hipStream_t st);

// init modes
// m of Eq. 3 / 4: the threshold is the (m+1)-th smallest score, m = min(floor(lambda n), n-1);
// the m tokens below it are pruned, all of them when no other score equals the threshold.
__host__ __device__ inline int prune_rank(float lambda, int n) {
    int m = (int)floor((double)lambda * (double)n);
    if (m > n - 1) m = n - 1;
    return m < 0 ? 0 : m;
}

enum { INIT_REDUCE = 0, INIT_DBDPC_ALL = 1, INIT_DBDPC_SUBSET = 2, INIT_REINC = 3, INIT_SCORE = 4 };

// Worst-case rounding error of an fp32-accumulated matrix-core cosine of two dk-long rows, plus
// slack for the scaling multiplies and, for fp32 keys, for what their three-part bf16 form
// leaves out (below 2^-22 of |u||v|); decisions closer than this to a threshold are re-made in fp64.
inline double cos_margin(int dk) { return (double)(dk + 16) * (1.0 / 8388608.0) + 2.5e-6; }

// Internal element type of the Gram kernel for fp32 keys: each value as the sum of three bf16
// parts (hi + mid + lo, 24 significant bits), in three planes per token.
enum { PACT_F32X3 = 2 };

}  // namespace pact

// ---------------------------------------------------------------------------------------
// Device helpers
#ifdef __HIPCC__
namespace pact {

// LDS-qualified pointer types: accesses through them compile to ds_* instructions even when
// the pointer travels through function arguments (a generic pointer would give flat_*).
typedef __attribute__((address_space(3))) volatile unsigned char lds_vu8;
typedef __attribute__((address_space(3))) int lds_i32;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) uint16_t lds_u16;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// Counts read back from a device-side report are clamped to the sample size, so that a report
// the caller never initialised cannot send a kernel out of bounds.
__device__ __forceinline__ int clamp_count(int v, int n) { return v < 0 ? 0 : (v > n ? n : v); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;   // NaN stays NaN
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// 16 bytes of a row -> up to 8 doubles.  EPL = elements per 16-byte load.
template <int DT> struct Elem;
template <> struct Elem<PACT_BF16> {
    static constexpr int EPL = 8;
    static constexpr int BYTES = 2;
    __device__ static __forceinline__ void widen(const uint4& v, double* out) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = (double)__uint_as_float(w[i] << 16);
            out[2 * i + 1] = (double)__uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
    __device__ static __forceinline__ void widenf(const uint4& v, float* out) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
    }
};
template <> struct Elem<PACT_F32> {
    static constexpr int EPL = 4;
    static constexpr int BYTES = 4;
    __device__ static __forceinline__ void widen(const uint4& v, double* out) {
        out[0] = (double)__uint_as_float(v.x); out[1] = (double)__uint_as_float(v.y);
        out[2] = (double)__uint_as_float(v.z); out[3] = (double)__uint_as_float(v.w);
    }
    __device__ static __forceinline__ void widenf(const uint4& v, float* out) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y);
        out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    }
};

// Reductions over each group of `width` neighbouring lanes (a power of two), left in every lane
// of the group: lane l combines with lane l ^ 1, l ^ 2, ... in turn.  Inside a row of 16 lanes the
// partner's value comes through the data-parallel lane permutes of the vector unit (for a sum or
// a maximum a mirror image of the group of 8 or 16 serves as well as the exchange of its halves:
// the partner holds the same partial result, so the values are those of the exchange, bit for bit),
// beyond that through a shuffle; a shuffle of a double is two trips through the LDS crossbar, and
// 28 of them per wavefront were a quarter of the logits kernel with 28 query heads.
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v) {
    const int u = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(u, u, CTRL, 0xF, 0xF, true));
}
template <int CTRL> __device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)u, (int)(uint32_t)u, CTRL, 0xF, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp((int)(uint32_t)(u >> 32), (int)(uint32_t)(u >> 32), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_MIRROR = 0x140;   // quad_perm [1,0,3,2], [2,3,0,1], row_half_mirror, row_mirror
__device__ __forceinline__ double group_sum_f64(double v, int width) {
    if (width > 1) v += dpp_f64<DPP_XOR1>(v);
    if (width > 2) v += dpp_f64<DPP_XOR2>(v);
    if (width > 4) v += dpp_f64<DPP_HALF_MIRROR>(v);
    if (width > 8) v += dpp_f64<DPP_MIRROR>(v);
    for (int sft = 16; sft < width; sft <<= 1) v += __shfl_xor(v, sft, 64);
    return v;
}
template <int WIDTH> __device__ __forceinline__ double group_max_f64(double v) {
    static_assert(WIDTH == 8 || WIDTH == 16, "within a row of 16 lanes");
    v = fmax(v, dpp_f64<DPP_XOR1>(v));
    v = fmax(v, dpp_f64<DPP_XOR2>(v));
    v = fmax(v, dpp_f64<DPP_HALF_MIRROR>(v));
    if (WIDTH > 8) v = fmax(v, dpp_f64<DPP_MIRROR>(v));
    return v;
}
template <int WIDTH> __device__ __forceinline__ float group_sum_f32(float v) {
    static_assert(WIDTH == 8 || WIDTH == 16, "within a row of 16 lanes");
    v += dpp_f32<DPP_XOR1>(v);
    v += dpp_f32<DPP_XOR2>(v);
    v += dpp_f32<DPP_HALF_MIRROR>(v);
    if (WIDTH > 8) v += dpp_f32<DPP_MIRROR>(v);
    return v;
}
template <int WIDTH> __device__ __forceinline__ float group_max_f32(float v) {
    static_assert(WIDTH == 8 || WIDTH == 16, "within a row of 16 lanes");
    v = fmaxf(v, dpp_f32<DPP_XOR1>(v));
    v = fmaxf(v, dpp_f32<DPP_XOR2>(v));
    v = fmaxf(v, dpp_f32<DPP_HALF_MIRROR>(v));
    if (WIDTH > 8) v = fmaxf(v, dpp_f32<DPP_MIRROR>(v));
    return v;
}

// Inclusive prefix sum over the 64 lanes of a wavefront (all active), on the vector unit's lane
// permutes: shifts by 1, 2, 4 and 8 inside each row of 16, then lane 15 of rows 0 and 2 to rows 1
// and 3, then lane 31 to rows 2 and 3.  Six dependent vector instructions instead of six trips
// through the LDS crossbar.
__device__ __forceinline__ int wave_scan_incl_i32(int v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, false);     // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, false);     // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, false);     // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, false);     // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);     // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);     // row_bcast:31 -> rows 2, 3
    return v;
}
// value of lane 0 / lane 63 of a wavefront-wide register, as a scalar
__device__ __forceinline__ int lane0_of(int v) { return __builtin_amdgcn_readlane(v, 0); }
__device__ __forceinline__ int lane63_of(int v) { return __builtin_amdgcn_readlane(v, 63); }

// Over the whole wavefront (all 64 lanes active): neighbours first, inside the rows of 16 lanes through
// the lane permutes, then the four rows through two shuffles - 4 trips through the LDS crossbar instead
// of 12, which is half a microsecond in a wavefront that waits for the result.
__device__ __forceinline__ double wave_sum_f64(double v) {
    return group_sum_f64(v, 64);   // butterfly: every lane ends with the bit-identical total
}
__device__ __forceinline__ double wave_max_f64(double v) {
    v = group_max_f64<16>(v);
    v = fmax(v, __shfl_xor(v, 16, 64));
    return fmax(v, __shfl_xor(v, 32, 64));
}

// fp64 dot product of two rows of dk elements, computed by one full wavefront; the partition
// of elements over lanes and the reduction tree are fixed, so dot(a,b) of bit-identical rows
// equals dot(a,a) bit for bit.
template <int DT>
__device__ __forceinline__ double wave_dot64(const char* ra, const char* rb, int dk, int lane) {
    constexpr int EPL = Elem<DT>::EPL;
    double acc = 0.0;
    for (int e = lane * EPL; e < dk; e += 64 * EPL) {
        const uint4 va = *(const uint4*)(ra + (size_t)e * Elem<DT>::BYTES);
        const uint4 vb = *(const uint4*)(rb + (size_t)e * Elem<DT>::BYTES);
        double a[8], b[8];
        Elem<DT>::widen(va, a);
        Elem<DT>::widen(vb, b);
#pragma unroll
        for (int i = 0; i < EPL; ++i) acc = fma(a[i], b[i], acc);
    }
    return wave_sum_f64(acc);
}

// 16 bytes that this launch touches once: loads and stores with the streaming hint.  Used when a
// call's hidden states are larger than what the 256 MB last-level cache can keep between the norm
// pass and the merge anyway; for smaller calls the hint costs those later hits (one 7290-token
// image: +4 us per call with it, 8 videos of 6272 tokens: -30 us; batches of 2 to 6 such videos,
// 43 MiB each: +8, +4, -6, -13, -20 us, hence the 150 MiB).
inline bool hidden_streams(long total_tokens, int h, int elem_bytes) {
    return (double)total_tokens * (double)h * (double)elem_bytes > 150.0 * 1024.0 * 1024.0;
}
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_once16(const void* p) {
    const u32x4_t v = __builtin_nontemporal_load((const u32x4_t*)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_once16(void* p, uint4 w) {
    const u32x4_t v = {w.x, w.y, w.z, w.w};
    __builtin_nontemporal_store(v, (u32x4_t*)p);
}

// Eq. 5 in fp64 from a dot product and the two squared norms; zero vector -> cosine 0.
__device__ __forceinline__ double cos_dist64(double dot, double nna, double nnb) {
    const double den = sqrt(nna * nnb);
    const double c = den > 0.0 ? dot / den : 0.0;
    return fmin(fmax(1.0 - c, 0.0), 2.0);
}

}  // namespace pact
#endif

/*
 * pact.h - C ABI of the MI355X (gfx950) implementation of PACT's token-reduction step:
 * score and prune visual tokens (EUTI), cluster the survivors' keys (DBDPC), recover
 * pruned tokens that lie close to a centre, merge each cluster into one token.
 *
 * Paper: "PACT: Pruning and Clustering-Based Token Reduction for Faster Visual Language
 * Models" (arXiv 2504.08966).  Alg. 1 = EUTI, Alg. 2 = DBDPC, Alg. 3 = PACT, Alg. 4 =
 * recursive centre identification (appendix D); Eq. 1 global query, Eq. 2 score, Eq. 3/4
 * important / unimportant sets, Eq. 5 distance, Eq. 6 density, Eq. 8/9 recovery, Eq. 10 merge.
 *
 * Conventions shared by every entry point
 *  - Every pointer is a DEVICE pointer unless its comment says "host".  The caller owns all
 *    buffers.  The library never allocates or frees device memory and never synchronises:
 *    all work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default stream).
 *  - Tensors are row-major and contiguous; every row must start on a 16-byte boundary
 *    (PACT_ERR_ALIGN otherwise), which for contiguous rows means: base pointer 16-byte
 *    aligned and row bytes a multiple of 16.
 *  - Token indices written by the library are int32 and LOCAL to their sample (0..n-1).
 *  - Data-dependent counts (kept tokens, centres, ...) stay on the device, in pact_report;
 *    output buffers are sized by the caller for the worst case stated at each argument.
 *    The host may read the report after synchronising the stream itself.
 *  - Cluster ids are 0..C-1 in ascending order of the centre's token index, so `merged`
 *    rows and `center_idx` are in sequence order and the position id of merged row s is
 *    the caller's P[center_idx[s]] (Alg. 3 step 4).  cluster_id[i] = -1 means token i
 *    was pruned and not recovered.
 *  - Return value: PACT_OK, or an error code.  Every code except PACT_ERR_HIP comes from a
 *    check of the arguments on the host, made before anything is enqueued: no output was
 *    touched.  PACT_ERR_HIP means a launch failed part-way through a call: kernels of that
 *    call enqueued before it still run, and the outputs are then undefined.
 *  - Data anomalies that cannot be seen without reading device memory are not errors and are
 *    counted in pact_report: a zero-norm clustering key follows the rule below
 *    (zero_norm_seen); non-finite values (NaN, Inf) in the hidden states, keys or queries
 *    make the results unspecified - every index written still lies inside its sample - and
 *    are counted in nonfinite_seen.
 *  - `ws` is scratch of at least pact_workspace_bytes(...) bytes, 256-byte aligned.  Calls
 *    that share a workspace must be ordered on one stream.  Its contents on entry are
 *    arbitrary (every call initialises what it reads).
 *  - Cache use: a call whose hidden states are larger than 150 MiB reads them, and writes
 *    its merged rows, with the non-temporal hint (they would not stay in the 256 MB
 *    last-level cache anyway); smaller calls use plain loads and stores.  Results do not
 *    depend on this.
 *
 * Arithmetic (what "the same result as the definition" means here)
 *  - Scores (Eq. 2) are evaluated in fp64 and rounded once to fp32; the percentile split
 *    (Eq. 3/4) compares those fp32 values.
 *  - Distances (Eq. 5) that decide something (within d_c of a centre or not, nearest centre,
 *    within alpha*d_c or not) are evaluated in fp64 whenever the fp32 matrix-core value is
 *    closer to the threshold than its worst-case rounding error, and always for the final
 *    nearest-centre choice, so those decisions are the fp64 ones.
 *  - Densities (Eq. 6) are fp64 sums of fp32 terms exp2-evaluated from matrix-core cosines
 *    (bf16 keys as they are; fp32 keys as three bf16 parts per value, all 24 bits of them).
 *    The density order (Alg. 2) only matters between tokens within d_c of each other; where
 *    two such tokens have densities closer than a band of about fifty standard errors of
 *    that fp32 sum, both densities are evaluated again entirely in fp64 (Eq. 5 and Eq. 6 as
 *    written) and those decide (pact_report.rho_rechecked, rho_near_ties).
 *  - Ties: equal scores at the percentile are all kept; equal densities are processed in
 *    ascending token index; equal distances pick the centre with the lower token index.
 *  - A zero-norm key has cosine 0 (distance 1) to every other token; d_ii = 0.
 */
#ifndef PACT_H
#define PACT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PACT_OK = 0,
    PACT_ERR_NULL = 1,      /* a required pointer is NULL */
    PACT_ERR_SHAPE = 2,     /* a size is out of range or inconsistent */
    PACT_ERR_DTYPE = 3,     /* unknown pact_dtype */
    PACT_ERR_PARAM = 4,     /* lambda, d_c, d_n or alpha out of range */
    PACT_ERR_WORKSPACE = 5, /* ws is NULL, misaligned or too small */
    PACT_ERR_ALIGN = 6,     /* a tensor row is not 16-byte aligned */
    PACT_ERR_HIP = 7,       /* a HIP call failed while enqueueing */
    PACT_ERR_NOGPU = 8      /* no usable gfx950 device */
} pact_status;

typedef enum { PACT_F32 = 0, PACT_BF16 = 1 } pact_dtype;

/* Limits.  n: tokens of one sample; batch: samples per varlen call. */
#define PACT_MAX_TOKENS 32768
#define PACT_MAX_BATCH 64
#define PACT_MAX_QHEADS 64

/* Hyper-parameters of Alg. 3 (host memory).  The paper's defaults: d_n = 2, alpha = 1.5,
 * fallback_T = 10 (appendix D/E).  lambda in [0,1] is the fraction of tokens deemed
 * unimportant; d_c >= 0; d_n > 0; alpha >= 0.  fallback_T >= 0 is Alg. 4's threshold for
 * leaving its recursion to the sequential loop; here every round runs inside one workgroup
 * and gives the sequential loop's centres whatever the threshold, so the value is validated
 * and otherwise unused.
 * flags: bit 0 (PACT_FLAG_NO_MERGE) writes the centre token's hidden state instead of the
 * cluster mean (the paper's "no merging" ablation); bits 1 and 2 select the two ablations of
 * Eq. 2 (Sec. "Ablation study", Table "Ablation Studies on the EUTI-based Visual Token
 * Pruning"): PACT_FLAG_SCORE_NO_NORM drops the factor |h_i|, PACT_FLAG_SCORE_NORM_ONLY replaces
 * the softmax term by the constant 1/n, i.e. scores by hidden-state norm alone;
 * bit 3 (PACT_FLAG_KEY_STATS) makes pact_reduce fill pact_report.max_key_distance (0 otherwise;
 * dbdpc_cluster always fills it). */
typedef struct {
    float lambda;
    float d_c;
    float d_n;
    float alpha;
    int32_t fallback_T;
    uint32_t flags;
} pact_params;

#define PACT_FLAG_NO_MERGE 1u
#define PACT_FLAG_SCORE_NO_NORM 2u
#define PACT_FLAG_SCORE_NORM_ONLY 4u
#define PACT_FLAG_KEY_STATS 8u

/* Per-sample counters, in DEVICE memory, written by the entry points that produce them. */
typedef struct {
    int32_t n_kept;            /* |S_important| = q                         (pact_prune)   */
    int32_t n_pruned;          /* |S_unimportant|                           (pact_prune)   */
    int32_t n_centers;         /* C                                         (dbdpc_cluster) */
    int32_t n_reincorporated;  /* pruned tokens recovered by Eq. 8          (pact_reincorporate) */
    int32_t n_dropped;         /* pruned tokens not recovered                (pact_reincorporate) */
    int32_t rounds;            /* parallel centre rounds run, the last one confirming that no token is left (a
                                * round may use decisions other wavefronts took earlier in the same round, so
                                * the count can differ by one or two between runs; the centres cannot) */
    int32_t dc_checked_pairs;  /* ordered kept pairs re-evaluated in fp64 near d_c */
    int32_t dc_near_ties;      /* of those, pairs with |d - d_c| <= 1e-6 (each pair counted twice) */
    int32_t refine_overflow;   /* bit 0: the near-d_c list overflowed (those pairs keep their fp32 decision);
                                * bit 1: more than PACT_MAX_RHO_RECHECK tokens had a neighbour with a
                                * density inside the band (none was re-evaluated: fp32-term densities decide) */
    int32_t zero_norm_seen;    /* kept or pruned tokens with a zero-norm clustering key */
    float   max_key_distance;  /* largest Eq. 5 distance between two clustered keys, from the fp32 pass
                                * (the statistic Sec. "Selecting the layer L" looks at)  (dbdpc_cluster) */
    int32_t rho_rechecked;     /* kept tokens whose density was evaluated again in fp64 because a token
                                * within d_c had a density inside the band              (dbdpc_cluster) */
    int32_t rho_near_ties;     /* pairs of those whose fp64 densities differ, but by less than 1e-11 of
                                * their sum: an order even fp64 cannot vouch for        (dbdpc_cluster) */
    int32_t score_near_ties;   /* tokens whose score differs from the percentile threshold tau by at
                                * most 1e-6 * tau without being equal to it              (pact_prune) */
    int32_t nonfinite_seen;    /* tokens with a non-finite score, plus kept or pruned tokens whose
                                * clustering key has a non-finite norm        (pact_prune, dbdpc_cluster,
                                * pact_reincorporate) */
    int32_t reserved[1];       /* library use (clusters the merge takes first) */
} pact_report;

/* At most this many tokens of a sample have their density evaluated again in fp64. */
#define PACT_MAX_RHO_RECHECK 1024

/* Scratch bytes needed for one call on samples of at most n_max tokens each, `batch`
 * samples, clustering keys of width dk and type k_dt (fp32 keys need room for their three-part
 * bf16 form), n_q query heads of width d_h.  0 if an argument is out of range. */
size_t pact_workspace_bytes(int32_t n_max, int32_t batch, int32_t dk, pact_dtype k_dt, int32_t n_q, int32_t d_h);

/* Eq. 1 + Eq. 2 (Alg. 1 steps 1-2): importance score of every token.
 *   hidden   [n, h]           h_dt   hidden states at the reduction layer
 *   keys_pre [n, n_kv*d_h]    k_dt   keys before rotary embedding, heads concatenated
 *   q        [q_rows, n_q*d_h] q_dt  queries before rotary embedding; q_rows == n (Eq. 1 is
 *                                    applied) or q_rows == 1 (already the global query)
 *   flags    0, PACT_FLAG_SCORE_NO_NORM and / or PACT_FLAG_SCORE_NORM_ONLY (other bits ignored)
 *   scores   [n] fp32 out
 * n_q must be a multiple of n_kv: query head j reads key head j / (n_q / n_kv).  Softmax is
 * taken across the n tokens inside each head; no 1/sqrt(d_h) factor (Eq. 2 has none). */
int pact_score(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
               const void* keys_pre, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
               const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q, uint32_t flags,
               float* scores, void* ws, size_t ws_bytes, void* stream);

/* Eq. 3/4 (Alg. 1 step 3): tau = the (m+1)-th smallest score, m = min(floor(lambda*n), n-1);
 * kept = {s_i >= tau}, pruned = {s_i < tau}.
 *   kept_idx [n], pruned_idx [n] out, ascending; only the first n_kept / n_pruned are written
 *   rep      out: n_kept, n_pruned, score_near_ties, nonfinite_seen (scores only) */
int pact_prune(const float* scores, int32_t n, float lambda,
               int32_t* kept_idx, int32_t* pruned_idx, pact_report* rep,
               void* ws, size_t ws_bytes, void* stream);

/* Alg. 2 on the subset `idx` of the n tokens (Eq. 5, Eq. 6, density order, centre selection
 * with the bound d_c, nearest-centre assignment).
 *   keys       [n, dk] k_dt   keys after rotary embedding, heads concatenated (u_i of Sec. 3.2);
 *                             n * dk is limited (PACT_ERR_SHAPE beyond): n * dk * 2 < 2^32 for bf16 keys,
 *                             n * dk * 6 < 2^32 for fp32 keys (the same for every call with clustering keys)
 *   idx        [*n_idx_dev] ascending token indices to cluster, or NULL = all n tokens
 *   n_idx_dev  device int32 holding the subset size (ignored when idx is NULL)
 *   center_idx [n] out: token indices of the C centres, ascending (first C written)
 *   cluster_id [n] out: 0..C-1 for tokens in idx, -1 for the others
 *   rep        out: n_centers, rounds, dc_* and rho_* counters, refine_overflow, zero_norm_seen,
 *              nonfinite_seen, max_key_distance; when idx is NULL also n_kept = n, n_pruned = 0
 *   rho_opt    [n] fp64 out or NULL: density of idx[p] at position p, as it was used (fp64 sum of
 *              fp32 terms, or the fp64 value for the tokens counted in rho_rechecked)
 *   rank_opt   [n] int32 out or NULL: position of idx[p] in the descending order of those
 *              densities (0 = densest, equal densities by ascending index) */
int dbdpc_cluster(const void* keys, pact_dtype k_dt, int32_t n, int32_t dk,
                  const int32_t* idx, const int32_t* n_idx_dev,
                  float d_c, float d_n, int32_t fallback_T,
                  int32_t* center_idx, int32_t* cluster_id, pact_report* rep,
                  double* rho_opt, int32_t* rank_opt,
                  void* ws, size_t ws_bytes, void* stream);

/* Eq. 8/9 (Alg. 3 step 3): each pruned token joins its nearest centre s iff d_is < alpha*d_c.
 *   pruned_idx [rep->n_pruned], center_idx [rep->n_centers]  (n_kept, n_pruned and n_centers
 *   are read on the device from `rep`, as pact_prune and dbdpc_cluster left them)
 *   cluster_id [n] in/out: entries of pruned tokens are overwritten (cluster or -1)
 *   rep        in/out: n_reincorporated, n_dropped written; zero_norm_seen, nonfinite_seen added to */
int pact_reincorporate(const void* keys, pact_dtype k_dt, int32_t n, int32_t dk,
                       const int32_t* pruned_idx, const int32_t* center_idx,
                       float d_c, float alpha, int32_t* cluster_id, pact_report* rep,
                       void* ws, size_t ws_bytes, void* stream);

/* Eq. 10 (Alg. 3 step 4): merged[s] = mean of hidden[i] over cluster_id[i] == s.
 *   cluster_id     [n] values in -1..C-1, C = rep->n_centers (read on the device)
 *   rep            in/out: n_centers read; the library keeps a count of its own in reserved[]
 *   center_idx     [C] needed only with PACT_FLAG_NO_MERGE (may be NULL otherwise)
 *   merged         [n, h] out_dt, worst case; rows 0..C-1 written (a cluster id nobody carries
 *                  gives a row of zeros)
 *   cluster_counts [n] out: members per cluster (the weights W of Eq. 11) */
int pact_merge(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
               const int32_t* cluster_id, const int32_t* center_idx, pact_report* rep,
               uint32_t flags, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
               void* ws, size_t ws_bytes, void* stream);

/* Alg. 3 end to end for one sample, one enqueue, no host synchronisation.
 * Inputs as in pact_score (hidden, keys_pre, q) plus `keys` [n, dk = n_kv*d_h] for DBDPC
 * (may alias keys_pre).  Outputs: scores [n], kept_idx [n], pruned_idx [n], center_idx [n],
 * cluster_id [n], merged [n, h] out_dt, cluster_counts [n], rep (one record).  p: host. */
int pact_reduce(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
                const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                const pact_params* p,
                float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                pact_report* rep, void* ws, size_t ws_bytes, void* stream);

/* pact_reduce for callers that cannot allocate a workspace or pass one in: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation calls.  Arguments, outputs and
 * results are those of pact_reduce; the scratch is an array of PACT_STATIC_SCRATCH_BYTES bytes
 * that is part of the library's device code (each GPU the library runs on holds its own copy
 * until the process ends).  The call makes no allocation of any kind.
 *  - A call that would need more scratch than that (pact_workspace_bytes(n, 1, n_kv*d_h, k_dt,
 *    n_q, d_h) tells) returns PACT_ERR_WORKSPACE; every single image of up to 8748 tokens with
 *    512-wide bf16 keys and 28 query heads fits.
 *  - All calls on one GPU share that GPU's array: they must be ordered on one stream (or
 *    otherwise serialised); calls that overlap on one GPU race.  The array keeps the last call's
 *    contents, and like any workspace it is initialised by each call as far as the call reads it. */
#define PACT_STATIC_SCRATCH_BYTES (48u << 20)
int pact_reduce_static(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
                       const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                       const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                       const pact_params* p,
                       float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                       int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                       pact_report* rep, void* stream);

/* Alg. 3 for `batch` independent samples whose tokens are concatenated along dim 0.
 *   cu_seqlens host int32 [batch+1], cu_seqlens[0] = 0, strictly increasing; sample b owns
 *              rows cu_seqlens[b] .. cu_seqlens[b+1]-1 of every token-indexed tensor
 *   q_rows     total tokens (per-token queries) or batch (one global query per sample)
 *   p          host, [batch] parameter records
 * Token-indexed outputs are laid out like the inputs: sample b's kept_idx / pruned_idx /
 * center_idx / cluster_counts entries and merged rows start at offset cu_seqlens[b]; the
 * indices stored are local to the sample.  rep: [batch] records. */
int pact_reduce_varlen(const void* hidden, pact_dtype h_dt, int32_t h,
                       const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                       const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                       const int32_t* cu_seqlens, int32_t batch, const pact_params* p,
                       float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                       int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                       pact_report* rep, void* ws, size_t ws_bytes, void* stream);

/* What the layers after the reduction need besides the merged tokens (Alg. 3 last loop, Eq. 11):
 * the position id of merged token s, p'_s = positions[center_idx[s]] (the centre's own), and
 * the additive attention term of proportional attention, log_weight[s] = ln(cluster_counts[s]).
 * One sample, or `batch` samples laid out by cu_seqlens as in pact_reduce_varlen.
 *   center_idx, cluster_counts  as pact_reduce left them; entries 0..rep[b].n_centers-1 are read
 *   positions      [total] int32 position ids of the input tokens, or NULL for p_i = i (local)
 *   cu_seqlens     host, [batch+1], or NULL with batch == 1 and n tokens
 *   positions_out  [total] int32 out, log_weight [total] fp32 out: entries 0..n_centers-1 of
 *                  each sample are written */
int pact_attention_handoff(const int32_t* center_idx, const int32_t* cluster_counts, const pact_report* rep,
                           const int32_t* positions, const int32_t* cu_seqlens, int32_t batch, int32_t n,
                           int32_t* positions_out, float* log_weight, void* stream);

const char* pact_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PACT_H */

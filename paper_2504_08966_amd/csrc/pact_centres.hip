// DBDPC after the Gram pass (Alg. 2): density order, centre selection under the bound d_c
// done in parallel rounds (same centres as the sequential loop; cf. the recursive scheme of
// appendix D), nearest-centre assignment; and the recovery of pruned tokens (Eq. 8/9).
//
// Centre selection.  Token i "precedes" j when rho_i > rho_j, or rho_i == rho_j and i < j.
// Alg. 2 makes i a centre iff no centre that precedes it lies within d_c.  With the bitmap
// adj[i][j] = (d_ij <= d_c) this is a fixed point every token can evaluate on its own:
//     a preceding neighbour is a centre            -> i is not a centre
//     every preceding neighbour is known not to be -> i is a centre
// A round evaluates this for all undecided tokens at once (one wavefront per token); the
// densest undecided token is always decided, so the rounds terminate, and the result does
// not depend on how stale the statuses read within a round are.
#include "pact_internal.h"

namespace pact {

// ------------------------------------------------------------------------------------------
// Start-of-call initialisation of everything the later kernels accumulate into.
// grid (ceil(n_max/256), B), block 256.
__global__ __launch_bounds__(256) void init_kernel(Batch bt, Ws w, pact_report* rep, int32_t* cluster_id,
                                                   int32_t* cluster_counts, int mode,
                                                   const int32_t* n_idx_dev) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        w.near_cnt[b] = 0;
        for (int r = 0; r < MAX_ROUNDS; ++r) w.round_new[b * MAX_ROUNDS + r] = 0;
        pact_report* rp = rep + b;
        if (mode == INIT_REDUCE || mode == INIT_DBDPC_ALL || mode == INIT_DBDPC_SUBSET) {
            if (mode != INIT_REDUCE) {
                rp->n_kept = (mode == INIT_DBDPC_ALL) ? sg.n : min(max(*n_idx_dev, 0), sg.n);
                rp->n_pruned = (mode == INIT_DBDPC_ALL) ? 0 : sg.n - rp->n_kept;
            }
            rp->n_centers = 0; rp->rounds = 0; rp->dc_checked_pairs = 0; rp->dc_near_ties = 0;
            rp->refine_overflow = 0; rp->zero_norm_seen = 0;
            rp->n_reincorporated = 0; rp->n_dropped = 0;
            for (int k = 0; k < 6; ++k) rp->reserved[k] = 0;
        }
        if (mode == INIT_REINC) { rp->n_reincorporated = 0; rp->n_dropped = 0; rp->zero_norm_seen = 0; }
    }
    if (i >= sg.n) return;
    const size_t g = (size_t)sg.base + i;
    const size_t l = (size_t)b * bt.n_max + i;
    if (mode == INIT_REDUCE || mode == INIT_DBDPC_ALL || mode == INIT_DBDPC_SUBSET) {
        w.status[l] = ST_UNKNOWN;
        w.ident[g] = i;
        cluster_id[g] = -1;
        if (cluster_counts) cluster_counts[g] = 0;
    }
    if (mode == INIT_MERGE && cluster_counts) cluster_counts[g] = 0;
}

// ------------------------------------------------------------------------------------------
// Squared norm (fp64), reciprocal norm (fp32) of every token's clustering key, and a cleared
// bitmap row per token.  One wavefront per token; grid (ceil(n_max/4), B), block 256.
template <int DT>
__global__ __launch_bounds__(256) void key_prep_kernel(Batch bt, const char* __restrict__ keys, int dk,
                                                        double* __restrict__ nn, float* __restrict__ rinv,
                                                        uint64_t* __restrict__ adj, pact_report* rep) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= sg.n) return;
    const size_t g = (size_t)sg.base + i;
    const char* row = keys + g * (size_t)dk * Elem<DT>::BYTES;
    const double v = wave_dot64<DT>(row, row, dk, lane);
    if (lane == 0) {
        nn[g] = v;
        rinv[g] = v > 0.0 ? (float)(1.0 / sqrt(v)) : 0.0f;
        if (!(v > 0.0)) atomicAdd(&rep[b].zero_norm_seen, 1);
    }
    uint64_t* arow = adj + ((size_t)b * bt.n_max + i) * bt.W;
    const int Wn = (sg.n + 63) >> 6;
    for (int k = lane; k < Wn; k += 64) arow[k] = 0ull;
}

// ------------------------------------------------------------------------------------------
// Pairs the Gram epilogue could not decide in fp32: evaluate Eq. 5 in fp64 and clear the bit
// if the distance exceeds d_c.  One wavefront per pair, grid (64, B), block 256.
template <int DT>
__global__ __launch_bounds__(256) void refine_kernel(Batch bt, const char* __restrict__ keys, int dk,
                                                      const int32_t* __restrict__ idx,
                                                      const double* __restrict__ nn,
                                                      const uint32_t* __restrict__ near_list,
                                                      const int32_t* __restrict__ near_cnt,
                                                      uint64_t* __restrict__ adj, pact_report* rep) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nw = gridDim.x * 4;
    const int raw = near_cnt[b];
    const int cnt = min(raw, NEAR_CAP);
    if (gw == 0 && lane == 0) {
        rep[b].dc_checked_pairs = cnt;
        rep[b].refine_overflow = raw > NEAR_CAP;
    }
    const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
    const char* kb = keys + (size_t)sg.base * row_bytes;
    const int32_t* ix = idx + sg.base;
    const double* nnb = nn + sg.base;
    const double d_c = (double)sg.d_c;
    int ties = 0;
    for (int e = gw; e < cnt; e += nw) {
        const uint32_t pi = near_list[((size_t)b * NEAR_CAP + e) * 2];
        const uint32_t pj = near_list[((size_t)b * NEAR_CAP + e) * 2 + 1];
        const int ti = ix[pi], tj = ix[pj];
        double d = 0.0;
        if (pi != pj) {
            const double dot = wave_dot64<DT>(kb + (size_t)ti * row_bytes, kb + (size_t)tj * row_bytes, dk, lane);
            d = cos_dist64(dot, nnb[ti], nnb[tj]);
        }
        if (lane == 0) {
            if (d > d_c)
                atomicAnd((unsigned long long*)&adj[((size_t)b * bt.n_max + pi) * bt.W + (pj >> 6)],
                          ~(1ull << (pj & 63)));
            if (fabs(d - d_c) <= 1e-6) ++ties;
        }
    }
    if (lane == 0 && ties) atomicAdd(&rep[b].dc_near_ties, ties);
}

// ------------------------------------------------------------------------------------------
// Eq. 6 completed: rho_p = sum over the 64-row blocks of the column partials.  With d_n = 2
// every term is an fp32 value in [e^-1, 1], so these fp64 additions are exact and the result
// does not depend on the order.  grid (ceil(n_max/256), B), block 256.
__global__ __launch_bounds__(256) void rho_finalize_kernel(Batch bt, const pact_report* __restrict__ rep,
                                                           const double* __restrict__ rho_part,
                                                           double* __restrict__ rho, double* rho_opt) {
    const int b = blockIdx.y;
    const int q = clamp_count(rep[b].n_kept, bt.s[b].n);
    const int p = blockIdx.x * 256 + threadIdx.x;
    if (p >= q) return;
    const int nrt = (q + 63) >> 6;
    const double* in = rho_part + (size_t)b * bt.W * bt.n_max + p;
    double acc = 0.0;
    for (int r = 0; r < nrt; ++r) acc += in[(size_t)r * bt.n_max];
    rho[(size_t)b * bt.n_max + p] = acc;
    if (rho_opt) rho_opt[bt.s[b].base + p] = acc;
}

// Density order by enumeration: rank_p = #{j : rho_j > rho_p, or rho_j == rho_p and j < p}.
// grid (ceil(n_max/64), B), block 1024 = 64 tokens x 16 slices of the j range.
__global__ __launch_bounds__(1024) void rank_kernel(Batch bt, const pact_report* __restrict__ rep,
                                                    const double* __restrict__ rho,
                                                    int32_t* __restrict__ rank, int32_t* rank_opt) {
    __shared__ int s_cnt[16][64];
    const int b = blockIdx.y;
    const int q = clamp_count(rep[b].n_kept, bt.s[b].n);
    if (blockIdx.x * 64 >= q) return;
    const int lane = threadIdx.x & 63;
    const int slice = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int p = blockIdx.x * 64 + lane;
    const double* r = rho + (size_t)b * bt.n_max;
    const double mine = (p < q) ? r[p] : 0.0;
    const int per = (q + 15) / 16;
    const int j0 = slice * per, j1 = min(q, j0 + per);
    int cnt = 0;
    for (int j = j0; j < j1; ++j) {
        const double v = r[j];
        cnt += (v > mine) || (v == mine && j < p);
    }
    s_cnt[slice][lane] = cnt;
    __syncthreads();
    if (threadIdx.x < 64 && p < q) {
        int tot = 0;
#pragma unroll
        for (int s = 0; s < 16; ++s) tot += s_cnt[s][lane];
        rank[(size_t)b * bt.n_max + p] = tot;
        if (rank_opt) rank_opt[bt.s[b].base + p] = tot;
    }
}

// ------------------------------------------------------------------------------------------
// One parallel round of centre selection.  One wavefront per kept token;
// grid (ceil(n_max/4), B), block 256.
__global__ __launch_bounds__(256) void centre_round_kernel(Batch bt, const pact_report* __restrict__ rep,
                                                           const uint64_t* __restrict__ adj,
                                                           const int32_t* __restrict__ rank,
                                                           uint32_t* status, int32_t* round_new, int round) {
    const int b = blockIdx.y;
    const int q = clamp_count(rep[b].n_kept, bt.s[b].n);
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= q) return;
    const int T = bt.s[b].fallback_T;
    if (round > 0 && round_new[b * MAX_ROUNDS + round - 1] < T) return;   // leave the rest to the finisher
    uint32_t* st = status + (size_t)b * bt.n_max;
    if (st[p] != ST_UNKNOWN) return;
    const int32_t* rk = rank + (size_t)b * bt.n_max;
    const int myrank = rk[p];
    const uint64_t* row = adj + ((size_t)b * bt.n_max + p) * bt.W;
    const int Wq = (q + 63) >> 6;
    bool blocked = false, pending = false;
    for (int w0 = 0; w0 < Wq; w0 += 64) {
        const int w = w0 + lane;
        uint64_t word = (w < Wq) ? row[w] : 0ull;
        while (word) {
            const int bit = __builtin_ctzll(word);
            word &= word - 1;
            const int j = (w << 6) + bit;
            if (j < q && rk[j] < myrank) {
                const uint32_t sj = st[j];
                blocked |= (sj == ST_CENTER);
                pending |= (sj == ST_UNKNOWN);
            }
        }
    }
    blocked = __any(blocked);
    pending = __any(pending);
    if (lane == 0) {
        if (blocked) st[p] = ST_NOT;
        else if (!pending) { st[p] = ST_CENTER; atomicAdd(&round_new[b * MAX_ROUNDS + round], 1); }
    }
}

// Finishing kernel: one workgroup per sample repeats the round on the statuses held in LDS
// until nothing is undecided (at least the densest undecided token is decided per round, so
// at most q rounds), then numbers the centres in ascending token order and publishes them.
// grid (B), block 1024.
__global__ __launch_bounds__(1024) void centre_finish_kernel(Batch bt, pact_report* rep,
                                                             const uint64_t* __restrict__ adj,
                                                             const int32_t* __restrict__ rank,
                                                             const int32_t* __restrict__ idx,
                                                             uint32_t* status, const int32_t* round_new,
                                                             int32_t* cnum, uint64_t* cmask,
                                                             int32_t* center_idx) {
    extern __shared__ unsigned char s_st[];        // q bytes
    __shared__ int s_unknown;
    __shared__ int s_wtot[16];
    const int b = blockIdx.x;
    const Seg sg = bt.s[b];
    const int q = clamp_count(rep[b].n_kept, bt.s[b].n);
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    uint32_t* st = status + (size_t)b * bt.n_max;
    const int32_t* rk = rank + (size_t)b * bt.n_max;
    const int Wq = (q + 63) >> 6;
    for (int p = tid; p < q; p += 1024) s_st[p] = (unsigned char)st[p];
    int rounds = 0;
    for (int r = 0; r < MAX_ROUNDS; ++r) rounds += (round_new[b * MAX_ROUNDS + r] > 0);
    while (true) {
        if (tid == 0) s_unknown = 0;
        __syncthreads();
        bool any_unknown = false;
        for (int p = wave; p < q; p += 16) {
            if (s_st[p] != ST_UNKNOWN) continue;
            const int myrank = rk[p];
            const uint64_t* row = adj + ((size_t)b * bt.n_max + p) * bt.W;
            bool blocked = false, pending = false;
            for (int w0 = 0; w0 < Wq; w0 += 64) {
                const int w = w0 + lane;
                uint64_t word = (w < Wq) ? row[w] : 0ull;
                while (word) {
                    const int bit = __builtin_ctzll(word);
                    word &= word - 1;
                    const int j = (w << 6) + bit;
                    if (j < q && rk[j] < myrank) {
                        const unsigned char sj = ((volatile unsigned char*)s_st)[j];
                        blocked |= (sj == ST_CENTER);
                        pending |= (sj == ST_UNKNOWN);
                    }
                }
            }
            blocked = __any(blocked);
            pending = __any(pending);
            if (blocked) { if (lane == 0) s_st[p] = ST_NOT; }
            else if (!pending) { if (lane == 0) s_st[p] = ST_CENTER; }
            else any_unknown = true;
        }
        if (any_unknown && lane == 0) s_unknown = 1;
        __syncthreads();
        const int more = s_unknown;
        __syncthreads();
        if (!more) break;
        ++rounds;
    }
    // number the centres in ascending p (= ascending token index)
    const int chunk = (q + 1023) / 1024;
    const int p0 = min(q, tid * chunk), p1 = min(q, p0 + chunk);
    int cnt = 0;
    for (int p = p0; p < p1; ++p) cnt += (s_st[p] == ST_CENTER);
    int inc = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int v = __shfl_up(inc, d, 64);
        if (lane >= d) inc += v;
    }
    if (lane == 63) s_wtot[wave] = inc;
    __syncthreads();
    int woff = 0, total = 0;
    for (int w = 0; w < 16; ++w) {
        if (w < wave) woff += s_wtot[w];
        total += s_wtot[w];
    }
    int c = woff + inc - cnt;
    int32_t* cn = cnum + (size_t)b * bt.n_max;
    const int32_t* ix = idx + sg.base;
    int32_t* co = center_idx + sg.base;
    for (int p = p0; p < p1; ++p) {
        const bool isc = s_st[p] == ST_CENTER;
        st[p] = s_st[p];
        cn[p] = isc ? c : -1;
        if (isc) co[c++] = ix[p];
    }
    uint64_t* cm = cmask + (size_t)b * bt.W;
    for (int w = tid; w < Wq; w += 1024) {
        uint64_t m = 0;
        const int pe = min(q, (w + 1) << 6);
        for (int p = w << 6; p < pe; ++p) m |= (uint64_t)(s_st[p] == ST_CENTER) << (p & 63);
        cm[w] = m;
    }
    if (tid == 0) {
        rep[b].n_centers = total;
        rep[b].rounds = rounds;
    }
}

// ------------------------------------------------------------------------------------------
// Iterate, in ascending order, over the set bits of (row[w] & mask[w]) for w < nWords, calling
// f(bitIndex) with a wave-uniform index.  All 64 lanes must call it together.
template <typename F>
__device__ __forceinline__ void for_each_bit_uniform(const uint64_t* row, const uint64_t* mask, int nWords,
                                                     int lane, F f) {
    for (int w0 = 0; w0 < nWords; w0 += 64) {
        const int w = w0 + lane;
        uint64_t word = 0ull;
        if (w < nWords) word = mask ? (row[w] & mask[w]) : row[w];
        uint64_t have = __ballot(word != 0ull);
        while (have) {
            const int src = __builtin_ctzll(have);
            const uint32_t lo = __shfl((uint32_t)word, src, 64);
            const uint32_t hi = __shfl((uint32_t)(word >> 32), src, 64);
            uint64_t wv = ((uint64_t)hi << 32) | lo;
            while (wv) {
                const int bit = __builtin_ctzll(wv);
                wv &= wv - 1;
                f(((w0 + src) << 6) + bit);
            }
            have &= have - 1;
        }
    }
}

// Alg. 2 last loop: every kept token joins the nearest centre, distances in fp64 over the
// centres its bitmap row allows (the nearest centre is within d_c, hence among them).
// One wavefront per kept token; grid (ceil(n_max/4), B), block 256.
template <int DT>
__global__ __launch_bounds__(256) void assign_kernel(Batch bt, const pact_report* __restrict__ rep,
                                                      const char* __restrict__ keys, int dk,
                                                      const int32_t* __restrict__ idx,
                                                      const double* __restrict__ nn,
                                                      const uint64_t* __restrict__ adj,
                                                      const uint64_t* __restrict__ cmask,
                                                      const uint32_t* __restrict__ status,
                                                      const int32_t* __restrict__ cnum,
                                                      int32_t* cluster_id, int32_t* cluster_counts) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int q = clamp_count(rep[b].n_kept, bt.s[b].n);
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (p >= q) return;
    const int32_t* ix = idx + sg.base;
    const int32_t* cn = cnum + (size_t)b * bt.n_max;
    const int tok = ix[p];
    int cid;
    if (status[(size_t)b * bt.n_max + p] == ST_CENTER) {
        cid = cn[p];
    } else {
        const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
        const char* kb = keys + (size_t)sg.base * row_bytes;
        const double* nnb = nn + sg.base;
        const char* mine = kb + (size_t)tok * row_bytes;
        const double nnp = nnb[tok];
        double best = INFINITY;
        int bestj = -1;
        for_each_bit_uniform(adj + ((size_t)b * bt.n_max + p) * bt.W, cmask + (size_t)b * bt.W,
                             (q + 63) >> 6, lane, [&](int j) {
            if (j >= q) return;
            const int tj = ix[j];
            const double dot = wave_dot64<DT>(mine, kb + (size_t)tj * row_bytes, dk, lane);
            const double d = cos_dist64(dot, nnp, nnb[tj]);
            if (d < best) { best = d; bestj = j; }
        });
        cid = bestj >= 0 ? cn[bestj] : -1;
    }
    if (lane == 0) {
        cluster_id[sg.base + tok] = cid;
        if (cid >= 0 && cluster_counts) atomicAdd(&cluster_counts[sg.base + cid], 1);
    }
}

// Eq. 8/9: every pruned token joins the nearest centre iff its fp64 distance is below
// alpha*d_c; candidates come from the matrix-core pass (bitmap rows q + t, bits over centres).
// One wavefront per pruned token; grid (ceil(n_max/4), B), block 256.
template <int DT>
__global__ __launch_bounds__(256) void reinc_assign_kernel(Batch bt, pact_report* rep,
                                                            const char* __restrict__ keys, int dk,
                                                            const int32_t* __restrict__ pruned_idx,
                                                            const int32_t* __restrict__ center_idx,
                                                            const double* __restrict__ nn,
                                                            const uint64_t* __restrict__ adj,
                                                            int32_t* cluster_id, int32_t* cluster_counts) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int q = clamp_count(rep[b].n_kept, sg.n), np = clamp_count(rep[b].n_pruned, sg.n - q),
              C = clamp_count(rep[b].n_centers, q);
    const int lane = threadIdx.x & 63;
    const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= np) return;
    const int tok = pruned_idx[sg.base + t];
    const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
    const char* kb = keys + (size_t)sg.base * row_bytes;
    const double* nnb = nn + sg.base;
    const int32_t* co = center_idx + sg.base;
    const char* mine = kb + (size_t)tok * row_bytes;
    const double nnp = nnb[tok];
    const double thr = (double)sg.alpha * (double)sg.d_c;
    double best = INFINITY;
    int bestc = -1;
    if (thr > 0.0 && C > 0) {
        for_each_bit_uniform(adj + ((size_t)b * bt.n_max + q + t) * bt.W, nullptr, (C + 63) >> 6, lane,
                             [&](int c) {
            if (c >= C) return;
            const int tc = co[c];
            const double dot = wave_dot64<DT>(mine, kb + (size_t)tc * row_bytes, dk, lane);
            const double d = cos_dist64(dot, nnp, nnb[tc]);
            if (d < thr && d < best) { best = d; bestc = c; }
        });
    }
    if (lane == 0) {
        cluster_id[sg.base + tok] = bestc;
        if (bestc >= 0) {
            if (cluster_counts) atomicAdd(&cluster_counts[sg.base + bestc], 1);
            atomicAdd(&rep[b].n_reincorporated, 1);
        } else {
            atomicAdd(&rep[b].n_dropped, 1);
        }
    }
}

// ------------------------------------------------------------------------------------------
int launch_init(const Batch& bt, const Ws& w, pact_report* rep, int32_t* cluster_id,
                int32_t* cluster_counts, int mode, const int32_t* n_idx_dev, hipStream_t st) {
    PACT_LAUNCH("init", init_kernel, dim3((bt.n_max + 255) / 256, bt.B), dim3(256), st, bt, w, rep,
                cluster_id, cluster_counts, mode, n_idx_dev);
    return PACT_OK;
}

int launch_key_prep(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                    pact_report* rep, hipStream_t st) {
    dim3 grid((bt.n_max + 3) / 4, bt.B);
    if (k_dt == PACT_BF16)
        PACT_LAUNCH("key_prep", key_prep_kernel<PACT_BF16>, grid, dim3(256), st, bt, (const char*)keys, dk,
                    w.nn, w.rinv, w.adj, rep);
    else
        PACT_LAUNCH("key_prep", key_prep_kernel<PACT_F32>, grid, dim3(256), st, bt, (const char*)keys, dk,
                    w.nn, w.rinv, w.adj, rep);
    return PACT_OK;
}

int launch_centres(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                   const int32_t* idx, int32_t* center_idx, int32_t* cluster_id,
                   int32_t* cluster_counts, pact_report* rep, double* rho_opt, int32_t* rank_opt,
                   hipStream_t st) {
    const char* k = (const char*)keys;
    if (k_dt == PACT_BF16)
        PACT_LAUNCH("refine_pairs", refine_kernel<PACT_BF16>, dim3(64, bt.B), dim3(256), st, bt, k, dk, idx,
                    w.nn, w.near_list, w.near_cnt, w.adj, rep);
    else
        PACT_LAUNCH("refine_pairs", refine_kernel<PACT_F32>, dim3(64, bt.B), dim3(256), st, bt, k, dk, idx,
                    w.nn, w.near_list, w.near_cnt, w.adj, rep);
    PACT_LAUNCH("rho_finalize", rho_finalize_kernel, dim3((bt.n_max + 255) / 256, bt.B), dim3(256), st, bt,
                rep, w.rho_part, w.rho, rho_opt);
    PACT_LAUNCH("density_rank", rank_kernel, dim3((bt.n_max + 63) / 64, bt.B), dim3(1024), st, bt, rep,
                w.rho, w.rank, rank_opt);
    const int n_par = 4;
    for (int r = 0; r < n_par; ++r)
        PACT_LAUNCH("centre_round", centre_round_kernel, dim3((bt.n_max + 3) / 4, bt.B), dim3(256), st, bt,
                    rep, w.adj, w.rank, w.status, w.round_new, r);
    PACT_LAUNCH_SHMEM("centre_finish", centre_finish_kernel, dim3(bt.B), dim3(1024),
                      (size_t)((bt.n_max + 255) / 256 * 256), st, bt, rep, w.adj, w.rank, idx, w.status,
                      w.round_new, w.cnum, w.cmask, center_idx);
    dim3 grid((bt.n_max + 3) / 4, bt.B);
    if (k_dt == PACT_BF16)
        PACT_LAUNCH("assign", assign_kernel<PACT_BF16>, grid, dim3(256), st, bt, rep, k, dk, idx, w.nn,
                    w.adj, w.cmask, w.status, w.cnum, cluster_id, cluster_counts);
    else
        PACT_LAUNCH("assign", assign_kernel<PACT_F32>, grid, dim3(256), st, bt, rep, k, dk, idx, w.nn,
                    w.adj, w.cmask, w.status, w.cnum, cluster_id, cluster_counts);
    return PACT_OK;
}

int launch_gram_candidates(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                           const int32_t* pruned_idx, const int32_t* center_idx, pact_report* rep,
                           hipStream_t st);

int launch_reincorporate(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                         const int32_t* pruned_idx, const int32_t* center_idx, int32_t* cluster_id,
                         int32_t* cluster_counts, pact_report* rep, hipStream_t st) {
    int rc = launch_gram_candidates(bt, w, keys, k_dt, dk, pruned_idx, center_idx, rep, st);
    if (rc != PACT_OK) return rc;
    dim3 grid((bt.n_max + 3) / 4, bt.B);
    if (k_dt == PACT_BF16)
        PACT_LAUNCH("reinc_assign", reinc_assign_kernel<PACT_BF16>, grid, dim3(256), st, bt, rep,
                    (const char*)keys, dk, pruned_idx, center_idx, w.nn, w.adj, cluster_id, cluster_counts);
    else
        PACT_LAUNCH("reinc_assign", reinc_assign_kernel<PACT_F32>, grid, dim3(256), st, bt, rep,
                    (const char*)keys, dk, pruned_idx, center_idx, w.nn, w.adj, cluster_id, cluster_counts);
    return PACT_OK;
}

}  // namespace pact

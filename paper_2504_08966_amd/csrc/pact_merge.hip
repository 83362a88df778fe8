// Merge (Eq. 10, Alg. 3 step 4): h'_s = mean of the hidden states of cluster s.
// Member lists are built with integer atomics (their order inside a cluster is then sorted,
// so the fp64 accumulation order - ascending token index - and hence every output bit is
// the same on every run).  The stage is bound by reading the member rows of H once and
// writing C rows.
#include "pact_internal.h"

namespace pact {

// The large clusters (MERGE_BIG rows or more) are merged first; the others follow in cluster order,
// i.e. in token order, which their reads profit from.

// Member lists (CSR) of all clusters of a sample, by one workgroup: cluster sizes (taken from
// cluster_counts, or recounted from cluster_id for a stand-alone merge), their exclusive scan,
// and the fill with LDS cursors.  grid (B), block 1024, dynamic LDS n_max * 4 bytes.
// offsets of sample b live at [base + b, base + b + C].
__global__ __launch_bounds__(1024) void scan_fill_kernel(Batch bt, const int32_t* __restrict__ cluster_id,
                                                         pact_report* rep,
                                                         int32_t* cluster_counts, int recount,
                                                         int write_totals, int32_t* offsets,
                                                         int32_t* members, int32_t* big) {
    extern __shared__ int s_cur[];          // [C]: sizes, then running fill cursors
    __shared__ int s_wtot[16];
    __shared__ int s_nbig;
    const int b = blockIdx.x;
    const Seg sg = bt.s[b];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int32_t* cnt = cluster_counts + sg.base;
    int32_t* off = offsets + sg.base + b;
    const int32_t* cid = cluster_id + sg.base;
    // the cluster ids of this thread's tokens (i = tid, tid + 1024, ...): fetched now, beside the
    // sizes, so that the fill below does not start with a trip to memory
    constexpr int PRE = 8;
    int cid_pre[PRE];
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        const int i = tid + 1024 * k;
        cid_pre[k] = (i < sg.n) ? cid[i] : -1;
    }
    int cnt_pre[4];                          // likewise the sizes of the first clusters (an entry exists for every index below n)
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = tid + 1024 * k;
        cnt_pre[k] = (!recount && c < sg.n) ? cnt[c] : 0;
    }
    const int C = clamp_count(rep[b].n_centers, sg.n);
    if (recount) {
        for (int c = tid; c < C; c += 1024) s_cur[c] = 0;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < PRE; ++k) {
            const int c = cid_pre[k];
            if (c >= 0 && c < C) atomicAdd(&s_cur[c], 1);
        }
        for (int i = tid + 1024 * PRE; i < sg.n; i += 1024) {
            const int c = cid[i];
            if (c >= 0 && c < C) atomicAdd(&s_cur[c], 1);
        }
        __syncthreads();
        for (int c = tid; c < C; c += 1024) cnt[c] = s_cur[c];
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (tid + 1024 * k < C) s_cur[tid + 1024 * k] = cnt_pre[k];
        for (int c = tid + 4096; c < C; c += 1024) s_cur[c] = cnt[c];
    }
    if (tid == 0) s_nbig = 0;
    __syncthreads();
    const int chunk = (C + 1023) / 1024;
    const int c0 = min(C, tid * chunk), c1 = min(C, c0 + chunk);
    int loc = 0;
    for (int c = c0; c < c1; ++c) loc += s_cur[c];
    const int inc = wave_scan_incl_i32(loc);
    if (lane == 63) s_wtot[wave] = inc;
    // the large clusters (sizes are still in s_cur), appended a wavefront at a time
    int32_t* bigl = big + sg.base;
    for (int cb = 0; cb < C; cb += 1024) {                   // (wave-uniform trip count)
        const int c = cb + tid;
        const bool isbig = c < C && s_cur[c] >= MERGE_BIG;
        const uint64_t m = __ballot(isbig);
        if (m) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_nbig, __popcll(m));
            base = lane0_of(base);
            if (isbig) bigl[base + __popcll(m & ((1ull << lane) - 1ull))] = c;
        }
    }
    __syncthreads();
    if (tid == 0) rep[b].reserved[0] = s_nbig;               // read by the merge together with the cluster count
    int run = inc - loc;
    for (int w = 0; w < wave; ++w) run += s_wtot[w];
    for (int c = c0; c < c1; ++c) {
        const int sz = s_cur[c];
        off[c] = run;
        s_cur[c] = run;                     // cursor starts at the segment's offset
        run += sz;
    }
    if (c1 == C && c0 < C) {
        off[C] = run;                        // run = all cluster members = kept + recovered
        if (write_totals) {
            const int q = clamp_count(rep[b].n_kept, sg.n);
            rep[b].n_reincorporated = run - q;
            rep[b].n_dropped = sg.n - run;
        }
    }
    if (C == 0 && tid == 0) off[0] = 0;
    __syncthreads();
    int32_t* mem = members + sg.base;
#pragma unroll
    for (int k = 0; k < PRE; ++k) {
        const int c = cid_pre[k];
        if (c >= 0 && c < C) mem[atomicAdd(&s_cur[c], 1)] = tid + 1024 * k;
    }
    for (int i = tid + 1024 * PRE; i < sg.n; i += 1024) {
        const int c = cid[i];
        if (c >= 0 && c < C) mem[atomicAdd(&s_cur[c], 1)] = i;
    }
}

constexpr int MERGE_LDS_MEMBERS = 1024;

template <int ODT> struct StoreOut;
template <> struct StoreOut<PACT_F32> {
    template <int N> __device__ static __forceinline__ void put(char* out, size_t e, const double* v, bool stream) {
        float* o = (float*)out + e;
#pragma unroll
        for (int i = 0; i < N; i += 4) {
            const float4 f = make_float4((float)v[i], (float)v[i + 1], (float)v[i + 2], (float)v[i + 3]);
            if (stream) store_once16(o + i, make_uint4(__float_as_uint(f.x), __float_as_uint(f.y), __float_as_uint(f.z), __float_as_uint(f.w)));
            else *(float4*)(o + i) = f;
        }
    }
};
template <> struct StoreOut<PACT_BF16> {
    template <int N> __device__ static __forceinline__ void put(char* out, size_t e, const double* v, bool stream) {
        uint16_t* o = (uint16_t*)out + e;
        uint32_t w[N / 2];
#pragma unroll
        for (int i = 0; i < N; i += 2)
            w[i / 2] = f32_to_bf16_rne((float)v[i]) | (f32_to_bf16_rne((float)v[i + 1]) << 16);
        if (N == 8) {
            if (stream) store_once16(o, make_uint4(w[0], w[1], w[2], w[3]));
            else *(uint4*)o = make_uint4(w[0], w[1], w[2], w[3]);
        } else {
            *(uint2*)o = make_uint2(w[0], w[1]);
        }
    }
};

// One workgroup per cluster (persistent over clusters).  grid (min(n_max, 4096), B), block 512.
// The members of a cluster come from the CSR lists (slots == nullptr), or from the cluster's
// member slots, or - a cluster with more members than slots - from a pass over cluster_id.
// With slots the last workgroup also derives the recovered / dropped totals from the sizes.
template <int HDT, int ODT>
__global__ __launch_bounds__(512) void merge_kernel(Batch bt, const char* __restrict__ hidden, int h,
                                                     const int32_t* __restrict__ cluster_id,
                                                     const int32_t* __restrict__ center_idx,
                                                     pact_report* rep,
                                                     const int32_t* __restrict__ cluster_counts,
                                                     const int32_t* __restrict__ offsets,
                                                     const int32_t* __restrict__ members,
                                                     const int32_t* __restrict__ slots,
                                                     const int32_t* __restrict__ big,
                                                     char* __restrict__ merged, int stream) {
    __shared__ int s_raw[MERGE_LDS_MEMBERS];
    __shared__ int s_sorted[MERGE_LDS_MEMBERS];
    __shared__ int s_n;
    constexpr int EPL = Elem<HDT>::EPL;
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int tid = threadIdx.x;
    const int C = clamp_count(rep[b].n_centers, sg.n);
    const int nbig = clamp_count(rep[b].reserved[0], C);      // (same cache line as the cluster count)
    const size_t hrow = (size_t)h * Elem<HDT>::BYTES;
    const char* hb = hidden + (size_t)sg.base * hrow;
    const bool no_merge = (sg.flags & PACT_FLAG_NO_MERGE) != 0;

    // work items 0 .. nbig-1: the large clusters; then all clusters in order, the large ones skipped
    for (int k = blockIdx.x; k < nbig + C; k += gridDim.x) {
        const int c = (k < nbig) ? big[sg.base + k] : k - nbig;
        // (the slots go out with the size: garbage beyond it, never used)
        const int slot_pre = (slots && tid < MERGE_SLOTS) ? slots[(size_t)(sg.base + c) * MERGE_SLOTS + tid] : 0;
        int m = cluster_counts[sg.base + c];
        if (k >= nbig && m >= MERGE_BIG) continue;                 // (uniform over the workgroup)
        bool in_lds = true;
        __syncthreads();                       // previous cluster's readers are done with the LDS lists
        if (no_merge) {
            if (tid == 0) s_sorted[0] = center_idx[sg.base + c];
        } else if (m <= MERGE_LDS_MEMBERS) {
            if (!slots) {
                const int32_t* mem = members + sg.base + offsets[sg.base + b + c];
                for (int k = tid; k < m; k += 512) s_raw[k] = mem[k];
            } else if (m <= MERGE_SLOTS) {
                if (tid < m) s_raw[tid] = slot_pre;
            } else {
                if (tid == 0) s_n = 0;
                __syncthreads();
                // (16 ids per thread and trip to memory)
                for (int i0 = tid; i0 < sg.n; i0 += 16 * 512) {
                    int ids[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u) ids[u] = (i0 + 512 * u < sg.n) ? cluster_id[sg.base + i0 + 512 * u] : -1;
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        if (ids[u] == c) s_raw[min(atomicAdd(&s_n, 1), MERGE_LDS_MEMBERS - 1)] = i0 + 512 * u;
                }
            }
            __syncthreads();
            for (int k = tid; k < m; k += 512) {
                const int v = s_raw[k];
                int pos = 0;
                for (int u = 0; u < m; ++u) pos += (s_raw[u] < v);
                s_sorted[pos] = v;
            }
        } else {
            in_lds = false;
        }
        __syncthreads();
        const int m_eff = no_merge ? 1 : m;
        const double inv_m = 1.0 / (double)(m_eff > 0 ? m_eff : 1);
        for (int e = tid * EPL; e < h; e += 512 * EPL) {
            double acc[EPL];
#pragma unroll
            for (int i = 0; i < EPL; ++i) acc[i] = -0.0;   // additive identity that keeps the sign of -0.0
            if (in_lds) {
                const char* hcol = hb + (size_t)e * Elem<HDT>::BYTES;
                for (int k = 0; k < m_eff; k += 4) {
                    uint4 v[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        v[u] = (k + u >= m_eff) ? make_uint4(0, 0, 0, 0)
                             : stream ? load_once16(hcol + (size_t)s_sorted[k + u] * hrow)   // (their last use in a call)
                                      : *(const uint4*)(hcol + (size_t)s_sorted[k + u] * hrow);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        if (k + u < m_eff) {          // (skipping keeps -0.0 rows exact)
                            double x[8];
                            Elem<HDT>::widen(v[u], x);
#pragma unroll
                            for (int i = 0; i < EPL; ++i) acc[i] += x[i];
                        }
                    }
                }
            } else {
                // very large cluster: walk the tokens in index order (no list to sort)
                for (int t = 0; t < sg.n; ++t) {
                    if (cluster_id[sg.base + t] != c) continue;
                    const uint4 v = *(const uint4*)(hb + (size_t)t * hrow + (size_t)e * Elem<HDT>::BYTES);
                    double x[8];
                    Elem<HDT>::widen(v, x);
#pragma unroll
                    for (int i = 0; i < EPL; ++i) acc[i] += x[i];
                }
            }
            // Eq. 10: the mean as sum * (1/m): an fp64 division per element would be most of this
            // kernel's arithmetic, and the result is rounded to the output type right after
            double outv[EPL];
#pragma unroll
            for (int i = 0; i < EPL; ++i) outv[i] = (m_eff == 1) ? acc[i] : (m_eff == 0 ? 0.0 : acc[i] * inv_m);
            StoreOut<ODT>::template put<EPL>(merged + ((size_t)sg.base + c) * (size_t)h * (ODT == PACT_BF16 ? 2 : 4),
                                             (size_t)e, outv, stream != 0);
        }
    }
    if (slots && blockIdx.x == gridDim.x - 1) {
        // every member of a cluster is a kept or a recovered token
        int loc = 0;
        for (int c = tid; c < C; c += 512) loc += cluster_counts[sg.base + c];
        loc = (int)wave_sum_f64((double)loc);
        __syncthreads();
        if (tid == 0) s_n = 0;
        __syncthreads();
        if ((tid & 63) == 0 && loc) atomicAdd(&s_n, loc);
        __syncthreads();
        if (tid == 0) {
            const int q = clamp_count(rep[b].n_kept, sg.n);
            rep[b].n_reincorporated = s_n - q;
            rep[b].n_dropped = sg.n - s_n;
        }
    }
}

template <int HDT>
static int launch_merge_k(const Batch& bt, const Ws& w, const void* hidden, int32_t h,
                          const int32_t* cluster_id, const int32_t* center_idx, pact_report* rep,
                          void* merged, pact_dtype out_dt, const int32_t* cluster_counts, const int32_t* slots,
                          hipStream_t st) {
    // One workgroup per cluster where the grid allows it (a tenth of the workgroups looping over
    // ten clusters each took a third longer: a cluster is a chain of two trips to memory).  The
    // number of clusters is known on the device only; in a batch a third of the longest sample's
    // tokens (the workloads here end with 0.25 .. 0.3 n clusters) saves the dispatch of thousands
    // of workgroups that find nothing to do (8 videos: 113 -> 109 us).
    int gx = bt.n_max < 4096 ? bt.n_max : 4096;
    if (bt.B > 1 && gx > bt.n_max / 3 + 64) gx = bt.n_max / 3 + 64;
    dim3 grid(gx, bt.B);
    // (the member rows are read for the last time and the merged rows are not read again by this
    //  library: both with the streaming hint when the hidden states alone exceed what the
    //  last-level cache keeps)
    const int stream = hidden_streams(bt.total, h, Elem<HDT>::BYTES) ? 1 : 0;
    if (out_dt == PACT_BF16)
        PACT_LAUNCH("merge_mean", (merge_kernel<HDT, PACT_BF16>), grid, dim3(512), st, bt, (const char*)hidden,
                    h, cluster_id, center_idx, rep, cluster_counts, w.offsets, w.members, slots, w.big, (char*)merged, stream);
    else
        PACT_LAUNCH("merge_mean", (merge_kernel<HDT, PACT_F32>), grid, dim3(512), st, bt, (const char*)hidden,
                    h, cluster_id, center_idx, rep, cluster_counts, w.offsets, w.members, slots, w.big, (char*)merged, stream);
    return PACT_OK;
}

// Positions and proportional-attention weights of the merged tokens (Alg. 3 last loop, Eq. 11).
// grid (ceil(n_max/256), B), block 256.
__global__ __launch_bounds__(256) void handoff_kernel(Batch bt, const int32_t* __restrict__ center_idx,
                                                       const int32_t* __restrict__ cluster_counts,
                                                       const pact_report* __restrict__ rep,
                                                       const int32_t* __restrict__ positions,
                                                       int32_t* __restrict__ positions_out,
                                                       float* __restrict__ log_weight) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int C = clamp_count(rep[b].n_centers, sg.n);
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    const int tok = center_idx[sg.base + c];
    positions_out[sg.base + c] = positions ? positions[sg.base + tok] : tok;
    log_weight[sg.base + c] = (float)log((double)cluster_counts[sg.base + c]);
}

int launch_handoff(const Batch& bt, const int32_t* center_idx, const int32_t* cluster_counts,
                   const pact_report* rep, const int32_t* positions, int32_t* positions_out,
                   float* log_weight, hipStream_t st) {
    PACT_LAUNCH("handoff", handoff_kernel, dim3((bt.n_max + 255) / 256, bt.B), dim3(256), st, bt, center_idx,
                cluster_counts, rep, positions, positions_out, log_weight);
    return PACT_OK;
}

int launch_merge(const Batch& bt, const Ws& w, const void* hidden, pact_dtype h_dt, int32_t h,
                 const int32_t* cluster_id, const int32_t* center_idx, pact_report* rep,
                 void* merged, pact_dtype out_dt, int32_t* cluster_counts, bool recount,
                 hipStream_t st) {
    // recount: a stand-alone merge, which has cluster_id alone to go by: member lists by a pass of
    // their own.  Otherwise the clustering stages have noted sizes, first members and large clusters.
    if (recount) {
        const size_t lds = (size_t)((bt.n_max + 63) / 64 * 64) * sizeof(int);
        static size_t raised = 0;
        if (lds > 48 * 1024 && lds > raised) {
            if (hipFuncSetAttribute((const void*)scan_fill_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds) != hipSuccess)
                return PACT_ERR_HIP;
            raised = lds;
        }
        PACT_LAUNCH_SHMEM("scan_fill", scan_fill_kernel, dim3(bt.B), dim3(1024), lds, st, bt, cluster_id,
                          rep, cluster_counts, 1, 0, w.offsets, w.members, w.big);
    }
    const int32_t* slots = recount ? nullptr : w.slots;
    if (h_dt == PACT_BF16)
        return launch_merge_k<PACT_BF16>(bt, w, hidden, h, cluster_id, center_idx, rep, merged, out_dt,
                                         cluster_counts, slots, st);
    return launch_merge_k<PACT_F32>(bt, w, hidden, h, cluster_id, center_idx, rep, merged, out_dt,
                                    cluster_counts, slots, st);
}

}  // namespace pact

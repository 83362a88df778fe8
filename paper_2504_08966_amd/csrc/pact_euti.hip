// EUTI (Alg. 1): global query (Eq. 1), importance score (Eq. 2), percentile split (Eq. 3/4).
// All arithmetic of the score is fp64 (the stage is bound by reading H from HBM, the ALU work
// is free), rounded once to fp32; the split then compares fp32 bit patterns exactly.
#include "pact_internal.h"

namespace pact {

// ------------------------------------------------------------------------------------------
// Eq. 1, pass 1: column sums of the queries of one row chunk.  grid (QG_CHUNKS, B), block 256.
// Each thread owns groups of 4 consecutive columns; partial sums go to qg_part[b][chunk][col].
template <int DT>
__global__ __launch_bounds__(256) void qglobal_partial_kernel(Batch bt, const char* __restrict__ q,
                                                               int qcols, double* __restrict__ qg_part) {
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int chunk = blockIdx.x;
    const int rows_per = (sg.n + QG_CHUNKS - 1) / QG_CHUNKS;
    const int r0 = chunk * rows_per;
    const int r1 = min(sg.n, r0 + rows_per);
    const size_t row_bytes = (size_t)qcols * Elem<DT>::BYTES;
    double* out = qg_part + ((size_t)b * QG_CHUNKS + chunk) * qcols;
    for (int c = threadIdx.x * 4; c < qcols; c += 256 * 4) {
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        for (int r = r0; r < r1; ++r) {
            const char* p = q + (size_t)(sg.base + r) * row_bytes + (size_t)c * Elem<DT>::BYTES;
            float f[4];
            if (DT == PACT_BF16) {
                const uint2 v = *(const uint2*)p;
                f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
                f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
            } else {
                const float4 v = *(const float4*)p;
                f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += (double)f[i];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) out[c + i] = acc[i];
    }
}

// Eq. 1, pass 2: sum the chunk partials in chunk order and divide by n.  grid (ceil(qcols/256), B).
__global__ __launch_bounds__(256) void qglobal_final_kernel(Batch bt, int qcols,
                                                            const double* __restrict__ qg_part,
                                                            double* __restrict__ qg) {
    const int b = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= qcols) return;
    const double* in = qg_part + (size_t)b * QG_CHUNKS * qcols + c;
    double acc = 0.0;
    for (int k = 0; k < QG_CHUNKS; ++k) acc += in[(size_t)k * qcols];
    qg[(size_t)b * qcols + c] = acc / (double)bt.s[b].n;
}

// Caller supplied the global query ([B, qcols]): widen it to fp64.
template <int DT>
__global__ __launch_bounds__(256) void qglobal_copy_kernel(Batch bt, const char* __restrict__ q, int qcols,
                                                            double* __restrict__ qg) {
    const int b = blockIdx.y;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= qcols) return;
    const char* p = q + ((size_t)b * qcols + c) * Elem<DT>::BYTES;
    float f;
    if (DT == PACT_BF16) f = __uint_as_float((uint32_t)(*(const uint16_t*)p) << 16);
    else f = *(const float*)p;
    qg[(size_t)b * qcols + c] = (double)f;
}

// ------------------------------------------------------------------------------------------
// Eq. 2, pass 1: one wavefront per token computes |h_i|_2 and the n_q logits
// k_i^(g(j)) . Qg^(j); the workgroup (16 tokens) then leaves one online-softmax partial
// (max, sum of exp) per head.  grid (ceil(n_max/16), B), block 256.
template <int HDT, int KDT>
__global__ __launch_bounds__(256) void score_logits_kernel(Batch bt, const char* __restrict__ hidden, int h,
                                                            const char* __restrict__ keys, int n_kv, int d_h,
                                                            int n_q, const double* __restrict__ qg,
                                                            double* __restrict__ logits,
                                                            double* __restrict__ hnorm,
                                                            double* __restrict__ sm_part) {
    __shared__ double s_l[SCORE_TOK_PER_WG][PACT_MAX_QHEADS];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t0 = blockIdx.x * SCORE_TOK_PER_WG;
    if (t0 >= sg.n) return;
    const int qcols = n_q * d_h;
    const int rep = n_q / n_kv;
    const double* qgb = qg + (size_t)b * qcols;
    const size_t hrow = (size_t)h * Elem<HDT>::BYTES;
    const size_t krow = (size_t)n_kv * d_h * Elem<KDT>::BYTES;

    for (int tt = wave; tt < SCORE_TOK_PER_WG; tt += 4) {
        const int i = t0 + tt;
        if (i >= sg.n) break;
        const size_t g = (size_t)sg.base + i;
        // hidden-state norm
        const char* hp = hidden + g * hrow;
        double ss = 0.0;
        for (int e = lane * Elem<HDT>::EPL; e < h; e += 64 * Elem<HDT>::EPL) {
            const uint4 v = *(const uint4*)(hp + (size_t)e * Elem<HDT>::BYTES);
            double x[8];
            Elem<HDT>::widen(v, x);
#pragma unroll
            for (int k = 0; k < Elem<HDT>::EPL; ++k) ss = fma(x[k], x[k], ss);
        }
        ss = wave_sum_f64(ss);
        // per-head logits
        const char* kp = keys + g * krow;
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
                s_l[tt][j] = acc;
            }
        }
        if (lane == 0) hnorm[g] = sqrt(ss);
    }
    __syncthreads();
    if (threadIdx.x < n_q) {
        const int j = threadIdx.x;
        const int cnt = min(SCORE_TOK_PER_WG, sg.n - t0);
        double m = s_l[0][j];
        for (int t = 1; t < cnt; ++t) m = fmax(m, s_l[t][j]);
        double s = 0.0;
        for (int t = 0; t < cnt; ++t) s += exp(s_l[t][j] - m);
        const int smwg = (bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
        double* out = sm_part + (((size_t)b * smwg + blockIdx.x) * n_q + j) * 2;
        out[0] = m;
        out[1] = s;
    }
}

// Eq. 2, pass 2: combine the partials into (max, normaliser) per head, then
// s_i = |h_i| * (1/n_q) sum_j exp(l_ij - M_j) / Z_j.  grid (ceil(n_max/256), B), block 256.
__global__ __launch_bounds__(256) void score_final_kernel(Batch bt, int n_q,
                                                          const double* __restrict__ logits,
                                                          const double* __restrict__ hnorm,
                                                          const double* __restrict__ sm_part,
                                                          float* __restrict__ scores) {
    __shared__ double s_M[PACT_MAX_QHEADS], s_Z[PACT_MAX_QHEADS];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    if (blockIdx.x * 256 >= sg.n) return;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int smwg = (bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    const int nwg = (sg.n + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG;
    for (int j = wave; j < n_q; j += 4) {
        const double* part = sm_part + ((size_t)b * smwg * n_q + j) * 2;
        double m = -INFINITY;
        for (int w = lane; w < nwg; w += 64) m = fmax(m, part[(size_t)w * n_q * 2]);
        m = wave_max_f64(m);
        double z = 0.0;
        for (int w = lane; w < nwg; w += 64)
            z += part[(size_t)w * n_q * 2 + 1] * exp(part[(size_t)w * n_q * 2] - m);
        z = wave_sum_f64(z);
        if (lane == 0) { s_M[j] = m; s_Z[j] = z; }
    }
    __syncthreads();
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= sg.n) return;
    const size_t g = (size_t)sg.base + i;
    double acc = 0.0;
    for (int j = 0; j < n_q; ++j) acc += exp(logits[g * n_q + j] - s_M[j]) / s_Z[j];
    scores[g] = (float)(hnorm[g] * (acc / (double)n_q));
}

// ------------------------------------------------------------------------------------------
// Eq. 3/4: exact radix select of the (m+1)-th smallest fp32 score, then an ordered
// compaction into kept / pruned index lists.  One workgroup of 1024 per sample.
__device__ __forceinline__ uint32_t ordered_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(1024) void prune_kernel(Batch bt, const float* __restrict__ scores,
                                                     int32_t* __restrict__ kept_idx,
                                                     int32_t* __restrict__ pruned_idx,
                                                     pact_report* __restrict__ rep) {
    __shared__ int s_hist[256];
    __shared__ int s_digit, s_newk;
    __shared__ int s_wtot[16];
    const int b = blockIdx.x;
    const Seg sg = bt.s[b];
    const int n = sg.n;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const float* s = scores + sg.base;

    int k = (int)floor((double)sg.lambda * (double)n);
    if (k > n - 1) k = n - 1;
    if (k < 0) k = 0;
    uint32_t prefix = 0, mask = 0;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) s_hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += 1024) {
            const uint32_t u = ordered_key(s[i]);
            if ((u & mask) == prefix) atomicAdd(&s_hist[(u >> shift) & 255], 1);
        }
        __syncthreads();
        if (tid < 64) {
            const int c0 = s_hist[4 * tid], c1 = s_hist[4 * tid + 1];
            const int c2 = s_hist[4 * tid + 2], c3 = s_hist[4 * tid + 3];
            const int loc = c0 + c1 + c2 + c3;
            int inc = loc;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int v = __shfl_up(inc, d, 64);
                if (lane >= d) inc += v;
            }
            int e = inc - loc;   // scores with a smaller digit in earlier bins
            const int c[4] = {c0, c1, c2, c3};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                if (k >= e && k < e + c[t]) { s_digit = 4 * tid + t; s_newk = k - e; }
                e += c[t];
            }
        }
        __syncthreads();
        prefix |= (uint32_t)s_digit << shift;
        mask |= 255u << shift;
        k = s_newk;
        __syncthreads();
    }
    const uint32_t tau = prefix;

    const int chunk = (n + 1023) / 1024;
    const int i0 = min(n, tid * chunk);
    const int i1 = min(n, i0 + chunk);
    int cnt = 0;
    for (int i = i0; i < i1; ++i) cnt += ordered_key(s[i]) >= tau;
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
    int kp = woff + inc - cnt;
    int pp = i0 - kp;
    int32_t* ko = kept_idx + sg.base;
    int32_t* po = pruned_idx + sg.base;
    for (int i = i0; i < i1; ++i) {
        if (ordered_key(s[i]) >= tau) ko[kp++] = i;
        else po[pp++] = i;
    }
    if (tid == 0) {
        rep[b].n_kept = total;
        rep[b].n_pruned = n - total;
    }
}

// ------------------------------------------------------------------------------------------
template <int HDT>
static int launch_logits_k(const Batch& bt, const Ws& w, const ScoreIn& in, hipStream_t st) {
    dim3 grid((bt.n_max + SCORE_TOK_PER_WG - 1) / SCORE_TOK_PER_WG, bt.B);
    if (in.k_dt == PACT_BF16)
        PACT_LAUNCH("score_logits", (score_logits_kernel<HDT, PACT_BF16>), grid, dim3(256), st, bt,
                    (const char*)in.hidden, in.h, (const char*)in.keys_pre, in.n_kv, in.d_h, in.n_q,
                    w.qg, w.logits, w.hnorm, w.sm_part);
    else
        PACT_LAUNCH("score_logits", (score_logits_kernel<HDT, PACT_F32>), grid, dim3(256), st, bt,
                    (const char*)in.hidden, in.h, (const char*)in.keys_pre, in.n_kv, in.d_h, in.n_q,
                    w.qg, w.logits, w.hnorm, w.sm_part);
    return PACT_OK;
}

int launch_score(const Batch& bt, const Ws& w, const ScoreIn& in, float* scores, hipStream_t st) {
    const int qcols = in.n_q * in.d_h;
    if (in.q_per_token) {
        if (in.q_dt == PACT_BF16)
            PACT_LAUNCH("qglobal_partial", qglobal_partial_kernel<PACT_BF16>, dim3(QG_CHUNKS, bt.B),
                        dim3(256), st, bt, (const char*)in.q, qcols, w.qg_part);
        else
            PACT_LAUNCH("qglobal_partial", qglobal_partial_kernel<PACT_F32>, dim3(QG_CHUNKS, bt.B),
                        dim3(256), st, bt, (const char*)in.q, qcols, w.qg_part);
        PACT_LAUNCH("qglobal_final", qglobal_final_kernel, dim3((qcols + 255) / 256, bt.B), dim3(256),
                    st, bt, qcols, w.qg_part, w.qg);
    } else {
        if (in.q_dt == PACT_BF16)
            PACT_LAUNCH("qglobal_copy", qglobal_copy_kernel<PACT_BF16>, dim3((qcols + 255) / 256, bt.B),
                        dim3(256), st, bt, (const char*)in.q, qcols, w.qg);
        else
            PACT_LAUNCH("qglobal_copy", qglobal_copy_kernel<PACT_F32>, dim3((qcols + 255) / 256, bt.B),
                        dim3(256), st, bt, (const char*)in.q, qcols, w.qg);
    }
    int rc = (in.h_dt == PACT_BF16) ? launch_logits_k<PACT_BF16>(bt, w, in, st)
                                    : launch_logits_k<PACT_F32>(bt, w, in, st);
    if (rc != PACT_OK) return rc;
    PACT_LAUNCH("score_final", score_final_kernel, dim3((bt.n_max + 255) / 256, bt.B), dim3(256), st,
                bt, in.n_q, w.logits, w.hnorm, w.sm_part, scores);
    return PACT_OK;
}

int launch_prune(const Batch& bt, const float* scores, int32_t* kept_idx, int32_t* pruned_idx,
                 pact_report* rep, hipStream_t st) {
    PACT_LAUNCH("prune_select", prune_kernel, dim3(bt.B), dim3(1024), st, bt, scores, kept_idx,
                pruned_idx, rep);
    return PACT_OK;
}

}  // namespace pact

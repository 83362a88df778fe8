// DBDPC after the Gram pass (Alg. 2): density order, centre selection under the bound d_c
// done in parallel rounds (same centres as the sequential loop; cf. the recursive scheme of
// appendix D), nearest-centre assignment; and the recovery of pruned tokens (Eq. 8/9).
//
// Centre selection.  Token j "precedes" i when rho_j > rho_i, or rho_j == rho_i and j < i
// (the stable descending density order of Alg. 2).  Alg. 2 makes i a centre iff no centre
// that precedes it lies within d_c.  With adj[i][j] = (d_ij <= d_c) this is a fixed point
// every token can evaluate on its own from its list of preceding neighbours:
//     a preceding neighbour is a centre            -> i is not a centre
//     every preceding neighbour is known not to be -> i is a centre
// A round evaluates this for all undecided tokens at once; the densest undecided token is
// always decided, so the rounds terminate, and the result does not depend on how stale the
// statuses read within a round are.
#include <cstring>

#include "pact_internal.h"

namespace pact {

constexpr int KP = PRED_CAP - 1;   // preceding neighbours kept per token (slot 0 holds the count); more -> bitmap fallback

__device__ __forceinline__ int lanes_below(uint64_t mask, int lane) {
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// A clustering key whose squared norm is zero, or not a finite number, is counted in the report.
__device__ __forceinline__ void note_odd_norm(pact_report* rp, double nn) {
    if (nn > 0.0 && nn < INFINITY) return;
    if (nn == 0.0) atomicAdd(&rp->zero_norm_seen, 1);
    else atomicAdd(&rp->nonfinite_seen, 1);
}

__device__ __forceinline__ bool precedes(double rho_j, int j, double rho_i, int i) {
    return rho_j > rho_i || (rho_j == rho_i && j < i);
}

// Nearest of `ncand` candidates (ids in LDS) of one token, by one wavefront; only distances
// < thr compete, ties go to the lower candidate id; (best, bestc) are updated, identical in
// every lane.  tok_of(c) maps a candidate id to its token.
//
// What such a search costs is the conversion of the rows to fp64, so it screens in fp32 first:
//  1. fp32 cosines of all candidates, eight at a time (the wavefront splits into eight groups
//     of 8 lanes, one candidate row each; lane `sub` takes the 16-byte chunks sub, sub + 8, ...
//     of the candidate's row against the token's own, four chunks of either in flight per lane);
//  2. a candidate whose fp32 cosine is more than 2 * margin below the largest one cannot be the
//     nearest (margin bounds the error of an fp32 cosine), so only the others - usually one -
//     are evaluated in fp64, each by the whole wavefront (Eq. 5 as wave_dot64 computes it: a
//     copy of the token's row is at distance exactly 0);
//  3. if a single candidate is left, `complete` says that the call sees all candidates of the
//     token, and its fp32 cosine is more than margin away from the threshold, it is decided
//     without fp64: `best` is then only a placeholder that no other call will be compared with.
template <int DT, typename TokOf>
__device__ __forceinline__ void nearest_candidate(lds_i32* cand, lds_i32* ctok, lds_f32* ccos, int ncand,
                                                  bool complete, const char* mine, double nnp,
                                                  const char* kb, size_t row_bytes, const double* nnb,
                                                  int dk, int lane, double thr, float margin, TokOf tok_of,
                                                  double& best, int& bestc) {
    constexpr int EPL = Elem<DT>::EPL;
    const int grp = lane >> 3, sub = lane & 7;
    const int nchunk = dk / EPL;                       // 16-byte chunks per row (rows are 16-byte multiples)
    // the tokens of all candidates in one round trip (not one per batch of eight)
    for (int i = lane; i < ncand; i += 64) ctok[i] = tok_of(cand[i]);
    // 1. fp32 cosines
    float top = -INFINITY;
    for (int c0 = 0; c0 < ncand; c0 += 8) {
        const int ci = c0 + grp;
        const bool valid = ci < ncand;
        const int tok = ctok[valid ? ci : c0];
        const char* rb = kb + (size_t)tok * row_bytes;
        const double nnc = nnb[tok];
        float acc = 0.0f;
        for (int k0 = sub; k0 < nchunk; k0 += 32) {    // 4 chunks of either row per lane per pass
            uint4 vb[4], va[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int k = k0 + 8 * u;
                const size_t o = (size_t)(k < nchunk ? k : k0) * 16;
                vb[u] = *(const uint4*)(rb + o);
                va[u] = *(const uint4*)(mine + o);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (k0 + 8 * u < nchunk) {
                    float a[8], x[8];
                    Elem<DT>::widenf(va[u], a);
                    Elem<DT>::widenf(vb[u], x);
#pragma unroll
                    for (int i = 0; i < EPL; ++i) acc = fmaf(a[i], x[i], acc);
                }
            }
        }
        acc = group_sum_f32<8>(acc);
        const double den = sqrt(nnp * nnc);
        float cv = den > 0.0 ? (float)((double)acc / den) : 0.0f;
        if (valid && sub == 0) ccos[ci] = cv;
        if (!valid) cv = -INFINITY;
        // (the eight lanes of a candidate hold the same value: the other candidate of the row of 16 through a rotation)
        cv = fmaxf(cv, dpp_f32<0x128>(cv));                  // row_ror:8
#pragma unroll
        for (int s = 16; s <= 32; s <<= 1) cv = fmaxf(cv, __shfl_xor(cv, s, 64));
        top = fmaxf(top, cv);
    }
    // 2. the candidates that can still be the nearest, compacted in place (order kept)
    const float floor32 = top - 2.0f * margin;
    int na = 0;
    for (int i0 = 0; i0 < ncand; i0 += 64) {
        const int i = i0 + lane;
        const bool amb = i < ncand && ccos[i] >= floor32;
        const int c = amb ? cand[i] : 0, t = amb ? ctok[i] : 0;
        const uint64_t m = __ballot(amb);
        if (amb) { cand[na + lanes_below(m, lane)] = c; ctok[na + lanes_below(m, lane)] = t; }
        na += __popcll(m);
    }
    // 3. decided by the fp32 screen alone?
    const double cthr = 1.0 - thr;                     // d < thr  <=>  cosine > 1 - thr
    if (complete && na == 1 && (double)top - cthr > (double)margin) {
        best = fmax(1.0 - (double)top, 0.0);
        bestc = cand[0];
        return;
    }
    if ((double)top < cthr - (double)margin) return;   // nothing can pass the threshold
    // fp64 for the rest, two candidates in flight
    for (int k = 0; k < na; k += 2) {
        const int k1 = min(k + 1, na - 1);
        const int c0 = cand[k], c1 = cand[k1];
        const int t0 = ctok[k], t1 = ctok[k1];
        const char* r0 = kb + (size_t)t0 * row_bytes;
        const char* r1 = kb + (size_t)t1 * row_bytes;
        const double n0 = nnb[t0], n1 = nnb[t1];
        double a0 = 0.0, a1 = 0.0;
        for (int e = lane * EPL; e < dk; e += 64 * EPL) {
            const size_t o = (size_t)e * Elem<DT>::BYTES;
            const uint4 va = *(const uint4*)(mine + o);
            const uint4 v0 = *(const uint4*)(r0 + o);
            const uint4 v1 = *(const uint4*)(r1 + o);
            double a[8], x[8];
            Elem<DT>::widen(va, a);
            Elem<DT>::widen(v0, x);
#pragma unroll
            for (int i = 0; i < EPL; ++i) a0 = fma(a[i], x[i], a0);
            Elem<DT>::widen(v1, x);
#pragma unroll
            for (int i = 0; i < EPL; ++i) a1 = fma(a[i], x[i], a1);
        }
        const double d0 = cos_dist64(wave_sum_f64(a0), nnp, n0);
        const double d1 = cos_dist64(wave_sum_f64(a1), nnp, n1);
        if (d0 < thr && (d0 < best || (d0 == best && c0 < bestc))) { best = d0; bestc = c0; }
        if (k1 != k && d1 < thr && (d1 < best || (d1 == best && c1 < bestc))) { best = d1; bestc = c1; }
    }
}

// ------------------------------------------------------------------------------------------
// After the density Gram pass, two independent jobs in one launch:
//   blocks [0, REFINE_BLOCKS): the pairs the epilogue could not decide in fp32 - evaluate
//       Eq. 5 in fp64 and clear the bit if the distance exceeds d_c (one wavefront per pair);
//   the other blocks: Eq. 6 completed, rho_p = sum over the row blocks of the column
//       partials (64 tokens x 4 slices per block).  With d_n = 2 every term is an fp32 value
//       in [e^-1, 1], so these fp64 additions are exact whatever their order; for other d_n they
//       are rounded, in an order that is fixed for a given shape (no atomics anywhere), and
//       the order of close densities is settled in fp64 further down the line anyway.
constexpr int REFINE_BLOCKS = 768;     // 3072 wavefronts: one pair each on the benchmark image (2 200 pairs), so that no
                                       // wavefront evaluates two or three rows one after the other (256: 1.2 us longer)

template <int DT>
__global__ __launch_bounds__(256) void post_gram_kernel(Batch bt, const char* __restrict__ keys, int dk,
                                                         const int32_t* __restrict__ idx,
                                                         const double* __restrict__ nn,
                                                         const uint32_t* __restrict__ near_list,
                                                         const int32_t* __restrict__ near_cnt,
                                                         const uint32_t* __restrict__ far_bits, int far_words,
                                                         uint64_t* adj, pact_report* rep,
                                                         const double* __restrict__ rho_part,
                                                         double* __restrict__ rho, double* rho_opt) {
    __shared__ double s_p[4][64];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if (blockIdx.x < REFINE_BLOCKS) {
        const int gw = blockIdx.x * 4 + wave;
        const int nw = REFINE_BLOCKS * 4;
        const uint32_t raw = (uint32_t)near_cnt[2 * b];
        const int cnt = (int)min(raw, (uint32_t)NEAR_CAP);
        if (gw == 0) {
            // largest key distance: the wavefronts of the density pass each left the bits of their
            // most negative exponent -(d / d_n) log2(e); negative floats order like those bits
            uint32_t fb = 0u;
            for (int k = lane; k < far_words; k += 64) fb = max(fb, far_bits[(size_t)b * far_words + k]);
#pragma unroll
            for (int sft = 32; sft >= 1; sft >>= 1) fb = max(fb, (uint32_t)__shfl_xor((int)fb, sft, 64));
            if (lane == 0) {
                // (a listed pair that stands for both orders counts twice)
                rep[b].dc_checked_pairs = raw > (uint32_t)NEAR_CAP ? cnt : near_cnt[2 * b + 1];
                rep[b].refine_overflow = raw > (uint32_t)NEAR_CAP;
                rep[b].max_key_distance = fb ? fminf(-__uint_as_float(fb) * sg.d_n * 0.6931471805599453f, 2.0f) : 0.0f;
            }
        }
        const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
        const char* kb = keys + (size_t)sg.base * row_bytes;
        const int32_t* ix = idx + sg.base;
        const double* nnb = nn + sg.base;
        const double d_c = (double)sg.d_c;
        int ties = 0;
        // lane l takes this wavefront's l-th pair (gw + l * nw): pair, tokens and norms of all of
        // them arrive in three trips, whatever their number; then one trip per pair for the rows
        static_assert(NEAR_CAP <= 64 * REFINE_BLOCKS * 4, "a wavefront's pairs fit its lanes");
        const int my_e = gw + lane * nw;
        uint32_t my_pi = 0, my_pj = 0;
        int my_ti = 0, my_tj = 0;
        double my_ni = 0.0, my_nj = 0.0;
        if (my_e < cnt) {
            const uint2 pr = *(const uint2*)(near_list + ((size_t)b * NEAR_CAP + my_e) * 2);
            my_pi = pr.x; my_pj = pr.y;
            my_ti = ix[my_pi & ~NEAR_MIRROR]; my_tj = ix[my_pj];
            my_ni = nnb[my_ti]; my_nj = nnb[my_tj];
        }
        const int mine = (cnt > gw) ? (cnt - gw + nw - 1) / nw : 0;     // pairs of this wavefront
        for (int k = 0; k < mine; ++k) {
            // (k is the same in every lane: scalar lane reads)
            const uint32_t pi_raw = (uint32_t)__builtin_amdgcn_readlane((int)my_pi, k), pj = (uint32_t)__builtin_amdgcn_readlane((int)my_pj, k);
            const uint32_t pi = pi_raw & ~NEAR_MIRROR;
            const bool both = (pi_raw & NEAR_MIRROR) != 0;
            const int ti = __builtin_amdgcn_readlane(my_ti, k), tj = __builtin_amdgcn_readlane(my_tj, k);
            double d = 0.0;
            if (pi != pj) {
                const double dot = wave_dot64<DT>(kb + (size_t)ti * row_bytes, kb + (size_t)tj * row_bytes, dk, lane);
                d = cos_dist64(dot, __shfl(my_ni, k, 64), __shfl(my_nj, k, 64));
            }
            if (lane == 0) {
                if (d > d_c) {
                    atomicAnd((unsigned long long*)&adj[((size_t)b * bt.n_max + pi) * bt.W + (pj >> 6)],
                              ~(1ull << (pj & 63)));
                    if (both)
                        atomicAnd((unsigned long long*)&adj[((size_t)b * bt.n_max + pj) * bt.W + (pi >> 6)],
                                  ~(1ull << (pi & 63)));
                }
                if (fabs(d - d_c) <= 1e-6) ties += both ? 2 : 1;
            }
        }
        if (lane == 0 && ties) atomicAdd(&rep[b].dc_near_ties, ties);
        return;
    }
    const int p0 = (blockIdx.x - REFINE_BLOCKS) * 64;
    const int p = p0 + lane;
    // the first 32 rows of partials are requested before the number of kept tokens is known
    // (they lie inside the workspace for any p < n_max; what is past the last row is masked)
    const double* in = rho_part + (size_t)b * bt.W * bt.n_max + p;
    double v0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int r = wave + 4 * u;
        v0[u] = (p < bt.n_max && r < bt.W) ? in[(size_t)r * bt.n_max] : 0.0;
    }
    const int q = clamp_count(rep[b].n_kept, sg.n);
    if (p0 >= q) return;
    const int nrt = (q + GRAM_RHO_ROWS - 1) / GRAM_RHO_ROWS;
    double acc = 0.0;
    if (p < q) {
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += (wave + 4 * u < nrt) ? v0[u] : 0.0;
        for (int r0 = wave + 32; r0 < nrt; r0 += 32) {
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int r = r0 + 4 * u;
                v[u] = (r < nrt) ? in[(size_t)r * bt.n_max] : 0.0;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
    }
    s_p[wave][lane] = acc;
    __syncthreads();
    if (wave == 0 && p < q) {
        const double t = (s_p[0][lane] + s_p[1][lane]) + (s_p[2][lane] + s_p[3][lane]);
        rho[(size_t)b * bt.n_max + p] = t;
        if (rho_opt) rho_opt[sg.base + p] = t;
    }
}

// Optional output: position of every kept token in the density order, by enumeration.
// grid (ceil(n_max/64), B), block 1024 = 64 tokens x 16 slices of the j range.
__global__ __launch_bounds__(1024) void rank_kernel(Batch bt, const pact_report* __restrict__ rep,
                                                    const double* __restrict__ rho, int32_t* rank_opt) {
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
    for (int j = j0; j < j1; ++j) cnt += precedes(r[j], j, mine, p);
    s_cnt[slice][lane] = cnt;
    __syncthreads();
    if (threadIdx.x < 64 && p < q) {
        int tot = 0;
#pragma unroll
        for (int s = 0; s < 16; ++s) tot += s_cnt[s][lane];
        rank_opt[bt.s[b].base + p] = tot;
    }
}

// ------------------------------------------------------------------------------------------
// Lock-step extraction of the set bits of one 64-bit word per lane: each call of `step`
// pops at most one bit per lane and reports, wave-wide, how many lanes popped one.
struct BitPop {
    uint64_t word;
    __device__ __forceinline__ bool any() const { return __any(word != 0ull); }
    // returns true if this lane popped bit `bit`
    __device__ __forceinline__ bool pop(int& bit) {
        const bool has = word != 0ull;
        bit = has ? __builtin_ctzll(word) : 0;
        if (has) word &= word - 1;
        return has;
    }
};

// Density order between neighbours (Alg. 2 sorts by density; only the order of tokens within
// d_c of each other can change which of them becomes a centre).  The densities summed by the
// matrix pass are fp64 sums of fp32 terms: each term carries the rounding of its exponent
// (matrix-core accumulation, scaling products, one fused multiply-add; a = log2(e) / d_n is the
// factor that turns a cosine error into an exponent error) and of the hardware exponential,
// independent from term to term, so the error of a sum grows like the square root of the number
// of terms that matter.  Measured against fp64 on 7290-token images: standard error of the
// difference of two neighbours' densities 2.1e-6 at d_n = 2 (rho = 2 400), 4.9e-6 at d_n = 0.5
// (rho = 570), 1.6e-6 at d_n = 8; largest seen 8e-6 / 3.2e-5 / 1.2e-5.  Two neighbours whose
// sums differ by less than
//     2^-20 (1 + 4a) sqrt(max(rho_i, rho_j))          (1.8e-4 / 2.8e-4 / 9.8e-5 for those cases)
// are both listed, and their densities are evaluated again entirely in fp64 before the order
// between them is used.  This is a statistical bound (fifty and more standard errors), not a
// worst-case one: the worst-case error of an fp32 cosine would list half the tokens of an image.
__device__ __forceinline__ double recheck_band2(float d_n) {
    const double a = 1.4426950408889634 / (double)d_n;
    const double c = (1.0 / 1048576.0) * (1.0 + 4.0 * a);
    return c * c;                          // compared with (rho_i - rho_j)^2 / max(rho_i, rho_j)
}

// For every kept token: the list of its neighbours (bitmap row) that precede it in the
// density order, as 16-bit positions in slots 1..KP of its PRED_CAP-slot record; slot 0 holds
// the list length, or KP+1 if the list did not fit (the token is then evaluated from its
// bitmap row).  The first four slots are also written to the token's 8-byte head: most tokens
// have at most three preceding neighbours, and the kernel that runs the rounds - a single
// workgroup - then has 8 bytes per token to fetch instead of 32.
// One wavefront per kept token p.  `odd` counts, wave-wide, the neighbours whose density is
// too close to this token's: DETECT: inside the band above; otherwise (second pass, on fp64
// densities): lower-numbered neighbours with a different density within 1e-11 of the sum.
constexpr int HEAD_PREDS = 3;
constexpr int PREDS_SPREAD = 256;      // set bits of 64 row words that are spread over the lanes through LDS
template <bool DETECT>
__device__ __forceinline__ int preds_of_row(int p, int q, const double* r, const uint64_t* row, uint16_t* out,
                                            uint16_t* head, volatile uint16_t* nb, int lane, double band2) {
    const double rp = r[p];
    const int Wq = (q + 63) >> 6;
    int total = 0, odd = 0;
    auto too_close = [&](bool has, int j, double rj) __attribute__((always_inline)) {
        const double d = rj - rp;
        if constexpr (DETECT) return has && j < q && j != p && d * d <= band2 * fmax(rj, rp);
        else return has && j < p && d != 0.0 && fabs(d) <= 1e-11 * (rj + rp);
    };
    // A token's neighbours are mostly close to it in the sequence, i.e. their bits sit in one or
    // two words of the row: lane by lane, a word's bits would be looked up one after the other,
    // each look-up (the neighbour's density) a trip to memory.  So the set bits of 64 words are
    // first spread over the lanes - the k-th set bit to lane k, through a small LDS list - and
    // the densities of up to 64 neighbours are fetched in one trip.
    for (int w0 = 0; w0 < Wq; w0 += 64) {
        const int w = w0 + lane;
        uint64_t word = (w < Wq) ? row[w] : 0ull;
        const int cnt = __popcll(word);
        const int inc = wave_scan_incl_i32(cnt);
        const int nbits = lane63_of(inc);
        if (nbits <= PREDS_SPREAD) {
            int at = inc - cnt;
            while (word) {                                   // (no memory access in this loop)
                nb[at++] = (uint16_t)((w << 6) + __builtin_ctzll(word));
                word &= word - 1;
            }
            __builtin_amdgcn_wave_barrier();
            for (int k0 = 0; k0 < nbits; k0 += 64) {        // (wave-uniform trip count)
                const int k = k0 + lane;
                const bool has = k < nbits;
                const int j = has ? nb[k] : p;
                const double rj = r[j < q ? j : p];
                const bool pre = has && j < q && precedes(rj, j, rp, p);
                const uint64_t m = __ballot(pre);
                const int slot = total + lanes_below(m, lane);
                if (pre && slot < KP) out[1 + slot] = (uint16_t)j;
                if (pre && slot < HEAD_PREDS) head[1 + slot] = (uint16_t)j;
                total += __popcll(m);
                odd += __popcll(__ballot(too_close(has, j, rj)));
            }
            __builtin_amdgcn_wave_barrier();                 // the list is rewritten for the next 64 words
        } else {
            // a very dense row: word by word, one bit per lane and turn
            BitPop bp{word};
            while (bp.any()) {
                int bit;
                const bool has = bp.pop(bit);
                const int j = (w << 6) + bit;
                const double rj = r[(has && j < q) ? j : p];
                const bool pre = has && j < q && precedes(rj, j, rp, p);
                const uint64_t m = __ballot(pre);
                const int slot = total + lanes_below(m, lane);
                if (pre && slot < KP) out[1 + slot] = (uint16_t)j;
                if (pre && slot < HEAD_PREDS) head[1 + slot] = (uint16_t)j;
                total += __popcll(m);
                odd += __popcll(__ballot(too_close(has, j, rj)));
            }
        }
    }
    if (lane == 0) {
        const uint16_t c = (uint16_t)(total > KP ? KP + 1 : total);
        out[0] = c;
        head[0] = c;
    }
    return odd;
}

// grid (ceil(n_max/4), B), block 256: one wavefront per kept token.  Tokens with a neighbour
// inside the band are appended to the sample's list, as position | token << 16 (tie_cnt[4b]
// counts them, also past the list's end: the re-evaluation is then skipped and reported).
__global__ __launch_bounds__(256) void build_preds_kernel(Batch bt, const pact_report* __restrict__ rep,
                                                          const uint64_t* __restrict__ adj,
                                                          const double* __restrict__ rho,
                                                          uint16_t* __restrict__ preds,
                                                          uint2* __restrict__ heads,
                                                          const int32_t* __restrict__ idx,
                                                          int32_t* __restrict__ tie_list,
                                                          int32_t* __restrict__ tie_cnt) {
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int p = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int q = clamp_count(rep[b].n_kept, bt.s[b].n);
    if (p >= q) return;
    __shared__ uint16_t s_nb[4][PREDS_SPREAD];
    const int odd = preds_of_row<true>(p, q, rho + (size_t)b * bt.n_max, adj + ((size_t)b * bt.n_max + p) * bt.W,
                                       preds + ((size_t)b * bt.n_max + p) * PRED_CAP,
                                       (uint16_t*)(heads + (size_t)b * bt.n_max + p), s_nb[threadIdx.x >> 6], lane,
                                       recheck_band2(bt.s[b].d_n));
    if (odd && lane == 0) {
        // position and token in one word (both below 2^15), so that the re-evaluation finds the
        // token's key without another look-up
        static_assert(PACT_MAX_TOKENS <= 32768, "two 15-bit numbers per list entry");
        const int slot = atomicAdd(&tie_cnt[4 * b], 1);
        if (slot < RHO_RECHECK_MAX) tie_list[(size_t)b * RHO_RECHECK_MAX + slot] = p | (idx[bt.s[b].base + p] << 16);
    }
}

// Set-up step of the kernel that runs the centre rounds, for a sample with listed tokens: their
// fp64 densities from the partial sums (one wavefront per token), written over the fp32-term
// ones; then their predecessor lists again from the new values.  All wavefronts of the workgroup
// call it; `nb` is a per-wavefront buffer of PREDS_SPREAD entries.
__device__ __forceinline__ void finish_rechecked_densities(const Batch& bt, int b, int q, int T, int wave, int nwaves, int lane,
                                                           const int32_t* list, const double* part_b, double* rho_b,
                                                           double* rho_opt_b, const uint64_t* adj, uint16_t* preds,
                                                           uint2* heads, volatile uint16_t* nb, pact_report* rep) {
    const int nch = (q + RHO_RECHECK_CHUNK - 1) / RHO_RECHECK_CHUNK;
    for (int t = wave; t < T; t += nwaves) {
        double ah = 0.0, al = 0.0;
        for (int c = lane; c < nch; c += 64) {
            const double2 v = *(const double2*)(part_b + ((size_t)t * nch + c) * 2);
            ah += v.x;
            al += v.y;
        }
        const double acc = wave_sum_f64(ah) + wave_sum_f64(al);
        if (lane == 0) {
            const int p = min(list[t] & 0xFFFF, q - 1);
            rho_b[p] = acc;
            if (rho_opt_b) rho_opt_b[p] = acc;
        }
    }
    __syncthreads();                                   // (the values are read back by this workgroup only)
    int fine = 0;
    for (int t = wave; t < T; t += nwaves) {
        const int p = min(list[t] & 0xFFFF, q - 1);
        fine += preds_of_row<false>(p, q, rho_b, adj + ((size_t)b * bt.n_max + p) * bt.W,
                                    preds + ((size_t)b * bt.n_max + p) * PRED_CAP,
                                    (uint16_t*)(heads + (size_t)b * bt.n_max + p), nb, lane, 0.0);
    }
    if (lane == 0 && fine) atomicAdd(&rep[b].rho_near_ties, fine);
    if (wave == 0 && lane == 0) rep[b].rho_rechecked = T;
    __syncthreads();
}

// Status checks of the list positions 1..15 of a predecessor record held in two 16-byte
// pieces; `pm` has bit s-1 set while the predecessor at position s is still undecided
// (positions past the list length never are).  A centre among them blocks the token; the ones
// found not to be centres are dropped from `pm`.
__device__ __forceinline__ bool check_pending15(const uint4& v0, const uint4& v1, uint32_t& pm, lds_vu8* st) {
    const uint32_t wv[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
    bool blocked = false;
#pragma unroll
    for (int s = 1; s < 16; ++s) {
        if (pm & (1u << (s - 1))) {
            const int j = (wv[s >> 1] >> ((s & 1) * 16)) & 0xFFFF;
            const unsigned char sj = st[j];
            blocked |= (sj == ST_CENTER);
            if (sj == ST_NOT) pm &= ~(1u << (s - 1));
        }
    }
    return blocked;
}

// The same re-evaluation on the fp64 matrix instruction, for key rows of whole 64-byte quarters
// (the usual widths).  A work item is (16 listed tokens, 64 kept tokens); each of the workgroup's four
// wavefronts forms the 16 x 16 dot products of the listed tokens with 16 of the kept ones by
// v_mfma_f64_16x16x4_f64: lane l supplies element k of row l % 16 of either operand, k running over
// the quarter l / 16 of the key width (the order of the summands of a dot product is then the same
// for every pair, which is all that the exactness argument above needs: equal rows give equal dot
// products), and receives the products of listed tokens 4 v + l / 16, v = 0..3, with kept token
// l % 16.  Norms are the per-token fp64 norms of the first kernel; everything after the dot product
// is as above, and the partial sums have the same layout.
// grid (blocks per sample, B), block 256.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
template <int DT>
__global__ __launch_bounds__(256) void rho_recheck_mfma_kernel(Batch bt, const char* keys, int dk, const int32_t* idx,
                                                                const double* __restrict__ nn, pact_report* rep, double* part,
                                                                const int32_t* tie_list, const int32_t* tie_cnt) {
    __shared__ double s_hi[4][16], s_lo[4][16];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int T = tie_cnt[4 * b];                      // (the same for every workgroup of the sample)
    const int q = clamp_count(rep[b].n_kept, sg.n);
    if (T <= 0) return;
    if (T > RHO_RECHECK_MAX) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&rep[b].refine_overflow, OVERFLOW_RHO_RECHECK);
        return;
    }
    constexpr int EPL = Elem<DT>::EPL;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nch = (q + RHO_RECHECK_CHUNK - 1) / RHO_RECHECK_CHUNK;
    const int nrt = (T + 15) >> 4;
    const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
    const int qchunks = (int)(row_bytes / 64);          // 16-byte chunks per quarter of a row
    const char* kb = keys + (size_t)sg.base * row_bytes;
    const double* nnb = nn + sg.base;
    const int32_t* ix = idx + sg.base;
    const int32_t* list = tie_list + (size_t)b * RHO_RECHECK_MAX;
    double* part_b = part + (size_t)b * 2 * rho_fix_tokens(bt.n_max) * rho_fix_chunks(bt.n_max);   // [T][nch][2]
    const double d_n = (double)sg.d_n;
    const int i16 = lane & 15, kq = lane >> 4;
    for (int item = blockIdx.x; item < nrt * nch; item += gridDim.x) {
        const int rt = item / nch, c = item - rt * nch;
        // this lane's row of either operand: listed token 16 rt + i16, kept token 64 c + 16 wave + i16
        const int t_mine = rt * 16 + i16;
        const int ent = list[min(t_mine, T - 1)];
        const int p_mine = min(ent & 0xFFFF, q - 1), tokA = min(max(ent >> 16, 0), sg.n - 1);
        const int pk_mine = c * RHO_RECHECK_CHUNK + wave * 16 + i16;
        const int tokB = ix[min(pk_mine, q - 1)];
        const double nnA = nnb[tokA], nnB = nnb[tokB];
        const char* ra = kb + (size_t)tokA * row_bytes + (size_t)kq * (row_bytes / 4);
        const char* rb = kb + (size_t)tokB * row_bytes + (size_t)kq * (row_bytes / 4);
        // eight chunks of either row per trip to memory, the next trip's requested before this one's are multiplied;
        // four accumulators, so that an instruction does not wait for the one before it
        constexpr int NBT = 8;
        f64x4_t acc[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] = f64x4_t{0.0, 0.0, 0.0, 0.0};
        uint4 va0[NBT], vb0[NBT], va1[NBT], vb1[NBT];
        auto fetch = [&](uint4 (&va)[NBT], uint4 (&vb)[NBT], int u0) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < NBT; ++u) {
                const size_t o = (size_t)min(u0 + u, qchunks - 1) * 16;
                va[u] = *(const uint4*)(ra + o);
                vb[u] = *(const uint4*)(rb + o);
            }
        };
        auto multiply = [&](const uint4 (&va)[NBT], const uint4 (&vb)[NBT], int u0) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < NBT; ++u) {
                if (u0 + u < qchunks) {                     // (uniform)
                    double a[8], x[8];
                    Elem<DT>::widen(va[u], a);
                    Elem<DT>::widen(vb[u], x);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) acc[e & 3] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[e], x[e], acc[e & 3], 0, 0, 0);
                }
            }
        };
        fetch(va0, vb0, 0);
#pragma unroll 1
        for (int u0 = 0; u0 < qchunks; u0 += 2 * NBT) {
            if (u0 + NBT < qchunks) fetch(va1, vb1, u0 + NBT);
            multiply(va0, vb0, u0);
            if (u0 + 2 * NBT < qchunks) fetch(va0, vb0, u0 + 2 * NBT);
            if (u0 + NBT < qchunks) multiply(va1, vb1, u0 + NBT);
        }
        // products of listed token 4 v + kq (of this tile) with kept token i16: terms, split, sums over the 16 kept tokens
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int src = 4 * v + kq;                     // the lane that holds that listed token's entry
            const int p_t = __shfl(p_mine, src, 64);
            const double nn_t = __shfl(nnA, src, 64);
            const double dot = (acc[0][v] + acc[1][v]) + (acc[2][v] + acc[3][v]);
            const double d = cos_dist64(dot, nn_t, nnB);
            const double term = pk_mine >= q ? 0.0 : (pk_mine == p_t ? 1.0 : exp(-d / d_n));
            double hi = rint(term * 1073741824.0) * (1.0 / 1073741824.0);
            double lo = term - hi;
            hi = group_sum_f64(hi, 16);
            lo = group_sum_f64(lo, 16);
            if (i16 == 0) { s_hi[wave][src] = hi; s_lo[wave][src] = lo; }
        }
        __syncthreads();
        if (tid < 16) {
            const int t = rt * 16 + tid;
            const double vh = (s_hi[0][tid] + s_hi[1][tid]) + (s_hi[2][tid] + s_hi[3][tid]);
            const double vl = (s_lo[0][tid] + s_lo[1][tid]) + (s_lo[2][tid] + s_lo[3][tid]);
            if (t < T) *(double2*)(part_b + ((size_t)t * nch + c) * 2) = make_double2(vh, vl);
        }
        __syncthreads();
    }
}

// All rounds of the centre selection in one workgroup per sample, statuses in LDS; then the
// centres are numbered in ascending token order and published.
//  * The first round needs no look-ups: nothing is decided yet, so exactly the tokens without a
//    preceding neighbour become centres.  It is folded into the set-up.
//  * Tokens with one to HEAD_PREDS preceding neighbours (most of the others) go on a work list of
//    8-byte entries (position and the predecessors that are still undecided).  A round reads the
//    list, looks the predecessors' statuses up, decides what it can and appends the entries that
//    stay undecided - without the predecessors found not to be centres - to the list of the next
//    round (a ballot and one LDS atomic per wavefront): a round costs what is still undecided, not
//    n, and the wavefronts beyond the list's end have nothing to do.  Two lists alternate; they
//    live in LDS (WL_LDS, samples of up to RESOLVE_LDS_TOKENS tokens) or in the workspace.
//  * Tokens with more preceding neighbours are collected in a list of their own; thread i keeps
//    the first 32 bytes of the i-th listed token's record and a bit mask of the predecessors
//    that are still undecided.
//  * Tokens whose list overflowed the record are evaluated from their bitmap row by a whole
//    wavefront.
// grid (B), block 1024, dynamic LDS: (n_max + 64) bytes (status) + n_max * 2 bytes (token
// lists: long lists from the front, overflowed from the back) + W * 4 bytes (centres per word)
// [+ 2 * 8 * n_max bytes of work lists].
constexpr int RESOLVE_CACHED = 4;
constexpr int RESOLVE_LOOKS = 2;         // looks at a work-list entry's predecessors per round (7 -> 5 rounds on a 4000-token image; a third look gains nothing, and two looks at the long lists cost more than the round they save)
typedef uint32_t wl_entry __attribute__((ext_vector_type(2)));      // position | predecessor << 16, two more predecessors (0xFFFF: none)
typedef __attribute__((address_space(3))) wl_entry lds_wl_entry;
template <bool WL_LDS> struct WorkList;
template <> struct WorkList<true> { typedef lds_wl_entry* ptr; };
template <> struct WorkList<false> { typedef wl_entry* ptr; };

template <bool WL_LDS>
__global__ __launch_bounds__(1024) void centre_resolve_kernel(Batch bt, pact_report* rep,
                                                              const uint64_t* __restrict__ adj,
                                                              double* rho, double* rho_opt,
                                                              uint16_t* preds, uint2* heads,
                                                              const int32_t* __restrict__ idx,
                                                              const int32_t* __restrict__ tie_list,
                                                              const int32_t* __restrict__ tie_cnt,
                                                              const double* __restrict__ rho_fix,
                                                              uint32_t* status, int32_t* cnum,
                                                              uint64_t* cmask, int32_t* center_idx, uint2* worklist) {
    extern __shared__ unsigned char s_raw[];
    __shared__ int s_flag[3], s_cnt[3], s_nlong, s_nover;
    __shared__ uint16_t s_nb[16][PREDS_SPREAD];
    const int b = blockIdx.x;
    const Seg sg = bt.s[b];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    // the heads of this thread's first tokens are requested before the number of kept tokens is
    // known (they lie inside the workspace for any position below n_max): one trip less
    uint2 h[RESOLVE_CACHED];
#pragma unroll
    for (int k = 0; k < RESOLVE_CACHED; ++k) {
        const int p = tid + 1024 * k;
        h[k] = (p < bt.n_max) ? heads[(size_t)b * bt.n_max + p] : make_uint2(0, 0);
    }
    const int T = tie_cnt[4 * b];
    const int q = clamp_count(rep[b].n_kept, sg.n);
    if (T > 0 && T <= RHO_RECHECK_MAX) {
        // tokens whose density was evaluated again in fp64: finish those sums and rebuild the
        // lists they decide, then fetch the heads again (some of them are new)
        finish_rechecked_densities(bt, b, q, T, wave, 16, lane, tie_list + (size_t)b * RHO_RECHECK_MAX,
                                   rho_fix + (size_t)b * 2 * rho_fix_tokens(bt.n_max) * rho_fix_chunks(bt.n_max),
                                   rho + (size_t)b * bt.n_max, rho_opt ? rho_opt + sg.base : nullptr, adj, preds, heads,
                                   s_nb[wave], rep);
#pragma unroll
        for (int k = 0; k < RESOLVE_CACHED; ++k) {
            const int p = tid + 1024 * k;
            h[k] = (p < bt.n_max) ? heads[(size_t)b * bt.n_max + p] : make_uint2(0, 0);
        }
    }
    const int qpad = (bt.n_max + 63) / 64 * 64;
    lds_vu8* s_st = (lds_vu8*)s_raw;                             // [qpad + 64]
    lds_u16* s_list = (lds_u16*)(s_raw + qpad + 64);             // [n_max]
    lds_i32* s_wcnt = (lds_i32*)(s_raw + qpad + 64 + (size_t)qpad * 2);   // [W + 1]
    // the two work lists, n_max entries each
    typedef typename WorkList<WL_LDS>::ptr wl_ptr;
    wl_ptr wl[2];
    if constexpr (WL_LDS) {
        const size_t off = ((size_t)qpad + 64 + (size_t)qpad * 2 + ((size_t)bt.W + 1) * 4 + 7) & ~(size_t)7;
        wl[0] = (wl_ptr)(s_raw + off);
        wl[1] = wl[0] + bt.n_max;
    } else {
        wl[0] = (wl_ptr)worklist + (size_t)b * 2 * bt.n_max;
        wl[1] = wl[0] + bt.n_max;
    }
    const double* r = rho + (size_t)b * bt.n_max;
    const uint4* rec = (const uint4*)(preds + (size_t)b * bt.n_max * PRED_CAP);   // 8 pieces per token
    const uint2* hd = heads + (size_t)b * bt.n_max;
    const int Wq = (q + 63) >> 6;
    const int last = bt.n_max - 1;                               // overflow list grows down from here

    if (tid == 0) {
        s_nlong = 0; s_nover = 0;
        s_flag[0] = 0; s_flag[1] = 0; s_flag[2] = 0;
        s_cnt[0] = 0; s_cnt[1] = 0; s_cnt[2] = 0;
    }
    __syncthreads();
    // the token indices this thread will publish at the end (words wave, wave + 16, ...): fetched
    // now, so that the last phase does not start with a trip to memory
    const int32_t* ix = idx + sg.base;
    int pub_ix[RESOLVE_CACHED];
#pragma unroll
    for (int k = 0; k < RESOLVE_CACHED; ++k) {
        const int p = ((wave + 16 * k) << 6) + lane;
        pub_ix[k] = (p < q) ? ix[p] : 0;
    }
    // set-up = round 1, and the three token lists (appended a wavefront at a time)
    auto setup = [&](int p, uint2 hv) __attribute__((always_inline)) {
        const int c = hv.x & 0xFFFF;
        const bool in = p < q;
        if (in) s_st[p] = (c == 0) ? ST_CENTER : ST_UNKNOWN;
        const bool sht = in && c >= 1 && c <= HEAD_PREDS, lng = in && c > HEAD_PREDS && c <= KP, ovr = in && c > KP;
        const uint64_t ms = __ballot(sht), ml = __ballot(lng), mo = __ballot(ovr);
        if (ms) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_cnt[1], __popcll(ms));
            base = lane0_of(base);
            if (sht) {
                // (slots of the head past its count hold nothing)
                const uint32_t j1 = c >= 2 ? (hv.y & 0xFFFFu) : 0xFFFFu, j2 = c >= 3 ? (hv.y >> 16) : 0xFFFFu;
                wl[1][base + lanes_below(ms, lane)] = wl_entry{(uint32_t)p | (hv.x & 0xFFFF0000u), j1 | (j2 << 16)};
            }
        }
        if (ml) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_nlong, __popcll(ml));
            base = lane0_of(base);
            if (lng) s_list[base + lanes_below(ml, lane)] = (uint16_t)p;
        }
        if (mo) {
            int base = 0;
            if (lane == 0) base = atomicAdd(&s_nover, __popcll(mo));
            base = lane0_of(base);
            if (ovr) s_list[last - (base + lanes_below(mo, lane))] = (uint16_t)p;
        }
    };
#pragma unroll
    for (int k = 0; k < RESOLVE_CACHED; ++k) setup(tid + 1024 * k, h[k]);
    for (int p0 = 1024 * RESOLVE_CACHED; p0 < q; p0 += 1024) {      // (wave-uniform trip count)
        const int p = p0 + tid;
        setup(p, p < q ? hd[p] : make_uint2(0, 0));
    }
    __syncthreads();
    const int nlong = s_nlong, nover = s_nover;
    int lp = -1, lc = 0;                                         // this thread's listed token
    uint4 l0 = make_uint4(0, 0, 0, 0), l1 = l0;
    uint32_t pml = 0;
    if (tid < nlong) {
        lp = s_list[tid];
        l0 = rec[(size_t)lp * 8];
        l1 = rec[(size_t)lp * 8 + 1];
        lc = l0.x & 0xFFFF;
        pml = (lc >= 15) ? 0x7FFFu : ((1u << lc) - 1u);
    }
    int rounds = 1;
    // One barrier per round: round r reads the work list r & 1 (s_cnt[r % 3] entries) and appends to the
    // other one (s_cnt[(r + 1) % 3]); it raises s_flag[r % 3] if it leaves a token of the other kinds
    // undecided, and clears the flag and the count of round r + 2 (last read before the previous
    // barrier) on the way.
    while (true) {
        if (tid == 0) { s_flag[(rounds + 1) % 3] = 0; s_cnt[(rounds + 2) % 3] = 0; }
        bool still = false;
        auto decide = [&](int p, bool blocked, bool pending) __attribute__((always_inline)) {
            if (blocked) s_st[p] = ST_NOT;
            else if (!pending) s_st[p] = ST_CENTER;
            else still = true;
        };
        // short lists: the work list
        {
            const int nA = s_cnt[rounds % 3];
            const wl_ptr A = wl[rounds & 1], Bn = wl[(rounds + 1) & 1];
            // (plain reads: the three look-ups of an entry go out together; a status that another
            //  wavefront changes meanwhile is seen in the next round at the latest)
            typedef __attribute__((address_space(3))) unsigned char lds_u8r;
            const lds_u8r* s_rd = (const lds_u8r*)s_st;
            for (int i0 = wave * 64; i0 < nA; i0 += 1024) {              // (wave-uniform trip count)
                const int i = i0 + lane;
                const bool have = i < nA;
                wl_entry e = {0xFFFF0000u, 0xFFFFFFFFu};
                if (have) e = A[i];
                const uint32_t p = e.x & 0xFFFFu;
                uint32_t j[HEAD_PREDS] = {e.x >> 16, e.y & 0xFFFFu, e.y >> 16};
                bool blocked = false, done = !have;
                uint32_t keep[HEAD_PREDS];
                int nk = 0;
                // (RESOLVE_LOOKS looks per round, each followed by what it decides: what the other
                //  wavefronts decide in their first look is there for the second)
#pragma unroll
                for (int look = 0; look < RESOLVE_LOOKS; ++look) {
                    nk = 0;
#pragma unroll
                    for (int t = 0; t < HEAD_PREDS; ++t) keep[t] = 0xFFFFu;
#pragma unroll
                    for (int t = 0; t < HEAD_PREDS; ++t) {
                        const bool real = j[t] != 0xFFFFu;
                        const unsigned char sj = look == 0 ? s_rd[real ? j[t] : 0u] : s_st[real ? j[t] : 0u];
                        blocked |= real && sj == ST_CENTER;
                        if (real && sj == ST_UNKNOWN) {                    // stays on the entry, moved to the front
                            if (nk == 0) keep[0] = j[t];
                            else if (nk == 1) keep[1] = j[t];
                            else keep[2] = j[t];
                            ++nk;
                        }
                    }
#pragma unroll
                    for (int t = 0; t < HEAD_PREDS; ++t) j[t] = keep[t];
                    if (!done) {
                        if (blocked) { s_st[p] = ST_NOT; done = true; }
                        else if (nk == 0) { s_st[p] = ST_CENTER; done = true; }
                    }
                }
                const bool stay = !done;
                const uint64_t m = __ballot(stay);
                if (m) {
                    int base = 0;
                    if (lane == 0) base = atomicAdd(&s_cnt[(rounds + 1) % 3], __popcll(m));
                    base = lane0_of(base);
                    if (stay) Bn[base + lanes_below(m, lane)] = wl_entry{p | (keep[0] << 16), keep[1] | (keep[2] << 16)};
                }
            }
        }
        // long lists: the first 15 positions from registers, the rest of the record from memory
        if (lp >= 0 && s_st[lp] == ST_UNKNOWN) {
            bool blocked = check_pending15(l0, l1, pml, s_st);
            bool pending = pml != 0;
            for (int piece = 2; piece * 8 <= lc && !blocked; ++piece) {
                const uint4 v = rec[(size_t)lp * 8 + piece];
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    if (piece * 8 + t <= lc) {
                        const unsigned char sj = s_st[(wv[t >> 1] >> ((t & 1) * 16)) & 0xFFFF];
                        blocked |= (sj == ST_CENTER);
                        pending |= (sj == ST_UNKNOWN);
                    }
                }
            }
            decide(lp, blocked, pending);
        }
        for (int i = tid + 1024; i < nlong; i += 1024) {                    // more listed tokens than threads
            const int p = s_list[i];
            if (s_st[p] != ST_UNKNOWN) continue;
            const int c = rec[(size_t)p * 8].x & 0xFFFF;
            bool blocked = false, pending = false;
            for (int piece = 0; piece * 8 <= c && !blocked; ++piece) {
                const uint4 v = rec[(size_t)p * 8 + piece];
                const uint32_t wv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int pos = piece * 8 + t;
                    if (pos >= 1 && pos <= c) {
                        const unsigned char sj = s_st[(wv[t >> 1] >> ((t & 1) * 16)) & 0xFFFF];
                        blocked |= (sj == ST_CENTER);
                        pending |= (sj == ST_UNKNOWN);
                    }
                }
            }
            decide(p, blocked, pending);
        }
        for (int o = wave; o < nover; o += 16) {                 // overflowed lists (wave-uniform trip count)
            const int p = s_list[last - o];
            if (s_st[p] != ST_UNKNOWN) continue;
            const double rp = r[p];
            const uint64_t* row = adj + ((size_t)b * bt.n_max + p) * bt.W;
            bool blocked = false, pending = false;
            for (int w0 = 0; w0 < Wq; w0 += 64) {
                const int w = w0 + lane;
                uint64_t word = (w < Wq) ? row[w] : 0ull;
                while (word) {
                    const int bit = __builtin_ctzll(word);
                    word &= word - 1;
                    const int j = (w << 6) + bit;
                    if (j < q && precedes(r[j], j, rp, p)) {
                        const unsigned char sj = s_st[j];
                        blocked |= (sj == ST_CENTER);
                        pending |= (sj == ST_UNKNOWN);
                    }
                }
            }
            blocked = __any(blocked);
            pending = __any(pending);
            if (blocked) { if (lane == 0) s_st[p] = ST_NOT; }
            else if (!pending) { if (lane == 0) s_st[p] = ST_CENTER; }
            else still = true;
        }
        if (still) s_flag[rounds % 3] = 1;
        __syncthreads();
        const int more = s_flag[rounds % 3] | s_cnt[(rounds + 1) % 3];
        ++rounds;
        if (!more) break;
    }
    // Publish: one ballot per 64 tokens gives the centre mask word; the centres are numbered in
    // ascending p (= ascending token index) from the running sum of the words' popcounts.
    uint64_t* cm = cmask + (size_t)b * bt.W;
    for (int w = wave; w < Wq; w += 16) {
        const int p = (w << 6) + lane;
        const uint64_t m = __ballot(p < q && s_st[p] == ST_CENTER);
        if (lane == 0) { cm[w] = m; s_wcnt[w] = __popcll(m); }
    }
    __syncthreads();
    if (wave == 0) {                                          // exclusive scan over the words
        int run = 0;
        for (int w0 = 0; w0 < Wq; w0 += 64) {
            const int w = w0 + lane;
            const int v = (w < Wq) ? s_wcnt[w] : 0;
            const int inc = wave_scan_incl_i32(v);
            if (w < Wq) s_wcnt[w] = run + inc - v;
            run += lane63_of(inc);
        }
        if (lane == 0) s_wcnt[Wq] = run;
    }
    __syncthreads();
    uint32_t* st = status + (size_t)b * bt.n_max;
    int32_t* cn = cnum + (size_t)b * bt.n_max;
    int32_t* co = center_idx + sg.base;
    auto publish_word = [&](int w, int tok, bool have_tok) __attribute__((always_inline)) {
        const int p = (w << 6) + lane;
        const unsigned char sv = (p < q) ? s_st[p] : (unsigned char)ST_NOT;
        const bool isc = sv == ST_CENTER;
        const uint64_t m = __ballot(isc);
        const int c = s_wcnt[w] + lanes_below(m, lane);
        if (p < q) {
            st[p] = sv;
            cn[p] = isc ? c : -1;
            if (isc) co[c] = have_tok ? tok : ix[p];
        }
    };
#pragma unroll
    for (int k = 0; k < RESOLVE_CACHED; ++k)
        if (wave + 16 * k < Wq) publish_word(wave + 16 * k, pub_ix[k], true);
    for (int w = wave + 16 * RESOLVE_CACHED; w < Wq; w += 16) publish_word(w, 0, false);
    if (tid == 0) {
        rep[b].n_centers = s_wcnt[Wq];
        rep[b].rounds = rounds;
    }
}

// ------------------------------------------------------------------------------------------
constexpr int CAND_BUF = 128;

// The two nearest-centre searches share one kernel (below): the assignment of the kept tokens
// needs only the centres, so in the fused path it runs beside the recovery of the pruned tokens
// (whose slowest wavefronts leave most of the chip idle) instead of before the candidate pass.
struct NearArgs {
    pact_report* rep;
    const char* keys; int dk;
    const double* nn;
    const uint64_t* adj;
    float margin;
    int32_t* cluster_id; int32_t* cluster_counts;
    int32_t* slots; int32_t* big;           // (optional) first members per cluster and the list of large clusters
    // assignment of kept tokens (Alg. 2 last loop); assign_blocks == 0: not in this launch
    const int32_t* idx; const uint64_t* cmask; const uint32_t* status; const int32_t* cnum; int assign_blocks;
    // recovery of pruned tokens (Eq. 8/9): the blocks before the assignment ones
    const int32_t* pruned_idx; const int32_t* center_idx; const float* cbest;
};

// Token `tok` joins cluster c (both local to the sample): the cluster's size goes up and, where
// the caller keeps them, the token takes the next of the cluster's member slots; the member that
// makes a cluster a large one puts it on the list of those.  counts/slots/big: the sample's.
__device__ __forceinline__ void join_cluster(const NearArgs& a, pact_report* rp, int base, int c, int tok) {
    const int s = atomicAdd(&a.cluster_counts[base + c], 1);
    if (a.slots) {
        if (s < MERGE_SLOTS) a.slots[(size_t)(base + c) * MERGE_SLOTS + s] = tok;
        if (s == MERGE_BIG - 1) a.big[base + atomicAdd(&rp->reserved[0], 1)] = c;
    }
}

// Alg. 2 last loop: every kept token joins the nearest centre.  Candidates are the centres
// its bitmap row reaches (the nearest centre is within d_c, hence one of them; it need not
// precede the token); with one candidate no distance is needed, otherwise Eq. 5 is
// evaluated (fp32 screen, fp64 where it matters).  One wavefront per kept token, 4 per block.
template <int DT>
__device__ __forceinline__ void assign_body(const Batch& bt, const NearArgs& a, int blk, lds_i32* cand,
                                            lds_i32* ctok, lds_f32* ccos) {
    pact_report* rep = a.rep;
    const char* keys = a.keys;
    const int dk = a.dk;
    const int32_t* idx = a.idx;
    const double* nn = a.nn;
    const uint64_t* adj = a.adj;
    const uint64_t* cmask = a.cmask;
    const uint32_t* status = a.status;
    const int32_t* cnum = a.cnum;
    const float margin = a.margin;
    int32_t* cluster_id = a.cluster_id;
    int32_t* cluster_counts = a.cluster_counts;
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int p = blk * 4 + wave;
    const int q = clamp_count(rep[b].n_kept, sg.n);
    if (p >= q) return;
    const int32_t* ix = idx + sg.base;
    const int32_t* cn = cnum + (size_t)b * bt.n_max;
    const uint32_t* st = status + (size_t)b * bt.n_max;
    const double* nnb = nn + sg.base;
    const uint64_t* row = adj + ((size_t)b * bt.n_max + p) * bt.W;
    const uint64_t* cm = cmask + (size_t)b * bt.W;
    const int tok = ix[p];
    const uint32_t stp = st[p];
    const int cnp = cn[p];
    // (the first 64 words of the row and of the centre mask go out with them, before the status
    //  is looked at: a trip less for the tokens that are not centres)
    const uint64_t first = (lane < bt.W) ? (row[lane] & cm[lane]) : 0ull;
    int cid;
    if (stp == ST_CENTER) {
        cid = cnp;
    } else {
        const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
        const char* kb = keys + (size_t)sg.base * row_bytes;
        const char* mine = kb + (size_t)tok * row_bytes;
        const double nnp = nnb[tok];
        double best = INFINITY;
        int bestj = 0x7FFFFFFF;
        auto tok_of = [&](int j) { return ix[j]; };
        const int Wq = (q + 63) >> 6;
        int nbuf = 0, ntot = 0;
        for (int w0 = 0; w0 < Wq; w0 += 64) {
            const int w = w0 + lane;
            BitPop bp{(w < Wq) ? (w0 == 0 ? first : (row[w] & cm[w])) : 0ull};
            while (bp.any()) {
                int bit;
                const bool has = bp.pop(bit);
                const int j = (w << 6) + bit;
                const bool ok = has && j < q;
                const uint64_t m = __ballot(ok);
                if (ok) cand[nbuf + lanes_below(m, lane)] = j;
                nbuf += __popcll(m);
                ntot += __popcll(m);
                if (nbuf > CAND_BUF - 64) {
                    nearest_candidate<DT>(cand, ctok, ccos, nbuf, false, mine, nnp, kb, row_bytes, nnb, dk,
                                          lane, INFINITY, margin, tok_of, best, bestj);
                    nbuf = 0;
                }
            }
        }
        if (ntot == 1) bestj = cand[0];                 // a single centre in reach: no distance needed
        else if (nbuf) nearest_candidate<DT>(cand, ctok, ccos, nbuf, nbuf == ntot, mine, nnp, kb, row_bytes, nnb,
                                             dk, lane, INFINITY, margin, tok_of, best, bestj);
        cid = bestj != 0x7FFFFFFF ? cn[bestj] : -1;
    }
    if (lane == 0) {
        cluster_id[sg.base + tok] = cid;
        if (cid >= 0 && cluster_counts) join_cluster(a, rep + b, sg.base, cid, tok);
        note_odd_norm(rep + b, nnb[tok]);
    }
}

// Dot product in fp64 of the rows `mine` and `other` by the 16 lanes part = 0..15 of a group
// (lane `part` takes the 16-byte chunks part, part + 16, ...; four chunks of either row in
// flight per lane).  Every lane of the group gets the sum.
template <int DT>
__device__ __forceinline__ double group_dot64(const char* mine, const char* other, int nchunk, int part) {
    constexpr int EPL = Elem<DT>::EPL;
    double acc = 0.0;
#pragma unroll 1
    for (int k0 = part; k0 < nchunk; k0 += 64) {
        uint4 va[4], vb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const size_t o = (size_t)(k0 + 16 * u < nchunk ? k0 + 16 * u : k0) * 16;
            va[u] = *(const uint4*)(mine + o);
            vb[u] = *(const uint4*)(other + o);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (k0 + 16 * u < nchunk) {
                // (the chunk is tied to the running sum so that the conversions of all chunks are
                //  not hoisted ahead of the additions: registers decide this kernel's occupancy)
                asm volatile("" : "+v"(va[u].x), "+v"(vb[u].x) : "v"(acc));
                double a[8], x[8];
                Elem<DT>::widen(va[u], a);
                Elem<DT>::widen(vb[u], x);
#pragma unroll
                for (int i = 0; i < EPL; ++i) acc = fma(a[i], x[i], acc);
            }
        }
    }
    return group_sum_f64(acc, 16);
}

// Dot product in fp64 of two rows whose 16-byte chunks the 16 lanes of a group already hold (chunks
// part, part + 16, .. of rows of at most 64 chunks; the first row widened to fp64 beforehand) and, in the
// same pass and the same order of
// operations, of the second row with itself: rows that are bit-identical then give bit-identical
// dot products and norms, i.e. a cosine of exactly 1.  Every lane of the group gets both sums.
template <int DT>
__device__ __forceinline__ void chunk_dots64(const double (&a)[4][8], const uint4 (&vb)[4], int nchunk, int part,
                                             double& dot, double& nn_other) {
    constexpr int EPL = Elem<DT>::EPL;
    double acc = 0.0, acc2 = 0.0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (part + 16 * u < nchunk) {
            double x[8];
            Elem<DT>::widen(vb[u], x);
#pragma unroll
            for (int i = 0; i < EPL; ++i) { acc = fma(a[u][i], x[i], acc); acc2 = fma(x[i], x[i], acc2); }
        }
    }
    dot = group_sum_f64(acc, 16);
    nn_other = group_sum_f64(acc2, 16);
}

// Densities of the listed tokens again, entirely in fp64 (Eq. 5 and Eq. 6 as they are written:
// dot product, two norms - recomputed here by the routine that computes the dot product, so
// that a copy of the token is at distance exactly 0 -, one division, one exponential per pair,
// the term of the token itself exactly 1).  This kernel leaves partial sums; the kernel that
// runs the centre rounds adds them up and rebuilds the predecessor lists of those tokens
// (finish_rechecked_densities below) before it looks at any list.
// Work items are (listed token, chunk of RHO_RECHECK_CHUNK kept tokens): one workgroup per item
// and turn, 16 lanes per pair.  The sums are exact, hence the same in any order and for any two
// tokens with the same terms (two tokens at equal distances from everything else tie exactly, as
// they do for a correctly rounded sum, and the index decides): every term t in (0, 1] is split
// into hi = t rounded to a multiple of 2^-30 and lo = t - hi; sums of at most 32768 such hi, and
// of such lo as long as t >= 2^-17 (d_n >= 0.17), fit the 53 bits of an fp64 whatever their
// order, and the density is hi_total + lo_total, rounded once.
// grid (blocks per sample, B), block 256.
template <int DT>
__global__ __launch_bounds__(256) void rho_recheck_kernel(Batch bt, const char* keys, int dk, const int32_t* idx,
                                                           pact_report* rep, double* part,
                                                           const int32_t* tie_list, const int32_t* tie_cnt) {
    __shared__ double s_hi[RHO_RECHECK_CHUNK], s_lo[RHO_RECHECK_CHUNK];
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int T = tie_cnt[4 * b];                      // (the same for every workgroup of the sample)
    const int q = clamp_count(rep[b].n_kept, sg.n);
    if (T <= 0) return;
    if (T > RHO_RECHECK_MAX) {
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&rep[b].refine_overflow, OVERFLOW_RHO_RECHECK);
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int nch = (q + RHO_RECHECK_CHUNK - 1) / RHO_RECHECK_CHUNK;
    const size_t row_bytes = (size_t)dk * Elem<DT>::BYTES;
    const int nchunk = (int)(row_bytes / 16);
    const char* kb = keys + (size_t)sg.base * row_bytes;
    const int32_t* ix = idx + sg.base;
    const int32_t* list = tie_list + (size_t)b * RHO_RECHECK_MAX;
    double* part_b = part + (size_t)b * 2 * rho_fix_tokens(bt.n_max) * rho_fix_chunks(bt.n_max);   // [T][nch][2], T <= q <= n_max
    const double d_n = (double)sg.d_n;
    const int g = tid >> 4, part16 = tid & 15;
    constexpr int PER = RHO_RECHECK_CHUNK / 16;          // pairs per group of 16 lanes and item
    static_assert(PER == 4, "a group's four rows are requested together");
    for (int item = blockIdx.x; item < T * nch; item += gridDim.x) {
        const int t = item / nch, c = item - t * nch;
        // this group's kept tokens: lane s of the group fetches the s-th one's token (one trip for all)
        const int pk_mine = c * RHO_RECHECK_CHUNK + (part16 & (PER - 1)) * 16 + g;
        const int tk_mine = ix[min(pk_mine, q - 1)];
        const int ent = list[t];
        const int p = min(ent & 0xFFFF, q - 1), tok = min(max(ent >> 16, 0), sg.n - 1);
        const char* mine = kb + (size_t)tok * row_bytes;
        if (nchunk <= 64) {
            // rows of at most 1 KB: a lane holds its (at most four) 16-byte chunks of the token's row and
            // those of the group's four other rows, all requested together
            uint4 vm[4], vk[PER][4];
#pragma unroll
            for (int u = 0; u < 4; ++u) vm[u] = *(const uint4*)(mine + (size_t)min(part16 + 16 * u, nchunk - 1) * 16);
#pragma unroll
            for (int s = 0; s < PER; ++s) {
                const int tk = __shfl(tk_mine, (lane & ~15) + s, 64);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    vk[s][u] = *(const uint4*)(kb + (size_t)tk * row_bytes + (size_t)min(part16 + 16 * u, nchunk - 1) * 16);
            }
            double am[4][8];
#pragma unroll
            for (int u = 0; u < 4; ++u) Elem<DT>::widen(vm[u], am[u]);
            double nnp, dd;
            chunk_dots64<DT>(am, vm, nchunk, part16, dd, nnp);
#pragma unroll
            for (int s = 0; s < PER; ++s) {
                const int pk = c * RHO_RECHECK_CHUNK + s * 16 + g;
                double dot, nnk;
                chunk_dots64<DT>(am, vk[s], nchunk, part16, dot, nnk);
                const double d = cos_dist64(dot, nnp, nnk);
                const double term = pk >= q ? 0.0 : (pk == p ? 1.0 : exp(-d / d_n));
                const double hi = rint(term * 1073741824.0) * (1.0 / 1073741824.0);
                if (part16 == 0) { s_hi[s * 16 + g] = hi; s_lo[s * 16 + g] = term - hi; }
            }
        } else {
            // longer rows: the group's four pairs advance together, four chunks of the token's row
            // and of each of the four other rows per trip (same order of operations per pair as above)
            constexpr int EPL = Elem<DT>::EPL;
            const char* rowk[PER];
#pragma unroll
            for (int s = 0; s < PER; ++s) rowk[s] = kb + (size_t)__shfl(tk_mine, (lane & ~15) + s, 64) * row_bytes;
            double nnp = 0.0, dot[PER], nnk[PER];
#pragma unroll
            for (int s = 0; s < PER; ++s) dot[s] = nnk[s] = 0.0;
#pragma unroll 1
            for (int k0 = part16; k0 < nchunk; k0 += 64) {
                uint4 vm[4], vk[PER][4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const size_t o = (size_t)min(k0 + 16 * u, nchunk - 1) * 16;
                    vm[u] = *(const uint4*)(mine + o);
#pragma unroll
                    for (int s = 0; s < PER; ++s) vk[s][u] = *(const uint4*)(rowk[s] + o);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (k0 + 16 * u < nchunk) {
                        double a[8], x[8];
                        Elem<DT>::widen(vm[u], a);
#pragma unroll
                        for (int i = 0; i < EPL; ++i) nnp = fma(a[i], a[i], nnp);
#pragma unroll
                        for (int s = 0; s < PER; ++s) {
                            Elem<DT>::widen(vk[s][u], x);
#pragma unroll
                            for (int i = 0; i < EPL; ++i) { dot[s] = fma(a[i], x[i], dot[s]); nnk[s] = fma(x[i], x[i], nnk[s]); }
                        }
                    }
                }
            }
            nnp = group_sum_f64(nnp, 16);
#pragma unroll
            for (int s = 0; s < PER; ++s) { dot[s] = group_sum_f64(dot[s], 16); nnk[s] = group_sum_f64(nnk[s], 16); }
#pragma unroll
            for (int s = 0; s < PER; ++s) {
                const int pk = c * RHO_RECHECK_CHUNK + s * 16 + g;
                const double d = cos_dist64(dot[s], nnp, nnk[s]);
                const double term = pk >= q ? 0.0 : (pk == p ? 1.0 : exp(-d / d_n));
                const double hi = rint(term * 1073741824.0) * (1.0 / 1073741824.0);
                if (part16 == 0) { s_hi[s * 16 + g] = hi; s_lo[s * 16 + g] = term - hi; }
            }
        }
        __syncthreads();
        if (tid < 64) {
            static_assert(RHO_RECHECK_CHUNK == 64, "one term per lane");
            const double vh = wave_sum_f64(s_hi[lane]);
            const double vl = wave_sum_f64(s_lo[lane]);
            if (lane == 0) *(double2*)(part_b + ((size_t)t * nch + c) * 2) = make_double2(vh, vl);
        }
        __syncthreads();
    }
}

// Eq. 8/9: every pruned token joins the nearest centre iff its fp64 distance is below
// alpha*d_c.  The matrix-core pass left, per pruned token t and group w of 64 centres, the
// group's largest fp32 cosine cbest[w][t] and a word of candidates (bits of the centres within
// reach whose cosine is at most 2 * margin below it), laid out [w][t].  With gm the largest of
// a token's cbest values, the nearest centre in exact arithmetic is a candidate of a group
// whose cbest >= gm - 2 * margin (margin bounds the error of an fp32 cosine).  Usually that is
// one centre, clear of the threshold: decided without touching a key.  Otherwise (several
// candidates, or one too close to alpha*d_c) Eq. 5 is evaluated in fp64 for each of them.
// What a token costs is its chain of dependent memory accesses, so 16 lanes work on one token
// (16 tokens per block and turn): the values and words of 64 groups arrive in one trip and are
// kept for the listing, a candidate row in another.  Blocks blk = 0 .. nblk-1, 256 threads.
// s_c: [16][RECOVER_LIST] candidate ids per token slot.
constexpr int RECOVER_LIST = 16;
template <int DT>
__device__ __forceinline__ void recover_body(const Batch& bt, const NearArgs& a, int blk, int nblk, lds_i32* s_c) {
    pact_report* rep = a.rep;
    const int b = blockIdx.y;
    const Seg sg = bt.s[b];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int t_first = blk * 16 + (tid >> 4);
    const int q = clamp_count(rep[b].n_kept, sg.n), np = clamp_count(rep[b].n_pruned, sg.n - q),
              C = clamp_count(rep[b].n_centers, q);
    const size_t row_bytes = (size_t)a.dk * Elem<DT>::BYTES;
    const int nchunk = (int)(row_bytes / 16);
    const char* kb = a.keys + (size_t)sg.base * row_bytes;
    const double* nnb = a.nn + sg.base;
    const int32_t* co = a.center_idx + sg.base;
    const int32_t* pruned = a.pruned_idx + sg.base;
    int32_t* cluster_id = a.cluster_id + sg.base;
    int32_t* cluster_counts = a.cluster_counts ? a.cluster_counts + sg.base : nullptr;
    const double thr = (double)sg.alpha * (double)sg.d_c;
    const double cthr = 1.0 - thr;                                  // d < thr  <=>  cosine > 1 - thr
    const float margin = a.margin;
    const float t_lo = (1.0f - sg.alpha * sg.d_c) - margin;         // as the matrix-core pass computes it
    const int Wc = (C + 63) >> 6;
    const float* cb = a.cbest + (size_t)b * bt.W * bt.n_max;        // [W][n_max]
    const uint64_t* cw = a.adj + ((size_t)b * bt.n_max + q) * bt.W; // [Wc][np]
    const int part = tid & 15, ts = tid >> 4, gbase = lane & ~15;
    lds_i32* list = s_c + ts * RECOVER_LIST;
    for (int t = t_first; t < np; t += nblk * 16) {
        const int tok = pruned[t];
        int res = -1;                                               // -1: no centre in reach
        if (thr > 0.0 && C > 0) {
            // groups part, part + 16, .. of the first 64 with their candidate words (a word is
            // only meaningful where the group's largest cosine is within reach); further
            // groups, if any, for the maximum only
            float v[4];
            uint64_t word[4];
            auto load_batch = [&](int wb) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int w = wb + part + 16 * u;
                    v[u] = w < Wc ? cb[(size_t)w * bt.n_max + t] : -INFINITY;
                    word[u] = w < Wc ? cw[(size_t)w * np + t] : 0ull;
                }
            };
            load_batch(0);
            float gm = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
            for (int w = 64 + part; w < Wc; w += 16) gm = fmaxf(gm, cb[(size_t)w * bt.n_max + t]);
            gm = group_max_f32<16>(gm);
            if (gm >= t_lo) {
                const float floor32 = fmaxf(gm - 2.0f * margin, t_lo);
                const bool clear = (double)gm - cthr > (double)margin;   // the nearest is certainly within alpha*d_c
                const char* mine = kb + (size_t)tok * row_bytes;
                double best = INFINITY;
                int bestc = 0x7FFFFFFF;
                bool first_batch_loaded = true;
                // The candidates are listed in the token's LDS slots, RECOVER_LIST per turn (one
                // turn unless the token is degenerate); all control flow from here on is uniform
                // within the 16 lanes of a token.
#pragma unroll 1
                for (int skip = 0;; skip += RECOVER_LIST) {
                    int n = 0, ntot = 0;
#pragma unroll 1
                    for (int wb = 0; wb < Wc; wb += 64) {
                        if (!first_batch_loaded) load_batch(wb);     // (the first turn starts with the values already here)
                        first_batch_loaded = false;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            const uint64_t wv = (v[u] >= floor32) ? word[u] : 0ull;
                            uint32_t who = (uint32_t)(__ballot(wv != 0) >> gbase) & 0xFFFFu;
                            while (who) {
                                const int src = __builtin_ctz(who);
                                who &= who - 1;
                                uint64_t bits = __shfl(wv, gbase + src, 64);
                                const int cbase = (wb + src + 16 * u) << 6;
                                while (bits) {
                                    const int c = cbase + __builtin_ctzll(bits);
                                    bits &= bits - 1;
                                    if (ntot >= skip && n < RECOVER_LIST) {
                                        if (part == 0) list[n] = c;
                                        ++n;
                                    }
                                    ++ntot;
                                }
                            }
                        }
                    }
                    if (ntot == 1 && clear) {                          // decided by the fp32 screen alone
                        bestc = list[0];
                        break;
                    }
                    // fp64 for the n listed candidates: their tokens and norms in one trip, then row by row
                    int ctk = 0, cid = 0;
                    double cnn = 0.0;
                    if (part < n) {
                        cid = list[part];
                        ctk = co[cid];
                        cnn = nnb[ctk];
                    }
                    const double nnp = nnb[tok];
#pragma unroll 1
                    for (int k = 0; k < n; ++k) {
                        const int c = __shfl(cid, gbase + k, 64);
                        const int tc = __shfl(ctk, gbase + k, 64);
                        const double nc = __shfl(cnn, gbase + k, 64);
                        const double d = cos_dist64(group_dot64<DT>(mine, kb + (size_t)tc * row_bytes, nchunk, part), nnp, nc);
                        if (d < thr && (d < best || (d == best && c < bestc))) { best = d; bestc = c; }
                    }
                    if (skip + RECOVER_LIST >= ntot) break;
                }
                res = bestc != 0x7FFFFFFF ? bestc : -1;
            }
        }
        if (part == 0) {
            cluster_id[tok] = res;
            // (recovered / dropped totals are derived from the cluster sizes by the merge: a
            //  counter that every wavefront hits would serialise at one L2 address)
            if (res >= 0 && cluster_counts) join_cluster(a, rep + b, sg.base, res, tok);
            note_odd_norm(rep + b, nnb[tok]);
        }
    }
}

// grid (recovery blocks + assign_blocks, B), block 256: the recovery blocks first - their chain of
// dependent accesses is the longest, and behind the assignment blocks (two turns of what the
// chip holds, the last ones idle: their number is sized by n, not by the kept tokens) they
// started 3 us late.
// PART: NEAREST_BOTH, or a build that holds one of the two searches only (the assignment alone
// needs fewer registers and runs four wavefronts per SIMD instead of three).
enum { NEAREST_BOTH = 0, NEAREST_ASSIGN = 1, NEAREST_RECOVER = 2 };
template <int DT, int PART>
__global__ __launch_bounds__(256) void nearest_centre_kernel(Batch bt, NearArgs a) {
    __shared__ int s_cand[4][CAND_BUF], s_ctok[4][CAND_BUF];
    __shared__ float s_ccos[4][CAND_BUF];
    __shared__ int s_list[16 * RECOVER_LIST];
    const int wave = threadIdx.x >> 6;
    lds_i32* cand = (lds_i32*)s_cand[wave];
    lds_i32* ctok = (lds_i32*)s_ctok[wave];
    lds_f32* ccos = (lds_f32*)s_ccos[wave];
    if constexpr (PART == NEAREST_ASSIGN) assign_body<DT>(bt, a, blockIdx.x, cand, ctok, ccos);
    else if constexpr (PART == NEAREST_RECOVER) recover_body<DT>(bt, a, blockIdx.x, gridDim.x, (lds_i32*)s_list);
    else if ((int)blockIdx.x >= (int)gridDim.x - a.assign_blocks)
        assign_body<DT>(bt, a, blockIdx.x - (gridDim.x - a.assign_blocks), cand, ctok, ccos);
    else recover_body<DT>(bt, a, blockIdx.x, gridDim.x - a.assign_blocks, (lds_i32*)s_list);
}

template <int PART>
static int launch_nearest_part(const Batch& bt, const NearArgs& a, int blocks, pact_dtype k_dt, const char* name,
                               hipStream_t st) {
    dim3 grid(blocks, bt.B);
    if (k_dt == PACT_BF16) PACT_LAUNCH(name, (nearest_centre_kernel<PACT_BF16, PART>), grid, dim3(256), st, bt, a);
    else PACT_LAUNCH(name, (nearest_centre_kernel<PACT_F32, PART>), grid, dim3(256), st, bt, a);
    return PACT_OK;
}
static int launch_nearest(const Batch& bt, const NearArgs& a, int recover_blocks, pact_dtype k_dt, const char* name,
                          hipStream_t st) {
    if (recover_blocks == 0) return launch_nearest_part<NEAREST_ASSIGN>(bt, a, a.assign_blocks, k_dt, name, st);
    if (a.assign_blocks == 0) return launch_nearest_part<NEAREST_RECOVER>(bt, a, recover_blocks, k_dt, name, st);
    return launch_nearest_part<NEAREST_BOTH>(bt, a, a.assign_blocks + recover_blocks, k_dt, name, st);
}

// Stand-alone pact_reincorporate: totals of recovered / dropped tokens (the fused path gets
// them from the cluster sizes).  grid (B), block 1024.
__global__ __launch_bounds__(1024) void count_recovered_kernel(Batch bt, pact_report* rep,
                                                               const int32_t* __restrict__ pruned_idx,
                                                               const int32_t* __restrict__ cluster_id) {
    __shared__ int s_tot;
    const int b = blockIdx.x;
    const Seg sg = bt.s[b];
    const int q = clamp_count(rep[b].n_kept, sg.n), np = clamp_count(rep[b].n_pruned, sg.n - q);
    if (threadIdx.x == 0) s_tot = 0;
    __syncthreads();
    int loc = 0;
    for (int t = threadIdx.x; t < np; t += 1024) loc += cluster_id[sg.base + pruned_idx[sg.base + t]] >= 0;
    loc = (int)wave_sum_f64((double)loc);
    if ((threadIdx.x & 63) == 0 && loc) atomicAdd(&s_tot, loc);
    __syncthreads();
    if (threadIdx.x == 0) { rep[b].n_reincorporated = s_tot; rep[b].n_dropped = np - s_tot; }
}

// ------------------------------------------------------------------------------------------
int launch_centres(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                   const int32_t* idx, int32_t* center_idx, int32_t* cluster_id,
                   int32_t* cluster_counts, pact_report* rep, double* rho_opt, int32_t* rank_opt,
                   int stat_words, bool assign_now, hipStream_t st) {
    const char* k = (const char*)keys;
    dim3 gpost(REFINE_BLOCKS + (bt.n_max + 63) / 64, bt.B);
    if (k_dt == PACT_BF16)
        PACT_LAUNCH("post_gram", post_gram_kernel<PACT_BF16>, gpost, dim3(256), st, bt, k, dk, idx, w.nn,
                    w.near_list, w.near_cnt, w.stat, stat_words, w.adj, rep, w.rho_part, w.rho, rho_opt);
    else
        PACT_LAUNCH("post_gram", post_gram_kernel<PACT_F32>, gpost, dim3(256), st, bt, k, dk, idx, w.nn,
                    w.near_list, w.near_cnt, w.stat, stat_words, w.adj, rep, w.rho_part, w.rho, rho_opt);
    dim3 gtok((bt.n_max + 3) / 4, bt.B);
    PACT_LAUNCH("build_preds", build_preds_kernel, gtok, dim3(256), st, bt, rep, w.adj, w.rho, w.preds,
                w.heads, idx, w.tie_list, w.tie_cnt);
    // neighbours whose densities the fp32 terms cannot order: fp64 (a few tokens of an image)
    // (one sample: 2048 workgroups, a work item each for up to 32 listed tokens of a 4000-token sample -
    //  the chip holds 512 of them at a time, and 4096 took 0.8 us longer to dispatch; a batch: 8192
    //  shared out equally, since the listed tokens are not spread evenly over the samples)
    const int rb = bt.B == 1 ? 2048 : 8192 / bt.B;
    // Rows of whole 64-byte quarters can go through the fp64 matrix instruction.  A 16 x 16 tile of dot
    // products is then one wavefront's chain of dk / 4 instructions (4 us at a key width of 512), against
    // a couple of trips to memory per 64 pairs for the vector version.  With the handful of listed tokens
    // of one image, or of a batch of small images, the vector version is the shorter one (4010 kept
    // tokens: 12.3 against 14.9 us; 16 ragged images: 13.4 against 22.5 us); with many kept tokens or wide
    // rows the matrix version (16384 kept tokens, 70 listed: 195 -> 58 us; 8 videos of 3450 kept tokens:
    // 48 -> 29 us; 3584-wide rows: 82 -> 52 us).  How many tokens are listed is known on the device only
    // (one kernel holding both versions behind a device-side choice ran each of them a quarter to a half
    // slower), so the host goes by the kept tokens it expects.
    const size_t recheck_row_bytes = (size_t)dk * (k_dt == PACT_BF16 ? 2 : 4);
    long kept_est = 0;
    for (int b = 0; b < bt.B; ++b) kept_est += bt.s[b].n - prune_rank(bt.s[b].lambda, bt.s[b].n);
    const bool quarters = recheck_row_bytes % 64 == 0 &&
                          (kept_est >= (bt.B == 1 ? 6000 : 20000) || recheck_row_bytes >= 4096);
    if (quarters && k_dt == PACT_BF16)
        PACT_LAUNCH("rho_recheck", rho_recheck_mfma_kernel<PACT_BF16>, dim3(rb, bt.B), dim3(256), st, bt, k, dk, idx,
                    w.nn, rep, w.rho_fix, w.tie_list, w.tie_cnt);
    else if (quarters)
        PACT_LAUNCH("rho_recheck", rho_recheck_mfma_kernel<PACT_F32>, dim3(rb, bt.B), dim3(256), st, bt, k, dk, idx,
                    w.nn, rep, w.rho_fix, w.tie_list, w.tie_cnt);
    else if (k_dt == PACT_BF16)
        PACT_LAUNCH("rho_recheck", rho_recheck_kernel<PACT_BF16>, dim3(rb, bt.B), dim3(256), st, bt, k, dk, idx,
                    rep, w.rho_fix, w.tie_list, w.tie_cnt);
    else
        PACT_LAUNCH("rho_recheck", rho_recheck_kernel<PACT_F32>, dim3(rb, bt.B), dim3(256), st, bt, k, dk, idx,
                    rep, w.rho_fix, w.tie_list, w.tie_cnt);
    const size_t qpad = (size_t)((bt.n_max + 63) / 64 * 64);
    const bool wl_lds = bt.n_max <= RESOLVE_LDS_TOKENS;       // the work lists fit beside the statuses
    const size_t lds_base = (qpad + 64 + qpad * 2 + ((size_t)bt.W + 1) * 4 + 7) & ~(size_t)7;
    const size_t lds = lds_base + (wl_lds ? (size_t)bt.n_max * 16 : 0);
    static size_t raised[2] = {0, 0};
    const void* fn = wl_lds ? (const void*)centre_resolve_kernel<true> : (const void*)centre_resolve_kernel<false>;
    if (lds > 48 * 1024 && lds > raised[wl_lds ? 1 : 0]) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return PACT_ERR_HIP;
        raised[wl_lds ? 1 : 0] = lds;
    }
    if (wl_lds)
        PACT_LAUNCH_SHMEM("centre_resolve", centre_resolve_kernel<true>, dim3(bt.B), dim3(1024), lds, st, bt, rep,
                          w.adj, w.rho, rho_opt, w.preds, w.heads, idx, w.tie_list, w.tie_cnt, w.rho_fix, w.status,
                          w.cnum, w.cmask, center_idx, w.worklist);
    else
        PACT_LAUNCH_SHMEM("centre_resolve", centre_resolve_kernel<false>, dim3(bt.B), dim3(1024), lds, st, bt, rep,
                          w.adj, w.rho, rho_opt, w.preds, w.heads, idx, w.tie_list, w.tie_cnt, w.rho_fix, w.status,
                          w.cnum, w.cmask, center_idx, w.worklist);
    if (rank_opt)          // (after the fp64 densities are in place)
        PACT_LAUNCH("density_rank", rank_kernel, dim3((bt.n_max + 63) / 64, bt.B), dim3(1024), st, bt, rep,
                    w.rho, rank_opt);
    if (!assign_now) return PACT_OK;          // the caller runs it with the recovery (launch_reincorporate)
    NearArgs a;
    std::memset(&a, 0, sizeof(a));
    a.rep = rep; a.keys = k; a.dk = dk; a.nn = w.nn; a.adj = w.adj; a.margin = (float)cos_margin(dk);
    a.cluster_id = cluster_id; a.cluster_counts = cluster_counts;
    a.idx = idx; a.cmask = w.cmask; a.status = w.status; a.cnum = w.cnum;
    a.assign_blocks = (bt.n_max + 3) / 4;
    return launch_nearest(bt, a, 0, k_dt, "assign", st);
}

int launch_gram_candidates(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                           const int32_t* pruned_idx, const int32_t* center_idx, pact_report* rep,
                           hipStream_t st);

// kept_idx != nullptr: the assignment of the kept tokens (deferred by launch_centres) runs in the
// same launch as the recovery.
int launch_reincorporate(const Batch& bt, const Ws& w, const void* keys, pact_dtype k_dt, int32_t dk,
                         const int32_t* pruned_idx, const int32_t* center_idx, int32_t* cluster_id,
                         int32_t* cluster_counts, pact_report* rep, bool count_totals,
                         const int32_t* kept_idx, hipStream_t st) {
    int rc = launch_gram_candidates(bt, w, keys, k_dt, dk, pruned_idx, center_idx, rep, st);
    if (rc != PACT_OK) return rc;
    NearArgs a;
    std::memset(&a, 0, sizeof(a));
    a.rep = rep; a.keys = (const char*)keys; a.dk = dk; a.nn = w.nn; a.adj = w.adj;
    a.margin = (float)cos_margin(dk);
    a.cluster_id = cluster_id; a.cluster_counts = cluster_counts;
    a.pruned_idx = pruned_idx; a.center_idx = center_idx; a.cbest = w.cbest;
    if (kept_idx) {
        a.idx = kept_idx; a.cmask = w.cmask; a.status = w.status; a.cnum = w.cnum;
        a.assign_blocks = (bt.n_max + 3) / 4;
        a.slots = w.slots; a.big = w.big;     // (a full reduction: the merge follows)
    }
    if (kept_idx && bt.total >= 20000) {
        // Large batches are bound by how many wavefronts of these searches the chip holds: the two
        // searches then go out as two launches, the assignment in its leaner build.  (One image:
        // one launch, the second launch floor would cost more than the occupancy gives.)
        NearArgs only = a;
        only.assign_blocks = 0;
        if ((rc = launch_nearest(bt, a, 0, k_dt, "assign", st))) return rc;
        if ((rc = launch_nearest(bt, only, (bt.n_max + 15) / 16, k_dt, "reincorporate", st))) return rc;
    } else if ((rc = launch_nearest(bt, a, (bt.n_max + 15) / 16, k_dt, "reinc_assign", st))) return rc;
    if (count_totals)
        PACT_LAUNCH("count_recovered", count_recovered_kernel, dim3(bt.B), dim3(1024), st, bt, rep,
                    pruned_idx, cluster_id);
    return PACT_OK;
}

}  // namespace pact

// C ABI of libpact: argument validation (host-only, before anything touches the GPU),
// workspace partitioning, stage sequencing.  Nothing here allocates or synchronises.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <vector>

#include "pact_internal.h"

namespace pact {

// ------------------------------------------------------------------------------ profiling
struct ProfRec { const char* name; hipEvent_t a, b; };
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof;
static size_t g_prof_used = 0;

void prof_begin(const char* name, hipStream_t s) {
    if (!g_prof_on) return;
    if (g_prof_used == g_prof.size()) {
        ProfRec r;
        r.name = name;
        if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) { g_prof_on = false; return; }
        g_prof.push_back(r);
    }
    g_prof[g_prof_used].name = name;
    (void)hipEventRecord(g_prof[g_prof_used].a, s);
}
void prof_end(hipStream_t s) {
    if (!g_prof_on) return;
    (void)hipEventRecord(g_prof[g_prof_used].b, s);
    ++g_prof_used;
}

// ------------------------------------------------------------------------------ validation
static inline bool dtype_ok(int d) { return d == PACT_F32 || d == PACT_BF16; }
static inline int esize(int d) { return d == PACT_BF16 ? 2 : 4; }
static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

static int check_params(float lambda, float d_c, float d_n, float alpha) {
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return PACT_ERR_PARAM;
    if (!(d_c >= 0.0f) || !std::isfinite(d_c)) return PACT_ERR_PARAM;
    if (!(d_n > 0.0f) || !std::isfinite(d_n)) return PACT_ERR_PARAM;
    if (!(alpha >= 0.0f) || !std::isfinite(alpha)) return PACT_ERR_PARAM;
    return PACT_OK;
}
static int check_tensor(const void* p, int dt, int64_t cols) {
    if (!p) return PACT_ERR_NULL;
    if (!dtype_ok(dt)) return PACT_ERR_DTYPE;
    if (cols < 1) return PACT_ERR_SHAPE;
    if (!aligned16(p) || (cols * esize(dt)) % 16 != 0) return PACT_ERR_ALIGN;
    return PACT_OK;
}
// The matrix passes address a sample's clustering keys with 32-bit byte offsets (fp32 keys in
// their three-part bf16 form, 6 bytes per value).
static int check_key_extent(int64_t n_max, int64_t dk, int k_dt) {
    const uint64_t tok_bytes = (k_dt == PACT_F32) ? 3ull * (((uint64_t)dk + 7) & ~7ull) * 2 : (uint64_t)dk * 2;
    return (uint64_t)n_max * tok_bytes > 0xFFFFFFFFull ? PACT_ERR_SHAPE : PACT_OK;
}
static int check_ws(const void* ws, size_t ws_bytes, size_t need) {
    if (!ws || ((uintptr_t)ws & 255u) != 0 || ws_bytes < need) return PACT_ERR_WORKSPACE;
    return PACT_OK;
}

static int g_dev_state = 0;   // 0 unknown, 1 ok, -1 bad
static int check_device() {
    if (g_dev_state == 1) return PACT_OK;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return PACT_ERR_NOGPU; }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return PACT_ERR_NOGPU; }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return PACT_ERR_NOGPU;
    g_dev_state = 1;
    return PACT_OK;
}

static void fill_single(Batch& bt, int32_t n, const pact_params& p) {
    std::memset(&bt, 0, sizeof(bt));
    bt.B = 1; bt.n_max = n; bt.W = (n + 63) / 64; bt.total = n;
    bt.s[0].base = 0; bt.s[0].n = n;
    bt.s[0].lambda = p.lambda; bt.s[0].d_c = p.d_c; bt.s[0].d_n = p.d_n; bt.s[0].alpha = p.alpha;
    bt.s[0].fallback_T = p.fallback_T; bt.s[0].flags = p.flags;
}

static pact_params default_params() {
    pact_params p; p.lambda = 0.0f; p.d_c = 0.0f; p.d_n = 2.0f; p.alpha = 1.5f; p.fallback_T = 10; p.flags = 0;
    return p;
}

// ------------------------------------------------------------------------------ own scratch
// Workspace of pact_reduce_static: one array per GPU, part of the loaded code object (no
// allocation call ever made for it), kept until the process ends.  `scratch` is the host-side
// handle of the symbol, not a device address: the address on the current device comes from
// hipGetSymbolAddress, once per device, and is what kernels are given.
static __device__ __align__(256) unsigned char scratch[PACT_STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_addr[MAX_DEVICES] = {};
static std::mutex g_scratch_mutex;

static int own_scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return PACT_ERR_NOGPU; }
    if (dev < 0 || dev >= MAX_DEVICES) return PACT_ERR_NOGPU;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_addr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return PACT_ERR_HIP; }
        if ((uintptr_t)ptr & 255u) return PACT_ERR_HIP;
        g_scratch_addr[dev] = ptr;
    }
    *out = g_scratch_addr[dev];
    return PACT_OK;
}

struct ReduceIO {
    const void* hidden; pact_dtype h_dt; int32_t h;
    const void* keys_pre; const void* keys; pact_dtype k_dt; int32_t n_kv, d_h;
    const void* q; pact_dtype q_dt; int32_t q_per_token, n_q;
    float* scores; int32_t *kept_idx, *pruned_idx, *center_idx, *cluster_id;
    void* merged; pact_dtype out_dt; int32_t* cluster_counts; pact_report* rep;
};

static int run_reduce(const Batch& bt, const Ws& w, const ReduceIO& io, hipStream_t st) {
    const int32_t dk = io.n_kv * io.d_h;
    int rc = launch_prep(bt, w, io.keys, io.k_dt, dk, io.q_per_token ? io.q : nullptr, io.q_dt,
                         io.n_q * io.d_h, io.rep, io.cluster_id, io.cluster_counts, INIT_REDUCE, nullptr, st);
    if (rc) return rc;
    ScoreIn si{io.hidden, io.h_dt, io.h, io.keys_pre, io.k_dt, io.n_kv, io.d_h, io.q, io.q_dt,
               io.q_per_token, io.n_q};
    if ((rc = launch_score(bt, w, si, st))) return rc;
    if ((rc = launch_score_only(bt, w, io.n_q, io.scores, st))) return rc;
    if ((rc = launch_score_prune(bt, io.scores, w.adj, io.kept_idx, io.pruned_idx, io.rep, st))) return rc;
    bool want_stat = false;                  // the key-distance statistic: only if a sample asks for it
    for (int b = 0; b < bt.B; ++b) want_stat = want_stat || (bt.s[b].flags & PACT_FLAG_KEY_STATS);
    int stat_words = 0;
    if ((rc = launch_gram_density(bt, w, io.keys, io.k_dt, dk, io.kept_idx, io.rep, want_stat, &stat_words, st)))
        return rc;
    if ((rc = launch_centres(bt, w, io.keys, io.k_dt, dk, io.kept_idx, io.center_idx, io.cluster_id,
                             io.cluster_counts, io.rep, nullptr, nullptr, stat_words, false, st))) return rc;
    // (the kept tokens are assigned in the same launch as the pruned ones are recovered)
    if ((rc = launch_reincorporate(bt, w, io.keys, io.k_dt, dk, io.pruned_idx, io.center_idx,
                                   io.cluster_id, io.cluster_counts, io.rep, false, io.kept_idx, st))) return rc;
    return launch_merge(bt, w, io.hidden, io.h_dt, io.h, io.cluster_id, io.center_idx, io.rep, io.merged,
                        io.out_dt, io.cluster_counts, false, st);
}

// Grid-stride copy of 16-byte words: the dispatch of known traffic behind pact_calibration_copy.
__global__ void __launch_bounds__(256) calibration_copy_kernel(uint4* __restrict__ dst,
                                                                const uint4* __restrict__ src, size_t n16) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace pact

using namespace pact;

extern "C" {

size_t pact_workspace_bytes(int32_t n_max, int32_t batch, int32_t dk, pact_dtype k_dt, int32_t n_q, int32_t d_h) {
    if (n_max < 1 || n_max > PACT_MAX_TOKENS || batch < 1 || batch > PACT_MAX_BATCH) return 0;
    if (dk < 1 || !dtype_ok(k_dt) || n_q < 1 || n_q > PACT_MAX_QHEADS || d_h < 1) return 0;
    return make_layout(n_max, batch, (int64_t)n_max * batch, (int64_t)n_q * d_h, n_q, dk, k_dt).total;
}

int pact_score(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
               const void* keys_pre, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
               const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q, uint32_t flags,
               float* scores, void* ws, size_t ws_bytes, void* stream) {
    if (!scores) return PACT_ERR_NULL;
    if (n < 1 || n > PACT_MAX_TOKENS || n_kv < 1 || d_h < 1 || n_q < 1 || n_q > PACT_MAX_QHEADS ||
        n_q % n_kv != 0 || (q_rows != n && q_rows != 1)) {
        if (!hidden || !keys_pre || !q) return PACT_ERR_NULL;
        return PACT_ERR_SHAPE;
    }
    int rc;
    if ((rc = check_tensor(hidden, h_dt, h))) return rc;
    if ((rc = check_tensor(keys_pre, k_dt, (int64_t)n_kv * d_h))) return rc;
    if ((rc = check_tensor(q, q_dt, (int64_t)n_q * d_h))) return rc;
    if (((int64_t)d_h * esize(k_dt)) % 16 != 0 || ((int64_t)d_h * esize(q_dt)) % 16 != 0) return PACT_ERR_ALIGN;
    const WsLayout L = make_layout(n, 1, n, (int64_t)n_q * d_h, n_q, 0, PACT_BF16);
    if ((rc = check_ws(ws, ws_bytes, L.total))) return rc;
    if ((rc = check_device())) return rc;
    Batch bt;
    pact_params sp = default_params();
    sp.flags = flags & (PACT_FLAG_SCORE_NO_NORM | PACT_FLAG_SCORE_NORM_ONLY);
    fill_single(bt, n, sp);
    const Ws w = resolve(ws, L);
    hipStream_t st = (hipStream_t)stream;
    ScoreIn si{hidden, h_dt, h, keys_pre, k_dt, n_kv, d_h, q, q_dt, q_rows == n ? 1 : 0, n_q};
    if (si.q_per_token &&
        (rc = launch_prep(bt, w, nullptr, k_dt, 0, q, q_dt, n_q * d_h, nullptr, nullptr, nullptr, INIT_SCORE,
                          nullptr, st)))
        return rc;
    if ((rc = launch_score(bt, w, si, st))) return rc;
    return launch_score_only(bt, w, n_q, scores, st);
}

int pact_prune(const float* scores, int32_t n, float lambda,
               int32_t* kept_idx, int32_t* pruned_idx, pact_report* rep,
               void* ws, size_t ws_bytes, void* stream) {
    (void)ws; (void)ws_bytes;       // the split needs no scratch
    if (!scores || !kept_idx || !pruned_idx || !rep) return PACT_ERR_NULL;
    if (n < 1 || n > PACT_MAX_TOKENS) return PACT_ERR_SHAPE;
    if (!(lambda >= 0.0f && lambda <= 1.0f)) return PACT_ERR_PARAM;
    int rc;
    if ((rc = check_device())) return rc;
    pact_params p = default_params();
    p.lambda = lambda;
    Batch bt;
    fill_single(bt, n, p);
    return launch_score_prune(bt, scores, nullptr, kept_idx, pruned_idx, rep, (hipStream_t)stream);
}

int dbdpc_cluster(const void* keys, pact_dtype k_dt, int32_t n, int32_t dk,
                  const int32_t* idx, const int32_t* n_idx_dev,
                  float d_c, float d_n, int32_t fallback_T,
                  int32_t* center_idx, int32_t* cluster_id, pact_report* rep,
                  double* rho_opt, int32_t* rank_opt,
                  void* ws, size_t ws_bytes, void* stream) {
    if (!center_idx || !cluster_id || !rep) return PACT_ERR_NULL;
    if (idx && !n_idx_dev) return PACT_ERR_NULL;
    if (n < 1 || n > PACT_MAX_TOKENS) return keys ? PACT_ERR_SHAPE : PACT_ERR_NULL;
    int rc;
    if ((rc = check_tensor(keys, k_dt, dk))) return rc;
    if ((rc = check_key_extent(n, dk, k_dt))) return rc;
    if ((rc = check_params(0.0f, d_c, d_n, 0.0f))) return rc;
    if (fallback_T < 0) return PACT_ERR_PARAM;
    const WsLayout L = make_layout(n, 1, n, 1, 1, dk, k_dt);
    if ((rc = check_ws(ws, ws_bytes, L.total))) return rc;
    if ((rc = check_device())) return rc;
    pact_params p = default_params();
    p.d_c = d_c; p.d_n = d_n; p.fallback_T = fallback_T;
    Batch bt;
    fill_single(bt, n, p);
    const Ws w = resolve(ws, L);
    hipStream_t st = (hipStream_t)stream;
    if ((rc = launch_prep(bt, w, keys, k_dt, dk, nullptr, PACT_F32, 0, rep, cluster_id, nullptr,
                          idx ? INIT_DBDPC_SUBSET : INIT_DBDPC_ALL, n_idx_dev, st))) return rc;
    const int32_t* use_idx = idx ? idx : w.ident;
    int stat_words = 0;
    if ((rc = launch_gram_density(bt, w, keys, k_dt, dk, use_idx, rep, true, &stat_words, st))) return rc;
    return launch_centres(bt, w, keys, k_dt, dk, use_idx, center_idx, cluster_id, nullptr, rep, rho_opt,
                          rank_opt, stat_words, true, st);
}

int pact_reincorporate(const void* keys, pact_dtype k_dt, int32_t n, int32_t dk,
                       const int32_t* pruned_idx, const int32_t* center_idx,
                       float d_c, float alpha, int32_t* cluster_id, pact_report* rep,
                       void* ws, size_t ws_bytes, void* stream) {
    if (!pruned_idx || !center_idx || !cluster_id || !rep) return PACT_ERR_NULL;
    if (n < 1 || n > PACT_MAX_TOKENS) return keys ? PACT_ERR_SHAPE : PACT_ERR_NULL;
    int rc;
    if ((rc = check_tensor(keys, k_dt, dk))) return rc;
    if ((rc = check_key_extent(n, dk, k_dt))) return rc;
    if ((rc = check_params(0.0f, d_c, 1.0f, alpha))) return rc;
    const WsLayout L = make_layout(n, 1, n, 1, 1, dk, k_dt);
    if ((rc = check_ws(ws, ws_bytes, L.total))) return rc;
    if ((rc = check_device())) return rc;
    pact_params p = default_params();
    p.d_c = d_c; p.alpha = alpha;
    Batch bt;
    fill_single(bt, n, p);
    const Ws w = resolve(ws, L);
    hipStream_t st = (hipStream_t)stream;
    if ((rc = launch_prep(bt, w, keys, k_dt, dk, nullptr, PACT_F32, 0, rep, cluster_id, nullptr, INIT_REINC,
                          nullptr, st))) return rc;
    return launch_reincorporate(bt, w, keys, k_dt, dk, pruned_idx, center_idx, cluster_id, nullptr, rep, true,
                                nullptr, st);
}

int pact_merge(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
               const int32_t* cluster_id, const int32_t* center_idx, pact_report* rep,
               uint32_t flags, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
               void* ws, size_t ws_bytes, void* stream) {
    if (!cluster_id || !rep || !merged || !cluster_counts) return PACT_ERR_NULL;
    if ((flags & PACT_FLAG_NO_MERGE) && !center_idx) return PACT_ERR_NULL;
    if (n < 1 || n > PACT_MAX_TOKENS) return hidden ? PACT_ERR_SHAPE : PACT_ERR_NULL;
    int rc;
    if ((rc = check_tensor(hidden, h_dt, h))) return rc;
    if (!dtype_ok(out_dt)) return PACT_ERR_DTYPE;
    if (!aligned16(merged) || ((int64_t)h * esize(out_dt)) % 16 != 0) return PACT_ERR_ALIGN;
    const WsLayout L = make_layout(n, 1, n, 1, 1, 0, PACT_BF16);
    if ((rc = check_ws(ws, ws_bytes, L.total))) return rc;
    if ((rc = check_device())) return rc;
    pact_params p = default_params();
    p.flags = flags;
    Batch bt;
    fill_single(bt, n, p);
    const Ws w = resolve(ws, L);
    hipStream_t st = (hipStream_t)stream;
    return launch_merge(bt, w, hidden, h_dt, h, cluster_id, center_idx, rep, merged, out_dt, cluster_counts,
                        true, st);
}

static int validate_reduce_common(const void* hidden, pact_dtype h_dt, int32_t h,
                                  const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv,
                                  int32_t d_h, const void* q, pact_dtype q_dt, int32_t n_q,
                                  const float* scores, const int32_t* kept_idx, const int32_t* pruned_idx,
                                  const int32_t* center_idx, const int32_t* cluster_id, const void* merged,
                                  pact_dtype out_dt, const int32_t* cluster_counts, const pact_report* rep) {
    if (!scores || !kept_idx || !pruned_idx || !center_idx || !cluster_id || !merged || !cluster_counts || !rep)
        return PACT_ERR_NULL;
    if (!hidden || !keys_pre || !keys || !q) return PACT_ERR_NULL;
    if (n_kv < 1 || d_h < 1 || n_q < 1 || n_q > PACT_MAX_QHEADS || n_q % n_kv != 0 || h < 1) return PACT_ERR_SHAPE;
    int rc;
    if ((rc = check_tensor(hidden, h_dt, h))) return rc;
    if ((rc = check_tensor(keys_pre, k_dt, (int64_t)n_kv * d_h))) return rc;
    if ((rc = check_tensor(keys, k_dt, (int64_t)n_kv * d_h))) return rc;
    if ((rc = check_tensor(q, q_dt, (int64_t)n_q * d_h))) return rc;
    if (((int64_t)d_h * esize(k_dt)) % 16 != 0 || ((int64_t)d_h * esize(q_dt)) % 16 != 0) return PACT_ERR_ALIGN;
    if (!dtype_ok(out_dt)) return PACT_ERR_DTYPE;
    if (!aligned16(merged) || ((int64_t)h * esize(out_dt)) % 16 != 0) return PACT_ERR_ALIGN;
    return PACT_OK;
}

// pact_reduce and pact_reduce_static: the same checks and the same launches; `ws` is the
// caller's workspace, or NULL for the library's own scratch array.
static int reduce_single(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
                         const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                         const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                         const pact_params* p,
                         float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                         int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                         pact_report* rep, void* ws, size_t ws_bytes, bool own_scratch, void* stream) {
    if (!p) return PACT_ERR_NULL;
    int rc = validate_reduce_common(hidden, h_dt, h, keys_pre, keys, k_dt, n_kv, d_h, q, q_dt, n_q, scores,
                                    kept_idx, pruned_idx, center_idx, cluster_id, merged, out_dt,
                                    cluster_counts, rep);
    if (rc) return rc;
    if (n < 1 || n > PACT_MAX_TOKENS || (q_rows != n && q_rows != 1)) return PACT_ERR_SHAPE;
    if ((rc = check_key_extent(n, (int64_t)n_kv * d_h, k_dt))) return rc;
    if ((rc = check_params(p->lambda, p->d_c, p->d_n, p->alpha))) return rc;
    if (p->fallback_T < 0) return PACT_ERR_PARAM;
    const WsLayout L = make_layout(n, 1, n, (int64_t)n_q * d_h, n_q, (int64_t)n_kv * d_h, k_dt);
    if (own_scratch) {
        if (L.total > (size_t)PACT_STATIC_SCRATCH_BYTES) return PACT_ERR_WORKSPACE;
    } else if ((rc = check_ws(ws, ws_bytes, L.total))) return rc;
    if ((rc = check_device())) return rc;
    if (own_scratch && (rc = own_scratch_address(&ws))) return rc;
    Batch bt;
    fill_single(bt, n, *p);
    const Ws w = resolve(ws, L);
    ReduceIO io{hidden, h_dt, h, keys_pre, keys, k_dt, n_kv, d_h, q, q_dt, q_rows == n ? 1 : 0, n_q,
                scores, kept_idx, pruned_idx, center_idx, cluster_id, merged, out_dt, cluster_counts, rep};
    return run_reduce(bt, w, io, (hipStream_t)stream);
}

int pact_reduce(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
                const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                const pact_params* p,
                float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                pact_report* rep, void* ws, size_t ws_bytes, void* stream) {
    return reduce_single(hidden, h_dt, n, h, keys_pre, keys, k_dt, n_kv, d_h, q, q_dt, q_rows, n_q, p, scores,
                         kept_idx, pruned_idx, center_idx, cluster_id, merged, out_dt, cluster_counts, rep,
                         ws, ws_bytes, false, stream);
}

int pact_reduce_static(const void* hidden, pact_dtype h_dt, int32_t n, int32_t h,
                       const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                       const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                       const pact_params* p,
                       float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                       int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                       pact_report* rep, void* stream) {
    return reduce_single(hidden, h_dt, n, h, keys_pre, keys, k_dt, n_kv, d_h, q, q_dt, q_rows, n_q, p, scores,
                         kept_idx, pruned_idx, center_idx, cluster_id, merged, out_dt, cluster_counts, rep,
                         nullptr, 0, true, stream);
}

int pact_reduce_varlen(const void* hidden, pact_dtype h_dt, int32_t h,
                       const void* keys_pre, const void* keys, pact_dtype k_dt, int32_t n_kv, int32_t d_h,
                       const void* q, pact_dtype q_dt, int32_t q_rows, int32_t n_q,
                       const int32_t* cu_seqlens, int32_t batch, const pact_params* p,
                       float* scores, int32_t* kept_idx, int32_t* pruned_idx, int32_t* center_idx,
                       int32_t* cluster_id, void* merged, pact_dtype out_dt, int32_t* cluster_counts,
                       pact_report* rep, void* ws, size_t ws_bytes, void* stream) {
    if (!p || !cu_seqlens) return PACT_ERR_NULL;
    int rc = validate_reduce_common(hidden, h_dt, h, keys_pre, keys, k_dt, n_kv, d_h, q, q_dt, n_q, scores,
                                    kept_idx, pruned_idx, center_idx, cluster_id, merged, out_dt,
                                    cluster_counts, rep);
    if (rc) return rc;
    if (batch < 1 || batch > PACT_MAX_BATCH || cu_seqlens[0] != 0) return PACT_ERR_SHAPE;
    Batch bt;
    std::memset(&bt, 0, sizeof(bt));
    int32_t n_max = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t nb = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
        if (nb < 1 || nb > PACT_MAX_TOKENS) return PACT_ERR_SHAPE;
        if ((rc = check_params(p[b].lambda, p[b].d_c, p[b].d_n, p[b].alpha))) return rc;
        if (p[b].fallback_T < 0) return PACT_ERR_PARAM;
        bt.s[b].base = cu_seqlens[b]; bt.s[b].n = (int32_t)nb;
        bt.s[b].lambda = p[b].lambda; bt.s[b].d_c = p[b].d_c; bt.s[b].d_n = p[b].d_n;
        bt.s[b].alpha = p[b].alpha; bt.s[b].fallback_T = p[b].fallback_T; bt.s[b].flags = p[b].flags;
        if (nb > n_max) n_max = (int32_t)nb;
    }
    const int32_t total = cu_seqlens[batch];
    if (q_rows != total && q_rows != batch) return PACT_ERR_SHAPE;
    if ((rc = check_key_extent(n_max, (int64_t)n_kv * d_h, k_dt))) return rc;
    bt.B = batch; bt.n_max = n_max; bt.W = (n_max + 63) / 64; bt.total = total;
    const WsLayout L = make_layout(n_max, batch, (int64_t)n_max * batch, (int64_t)n_q * d_h, n_q, (int64_t)n_kv * d_h, k_dt);
    if ((rc = check_ws(ws, ws_bytes, L.total))) return rc;
    if ((rc = check_device())) return rc;
    const Ws w = resolve(ws, L);
    const int per_token = q_rows == total ? 1 : 0;
    ReduceIO io{hidden, h_dt, h, keys_pre, keys, k_dt, n_kv, d_h, q, q_dt, per_token, n_q,
                scores, kept_idx, pruned_idx, center_idx, cluster_id, merged, out_dt, cluster_counts, rep};
    return run_reduce(bt, w, io, (hipStream_t)stream);
}

int pact_attention_handoff(const int32_t* center_idx, const int32_t* cluster_counts, const pact_report* rep,
                           const int32_t* positions, const int32_t* cu_seqlens, int32_t batch, int32_t n,
                           int32_t* positions_out, float* log_weight, void* stream) {
    if (!center_idx || !cluster_counts || !rep || !positions_out || !log_weight) return PACT_ERR_NULL;
    if (batch < 1 || batch > PACT_MAX_BATCH) return PACT_ERR_SHAPE;
    if (!cu_seqlens && batch != 1) return PACT_ERR_NULL;
    Batch bt;
    std::memset(&bt, 0, sizeof(bt));
    int32_t n_max = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t base = cu_seqlens ? cu_seqlens[b] : 0;
        const int64_t nb = cu_seqlens ? (int64_t)cu_seqlens[b + 1] - cu_seqlens[b] : n;
        if (nb < 1 || nb > PACT_MAX_TOKENS || base < 0 || (cu_seqlens && b == 0 && base != 0)) return PACT_ERR_SHAPE;
        bt.s[b].base = (int32_t)base; bt.s[b].n = (int32_t)nb;
        if (nb > n_max) n_max = (int32_t)nb;
    }
    bt.B = batch; bt.n_max = n_max; bt.W = (n_max + 63) / 64;
    bt.total = cu_seqlens ? cu_seqlens[batch] : n;
    int rc;
    if ((rc = check_device())) return rc;
    return launch_handoff(bt, center_idx, cluster_counts, rep, positions, positions_out, log_weight,
                          (hipStream_t)stream);
}

int pact_profile_enable(int on) {
    g_prof_on = on != 0;
    return PACT_OK;
}
int pact_profile_reset(void) {
    g_prof_used = 0;
    return PACT_OK;
}
int pact_profile_read(const char** names, float* ms, int32_t max_records) {
    int n = 0;
    for (size_t i = 0; i < g_prof_used && n < max_records; ++i, ++n) {
        float t = 0.0f;
        if (hipEventSynchronize(g_prof[i].b) != hipSuccess) return -1;
        if (hipEventElapsedTime(&t, g_prof[i].a, g_prof[i].b) != hipSuccess) return -1;
        if (names) names[n] = g_prof[i].name;
        if (ms) ms[n] = t;
    }
    return n;
}

int pact_calibration_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return PACT_ERR_NULL;
    if (bytes == 0 || bytes % 16 || bytes > (size_t(1) << 34)) return PACT_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15) return PACT_ERR_ALIGN;
    int rc;
    if ((rc = check_device())) return rc;
    const size_t n16 = bytes / 16;
    const unsigned grid = (unsigned)std::min<size_t>((n16 + 255) / 256, 256 * 16);
    hipLaunchKernelGGL(pact::calibration_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream,
                       (uint4*)dst, (const uint4*)src, n16);
    return hipGetLastError() == hipSuccess ? PACT_OK : PACT_ERR_HIP;
}

int pact_plan_workgroups(const int32_t* tiles, int32_t batch, uint16_t* wg_map, uint16_t* wg_count) {
    return plan_gram_workgroups(tiles, batch, wg_map, wg_count);
}

const char* pact_strerror(int status) {
    switch (status) {
        case PACT_OK: return "ok";
        case PACT_ERR_NULL: return "a required pointer is NULL";
        case PACT_ERR_SHAPE: return "a size is out of range or inconsistent";
        case PACT_ERR_DTYPE: return "unknown dtype";
        case PACT_ERR_PARAM: return "lambda, d_c, d_n, alpha or fallback_T out of range";
        case PACT_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
        case PACT_ERR_ALIGN: return "a tensor row is not 16-byte aligned";
        case PACT_ERR_HIP: return "a HIP call failed while enqueueing";
        case PACT_ERR_NOGPU: return "no usable gfx950 device";
        default: return "unknown status";
    }
}

}  // extern "C"

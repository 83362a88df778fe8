"""Plain CPU oracle for PACT's token-reduction step (EUTI -> DBDPC -> recovery -> merge).

TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of
what the GPU library must compute.  It is imported by tests/, by the smoke check
and by the benchmark's cpu_baseline leg, and by nothing on the product path.  It
shares no code with the HIP sources and does not import them.

Everything is float64 numpy.  Inputs may be float32 arrays (bf16 inputs arrive as
float32 arrays holding bf16-representable values); they are widened exactly.

Notation follows the paper:
  n      visual tokens, d hidden width, n_h heads of width d_h
  H      hidden states [n, d]                         (Method, first paragraph)
  K, Q   keys / queries [n, n_h, d_h]                  (Method, first paragraph)
  s      importance scores [n]                          (Eq. 2, Alg. 1)
  lambda fraction of tokens deemed unimportant          (Eq. 3/4)
  u_i    the vectors DBDPC clusters, here flattened keys (Sec. 3.2)
  d_ij   cosine distance                                (Eq. 5)
  rho_i  local density, normalised by d_n               (Eq. 6)
  d_c    cutoff distance, alpha recovery coefficient    (Alg. 2, Eq. 8)

Readings taken where the paper is silent (each is restated at the function that
uses it):
  * grouped-query attention: query head j reads key head j // (n_q / n_kv);
  * Percentile(s, lambda) is the (m+1)-th smallest score, m = min(floor(lambda n), n-1),
    so ties at the threshold are all kept;
  * equal densities: the lower index is processed first (stable descending sort);
  * equal distances in an argmin: the centre with the lower token index wins;
  * d_ii = 0 exactly; a zero vector has cosine 0 (distance 1) to everything else;
  * cluster ids number the centres in ascending token index.

No function here has "parity unpinned": every one is pinned by tests/test_oracle_*.py
(closed forms, brute force on tiny inputs, invariants of the paper's appendix B,
the equivalence with the recursive centre identification of appendix D, and the
membership picture of Fig. 1).
"""
from __future__ import annotations

import math

import numpy as np

F64 = np.float64


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=F64)


# --------------------------------------------------------------------------- EUTI (Alg. 1)

def q_global(Q) -> np.ndarray:
    """Eq. 1: the mean query over the n visual tokens, per head.  Q [n, n_q, d_h] -> [n_q, d_h]."""
    Q = _f64(Q)
    assert Q.ndim == 3
    return Q.sum(axis=0) / Q.shape[0]


def euti_logits(K, Qg) -> np.ndarray:
    """Per-head dot product k_i^(g(j)) . Q_global^(j) (inside Eq. 2).

    K [n, n_kv, d_h], Qg [n_q, d_h] -> [n, n_q].  With n_q == n_kv this is the
    paper's single-n_h formula; with n_q a multiple of n_kv, query head j is paired
    with key head j // (n_q // n_kv) (repeat-KV convention of grouped-query models).
    No 1/sqrt(d_h) scaling: Eq. 2 shows none.
    """
    K = _f64(K)
    Qg = _f64(Qg)
    n, n_kv, d_h = K.shape
    n_q = Qg.shape[0]
    assert Qg.shape[1] == d_h and n_q % n_kv == 0
    rep = n_q // n_kv
    out = np.empty((n, n_q), dtype=F64)
    for j in range(n_q):
        out[:, j] = K[:, j // rep, :] @ Qg[j, :]
    return out


def softmax_over_tokens(logits) -> np.ndarray:
    """Softmax across the visual tokens (axis 0) inside each head (text under Eq. 1)."""
    L = _f64(logits)
    e = np.exp(L - L.max(axis=0, keepdims=True))
    return e / e.sum(axis=0, keepdims=True)


def euti_scores(H, K, Q, *, use_norm: bool = True, use_query: bool = True) -> np.ndarray:
    """Eq. 2 / Alg. 1 step 2: s_i = mean_j softmax_i(k_i^(j) . Qg^(j)) * ||h_i||_2.

    Q may be [n, n_q, d_h] (Eq. 1 is applied) or an already averaged [n_q, d_h].
    use_norm=False / use_query=False are the two ablations of Eq. 2 the paper
    reports (score without the norm; norm only).
    """
    H = _f64(H)
    K = _f64(K)
    Q = _f64(Q)
    Qg = q_global(Q) if Q.ndim == 3 else Q
    n = H.shape[0]
    if use_query:
        p = softmax_over_tokens(euti_logits(K, Qg)).mean(axis=1)
    else:
        p = np.full(n, 1.0 / n, dtype=F64)
    if use_norm:
        return p * np.sqrt((H * H).sum(axis=1))
    return p


def percentile_rank(n: int, lam: float) -> int:
    """Number of scores strictly below the threshold when all scores are distinct:
    m = min(floor(lambda * n), n - 1).  lambda is 'the percentage of tokens deemed
    unimportant' (text above Eq. 3)."""
    return min(int(math.floor(float(lam) * n)), n - 1)


def percentile_split(s, lam: float):
    """Eq. 3/4: S_important = {s_i >= tau}, S_unimportant = {s_i < tau} with
    tau = Percentile(s, lambda) read as the (m+1)-th smallest score.  Returns
    (kept, pruned, tau), both index arrays ascending."""
    s = np.asarray(s)
    n = s.shape[0]
    m = percentile_rank(n, lam)
    tau = np.sort(s, kind="stable")[m]
    kept = np.flatnonzero(s >= tau)
    pruned = np.flatnonzero(s < tau)
    return kept, pruned, tau


# --------------------------------------------------------------------------- DBDPC (Alg. 2)

def cosine_distance_matrix(U) -> np.ndarray:
    """Eq. 5 for all pairs of rows of U [q, d_1]: d_ij = 1 - u_i.u_j / (|u_i||u_j|).
    d_ii = 0 exactly; a zero row has cosine 0; rounding is clipped into [0, 2]."""
    U = _f64(U)
    G = U @ U.T
    nn = np.diag(G).copy()
    D = _cos_to_dist(G, nn, nn)
    np.fill_diagonal(D, 0.0)
    return D


def cosine_distance_cross(A, B) -> np.ndarray:
    """Eq. 5 between every row of A [a, d_1] and every row of B [b, d_1]."""
    A = _f64(A)
    B = _f64(B)
    G = A @ B.T
    return _cos_to_dist(G, np.einsum("ij,ij->i", A, A), np.einsum("ij,ij->i", B, B))


def _cos_to_dist(G, nn_a, nn_b):
    denom = np.sqrt(np.outer(nn_a, nn_b))
    cos = np.zeros_like(G)
    np.divide(G, denom, out=cos, where=denom > 0)
    return np.clip(1.0 - cos, 0.0, 2.0)


def density(D, d_n: float) -> np.ndarray:
    """Eq. 6 / Alg. 2: rho_i = sum_{j=1..q} exp(-d_ij / d_n), the term j = i included.
    Each row is summed with math.fsum (the correctly rounded sum), so the value does
    not depend on the order of the terms: rows holding the same multiset of distances
    get bit-identical densities, as the algorithm's tie rule needs."""
    D = _f64(D)
    E = np.exp(-D / float(d_n))
    return np.array([math.fsum(row) for row in E], dtype=F64)


def density_order(rho) -> np.ndarray:
    """Alg. 2 'sort vectors by rho in descending order'.  Equal densities: lower
    index first (appendix D: one of them is treated as denser, by processing order)."""
    rho = _f64(rho)
    return np.argsort(-rho, kind="stable")


def select_centers(D, order, d_c: float) -> np.ndarray:
    """Alg. 2 centre loop, literally: the densest vector is a centre; each next vector
    in density order becomes a centre iff its minimum distance to the centres chosen
    so far is strictly greater than d_c.  Returns the centres in ascending index."""
    D = _f64(D)
    d_c = float(d_c)
    centers = []
    for k, i in enumerate(order):
        i = int(i)
        if k == 0 or D[i, centers].min() > d_c:
            centers.append(i)
    return np.array(sorted(centers), dtype=np.int64)


def assign_to_centers(D_to_centers) -> np.ndarray:
    """Alg. 2 last loop: s_i = argmin over centres of d_is.  D_to_centers [m, C] has one
    column per centre, centres in ascending token index; the first minimum wins, i.e.
    the centre with the lowest index."""
    Dc = _f64(D_to_centers)
    return np.argmin(Dc, axis=1).astype(np.int64)


def dbdpc(U, d_c: float, d_n: float):
    """Alg. 2 end to end on the rows of U.  Returns dict(centers, labels, rho, order, D):
    centers ascending row indices, labels[i] = position of i's centre in `centers`."""
    D = cosine_distance_matrix(U)
    rho = density(D, d_n)
    order = density_order(rho)
    centers = select_centers(D, order, d_c)
    labels = assign_to_centers(D[:, centers])
    return dict(centers=centers, labels=labels, rho=rho, order=order, D=D)


# --------------------------------------------------------------------------- PACT (Alg. 3)

def reincorporate(D_pruned_to_centers, d_c: float, alpha: float) -> np.ndarray:
    """Eq. 8/9, Alg. 3 step 3: an unimportant token joins its nearest centre s iff
    d_is < alpha * d_c (strict).  Returns labels [n_pruned], -1 = stays dropped."""
    Dp = _f64(D_pruned_to_centers)
    if Dp.shape[0] == 0:
        return np.zeros(0, dtype=np.int64)
    s = np.argmin(Dp, axis=1)
    dmin = Dp[np.arange(Dp.shape[0]), s]
    return np.where(dmin < float(alpha) * float(d_c), s, -1).astype(np.int64)


def merge(H, cluster_id, n_clusters: int):
    """Eq. 10, Alg. 3 step 4: h'_s = mean of h_i over the members of cluster s
    (DBDPC members and recovered tokens alike).  Returns (merged [C, d], counts [C])."""
    H = _f64(H)
    cluster_id = np.asarray(cluster_id)
    merged = np.zeros((n_clusters, H.shape[1]), dtype=F64)
    counts = np.zeros(n_clusters, dtype=np.int64)
    for c in range(n_clusters):
        members = np.flatnonzero(cluster_id == c)
        counts[c] = members.size
        if members.size:
            merged[c] = H[members].sum(axis=0) / members.size
    return merged, counts


def centre_representatives(H, center_idx) -> np.ndarray:
    """The "no merging" variant of the ablation study (Sec. "Ablation study": the centre of each
    cluster stands for the cluster instead of the mean of its members): row s of the reduced
    set is the hidden state of centre s, unchanged."""
    H = _f64(H)
    return H[np.asarray(center_idx, dtype=np.int64)].copy()


def max_pairwise_distance(U) -> float:
    """The statistic Sec. "Selecting the layer L" (and the figure on the maximum distance
    between keys) looks at: the largest Eq. 5 distance between two of the vectors; 0 for a
    single vector."""
    D = cosine_distance_matrix(U)
    return float(D.max()) if D.shape[0] > 1 else 0.0


def attention_handoff(center_idx, counts, positions=None):
    """What the layers after the reduction need besides H' (Alg. 3 last loop, Eq. 11):
    the position id of every merged token, p'_s = p_s of its cluster centre, and the
    additive attention term log W of proportional attention, log of the cluster sizes
    (a text token would carry log 1 = 0).  positions=None means p_i = i."""
    center_idx = np.asarray(center_idx, dtype=np.int64)
    counts = np.asarray(counts, dtype=np.int64)
    pos = center_idx.copy() if positions is None else np.asarray(positions)[center_idx]
    return pos, np.log(counts.astype(F64))


def pact_reduce(H, K_pre, Q, K_post, lam, d_c, d_n, alpha, *, score_dtype=np.float32,
                use_norm: bool = True, use_query: bool = True, merge_clusters: bool = True):
    """Alg. 3: EUTI on (H, K_pre, Q), DBDPC on the flattened K_post of the important
    tokens, recovery of unimportant tokens, merge, position = centre index.

    K_pre / Q are the keys and queries EUTI uses (before rotary embeddings), K_post
    the keys DBDPC uses (after); [n, n_kv, d_h] and [n, n_q, d_h] (or [n_q, d_h]).
    lam, d_c, d_n, alpha cross the library boundary as float32 and are rounded to it
    here first.  The scores also cross it as float32, so the percentile split is taken
    on the float32-rounded scores (score_dtype), the precision that decision is made
    in on both sides.  use_norm / use_query select the two ablations of Eq. 2 (see
    euti_scores); merge_clusters=False is the "no merging" variant (centre_representatives):
    clusters, recovery and counts as usual, the reduced rows are the centres' own.
    """
    lam, d_c, d_n, alpha = (float(np.float32(v)) for v in (lam, d_c, d_n, alpha))
    H = _f64(H)
    K_post = _f64(K_post)
    n = H.shape[0]
    U = K_post.reshape(n, -1)

    scores = euti_scores(H, K_pre, Q, use_norm=use_norm, use_query=use_query)
    s_dec = scores.astype(score_dtype)
    kept, pruned, tau = percentile_split(s_dec, lam)

    cl = dbdpc(U[kept], d_c, d_n)
    centers_local = cl["centers"]
    center_idx = kept[centers_local]
    cluster_id = np.full(n, -1, dtype=np.int64)
    cluster_id[kept] = cl["labels"]

    D_pc = cosine_distance_cross(U[pruned], U[center_idx])
    rl = reincorporate(D_pc, d_c, alpha)
    cluster_id[pruned] = rl

    merged, counts = merge(H, cluster_id, center_idx.size)
    if not merge_clusters:
        merged = centre_representatives(H, center_idx)
    return dict(
        scores=scores, scores_dec=s_dec, tau=tau, kept_idx=kept, pruned_idx=pruned,
        rho=cl["rho"], order=cl["order"], D_kept=cl["D"], D_pruned_centers=D_pc,
        center_idx=center_idx, cluster_id=cluster_id, merged=merged, counts=counts,
        n_reincorporated=int((rl >= 0).sum()), n_dropped=int((rl < 0).sum()),
    )

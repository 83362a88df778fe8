"""Pins for oracle/pact_oracle.py against things other than itself: closed forms,
library routines, brute force on tiny inputs, the invariants proved in the paper's
appendix B, the equivalence proved in appendix D, and the membership picture of Fig. 1.
CPU only."""
import math
import os

import numpy as np
import pytest
import scipy.spatial.distance as ssd
import scipy.special as ssp

from oracle import brute
from oracle import pact_oracle as po
from pact_synth import gen

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


# ------------------------------------------------------------------ Eq. 1 / Eq. 2

def test_q_global_is_token_mean_per_head():
    Q = np.array([[[1.0, 2.0]], [[3.0, 6.0]], [[5.0, 10.0]]])            # n=3, 1 head, d_h=2
    assert np.array_equal(po.q_global(Q), [[3.0, 6.0]])


def test_score_hand_example_one_head():
    # one head, d_h = 1: logits = k_i * Qg.  k = [0, ln3/2], Q = [1, 3] -> Qg = 2 -> logits [0, ln 3]
    # softmax over the two tokens = [1/4, 3/4]; |h| = [5, 13]
    K = np.array([[[0.0]], [[math.log(3.0) / 2]]])
    Q = np.array([[[1.0]], [[3.0]]])
    H = np.array([[3.0, 4.0], [5.0, 12.0]])
    s = po.euti_scores(H, K, Q)
    assert np.allclose(s, [0.25 * 5, 0.75 * 13], rtol=1e-14)


def test_softmax_is_over_tokens_not_heads():
    # 2 tokens x 2 heads; logits [[0, ln2], [ln3, 0]].  Over tokens: head0 -> [1/4, 3/4],
    # head1 -> [2/3, 1/3]; head mean -> [11/24, 13/24].  (Over heads it would be [1/3,2/3],[3/4,1/4].)
    L = np.array([[0.0, math.log(2.0)], [math.log(3.0), 0.0]])
    p = po.softmax_over_tokens(L)
    assert np.allclose(p, [[0.25, 2 / 3], [0.75, 1 / 3]], rtol=1e-14)
    K = np.zeros((2, 2, 2))
    K[0, 1, 0] = math.log(2.0)
    K[1, 0, 0] = math.log(3.0)
    Qg = np.array([[1.0, 0.0], [1.0, 0.0]])
    s = po.euti_scores(np.ones((2, 4)), K, Qg)
    assert np.allclose(s, np.array([11 / 24, 13 / 24]) * 2.0, rtol=1e-14)


def test_softmax_matches_library_routine():
    L = rng(0).normal(size=(50, 3)) * 4
    assert np.allclose(po.softmax_over_tokens(L), ssp.softmax(L, axis=0), rtol=1e-13)


def test_logits_against_explicit_loops_with_gqa():
    r = rng(1)
    n, n_kv, n_q, d_h = 7, 2, 6, 5
    K = r.normal(size=(n, n_kv, d_h))
    Qg = r.normal(size=(n_q, d_h))
    L = po.euti_logits(K, Qg)
    for i in range(n):
        for j in range(n_q):
            g = j // 3
            assert math.isclose(L[i, j], sum(K[i, g, k] * Qg[j, k] for k in range(d_h)),
                                rel_tol=1e-12, abs_tol=1e-14)


def test_scores_over_norm_sum_to_one_and_norm_only_cases():
    s = gen.make_sample("tiny_f32", 3)
    sc = po.euti_scores(s.hidden, s.keys, s.queries)
    hn = np.linalg.norm(s.hidden.astype(np.float64), axis=1)
    assert math.isclose((sc / hn).sum(), 1.0, rel_tol=1e-12)
    n = s.n
    same_keys = np.broadcast_to(s.keys[:1], s.keys.shape)
    assert np.allclose(po.euti_scores(s.hidden, same_keys, s.queries), hn / n, rtol=1e-12)
    zero_q = np.zeros_like(s.queries)
    assert np.allclose(po.euti_scores(s.hidden, s.keys, zero_q), hn / n, rtol=1e-12)
    assert np.allclose(po.euti_scores(s.hidden, s.keys, s.queries, use_query=False), hn / n, rtol=1e-12)
    assert np.allclose(po.euti_scores(s.hidden, s.keys, s.queries, use_norm=False) * hn, sc, rtol=1e-12)


def test_scores_rank_like_softmax_when_norms_equal():
    s = gen.make_sample("tiny_f32", 4)
    H = s.hidden / np.linalg.norm(s.hidden, axis=1, keepdims=True)
    sc = po.euti_scores(H, s.keys, s.queries)
    p = ssp.softmax(po.euti_logits(s.keys, po.q_global(s.queries)), axis=0).mean(axis=1)
    assert np.array_equal(np.argsort(sc, kind="stable"), np.argsort(p, kind="stable"))


# ------------------------------------------------------------------ Eq. 3 / Eq. 4

@pytest.mark.parametrize("lam", [0.0, 0.1, 0.3, 0.45, 0.5, 0.77, 1.0])
def test_percentile_split_bruteforce(lam):
    s = rng(5).permutation(101).astype(np.float64)          # distinct
    kept, pruned, tau = po.percentile_split(s, lam)
    m = min(int(math.floor(lam * 101)), 100)
    assert len(pruned) == m and len(kept) == 101 - m
    assert sorted(list(kept) + list(pruned)) == list(range(101))
    assert tau == sorted(s)[m]
    assert all(s[i] >= tau for i in kept) and all(s[i] < tau for i in pruned)
    assert list(kept) == sorted(kept) and list(pruned) == sorted(pruned)
    if m:
        assert s[kept].min() > s[pruned].max()


def test_percentile_extremes_and_ties():
    s = np.array([3.0, 1.0, 2.0, 2.0, 5.0])
    kept, pruned, _ = po.percentile_split(s, 0.0)
    assert list(kept) == [0, 1, 2, 3, 4] and len(pruned) == 0
    kept, pruned, tau = po.percentile_split(s, 1.0)          # m = n-1 -> tau = max
    assert list(kept) == [4] and tau == 5.0
    kept, pruned, tau = po.percentile_split(s, 0.4)          # m = 2 -> tau = 2.0, both 2.0's kept
    assert tau == 2.0 and list(kept) == [0, 2, 3, 4] and list(pruned) == [1]
    kept, pruned, _ = po.percentile_split(np.full(6, 7.0), 0.5)   # all equal: nothing below tau
    assert len(kept) == 6 and len(pruned) == 0


# ------------------------------------------------------------------ Eq. 5

def test_distance_closed_forms():
    U = np.array([[1.0, 0.0], [0.0, 2.0], [-3.0, 0.0], [1.0, 1.0], [0.0, 0.0], [5.0, 0.0]])
    D = po.cosine_distance_matrix(U)
    assert D[0, 1] == 1.0 and D[0, 2] == 2.0 and D[0, 5] == 0.0
    assert math.isclose(D[0, 3], 1 - math.sqrt(0.5), rel_tol=1e-15)
    assert np.all(D[4, [0, 1, 2, 3, 5]] == 1.0)               # zero vector: cosine 0
    assert np.all(np.diag(D) == 0.0)
    assert np.array_equal(D, D.T)


def test_distance_matches_library_and_loops():
    U = rng(7).normal(size=(23, 9))
    D = po.cosine_distance_matrix(U)
    ref = ssd.cdist(U, U, metric="cosine")
    np.fill_diagonal(ref, 0.0)
    assert np.allclose(D, ref, atol=1e-14)
    assert np.allclose(D, brute.distance_loops(U), atol=1e-14)
    assert D.min() >= 0 and D.max() <= 2
    scale = np.exp(rng(8).normal(size=(23, 1)))
    assert np.allclose(po.cosine_distance_matrix(U * scale), D, atol=1e-14)
    A, B = U[:5], U[5:]
    assert np.allclose(po.cosine_distance_cross(A, B), ssd.cdist(A, B, metric="cosine"), atol=1e-14)


# ------------------------------------------------------------------ Eq. 6

def test_density_closed_forms():
    d_n = 2.0
    q = 9
    same = np.tile(np.array([[0.3, -1.0, 2.0]]), (q, 1))
    assert np.array_equal(po.density(po.cosine_distance_matrix(same), d_n), np.full(q, float(q)))
    eye = np.eye(q)
    rho = po.density(po.cosine_distance_matrix(eye), d_n)
    assert np.allclose(rho, 1 + (q - 1) * math.exp(-1 / d_n), rtol=1e-15)
    assert len(set(rho.tolist())) == 1                        # bit-identical (needed by the tie rule)
    a, b = 4, 3
    U = np.array([[1.0, 0.0]] * a + [[-2.0, 0.0]] * b)
    rho = po.density(po.cosine_distance_matrix(U), 0.7)
    assert np.allclose(rho[:a], a + b * math.exp(-2 / 0.7), rtol=1e-15)
    assert np.allclose(rho[a:], b + a * math.exp(-2 / 0.7), rtol=1e-15)


def test_density_matches_loops_bounds_and_is_order_independent():
    U = rng(11).normal(size=(31, 6))
    D = po.cosine_distance_matrix(U)
    for d_n in (0.5, 2.0):
        rho = po.density(D, d_n)
        assert np.allclose(rho, brute.density_loops(D, d_n), rtol=1e-13)
        assert np.all(rho >= 1 + 30 * math.exp(-2 / d_n)) and np.all(rho <= 31)
    perm = rng(12).permutation(31)
    rho_p = po.density(D[np.ix_(perm, perm)], 2.0)           # same distances, other order
    assert np.array_equal(rho_p, po.density(D, 2.0)[perm])


# ------------------------------------------------------------------ density order, centres

def test_density_order_ties_lower_index_first():
    rho = np.array([2.0, 5.0, 5.0, 1.0, 5.0, 2.0])
    assert list(po.density_order(rho)) == [1, 2, 4, 0, 5, 3]
    assert list(po.density_order(rho)) == brute.order_by_definition(rho)


def _circle(deg):
    a = np.deg2rad(np.asarray(deg, dtype=np.float64))
    return np.stack([np.cos(a), np.sin(a)], axis=1)


def test_dbdpc_hand_example_on_circle():
    # Unit vectors at 0, 10, 20, 185, 196 degrees; d = 1 - cos(angle between); d_n = 2;
    # d_c = 1 - cos(15 deg).  Pairs within d_c: (0,10), (10,20), (185,196).
    # Sum of exp(-d/2) over the others, by hand:
    #   10 deg: 2 x 0.99243 (10 deg away) + 0.36860 (175) + 0.36889 (174)      = 2.7224
    #    0 deg: 0.99243 + 0.97030 (20 deg away) + 0.36860 (175) + 0.37507 (164) = 2.7064
    #  196 deg: 0.99084 (11) + 0.37507 (164) + 0.36889 (174) + 0.36832 (176)    = 2.1031
    #  185 deg: 0.99084 (11) + 0.36860 + 0.36860 (175, 175) + 0.37420 (165)     = 2.1022
    # -> 10 deg is the densest: centre; 0 and 20 are within d_c of it.  196 deg is denser than
    #    185 deg: centre; 185 is within d_c of it.  Centres {1, 4}.
    U = _circle([0, 10, 20, 185, 196])
    d_c = 1 - math.cos(math.radians(15))
    out = po.dbdpc(U, d_c, 2.0)
    assert np.allclose(out["rho"] - 1, [2.7064, 2.7224, 2.7064 + 0.0, 2.1022, 2.1031], atol=6e-3)
    assert int(out["order"][0]) == 1
    assert out["rho"][4] > out["rho"][3]
    assert list(out["centers"]) == [1, 4]
    assert list(out["labels"]) == [0, 0, 0, 1, 1]
    # with the cutoff below 10 degrees every point is its own centre
    out = po.dbdpc(U, 1 - math.cos(math.radians(9)), 2.0)
    assert list(out["centers"]) == [0, 1, 2, 3, 4]


def test_centre_strictness_at_exact_threshold():
    # orthogonal unit vectors: every distance is exactly 1.  Centre iff min distance > d_c.
    U = np.eye(4)
    D = po.cosine_distance_matrix(U)
    order = po.density_order(po.density(D, 2.0))
    assert list(order) == [0, 1, 2, 3]                        # all densities equal -> index order
    assert list(po.select_centers(D, order, 1.0)) == [0]      # 1 > 1 is false
    assert list(po.select_centers(D, order, np.nextafter(1.0, 0))) == [0, 1, 2, 3]
    assert list(po.select_centers(D, order, 2.0)) == [0]
    assert list(po.select_centers(D, order, 0.0)) == [0, 1, 2, 3]


@pytest.mark.parametrize("seed", range(12))
def test_centres_are_the_unique_fixed_point_tiny(seed):
    r = rng(100 + seed)
    q = int(r.integers(3, 11))
    U = r.normal(size=(q, 3))
    if seed % 3 == 1:                                         # exact duplicates -> distance and density ties
        U[q // 2] = U[0]
        U[q - 1] = 2 * U[1]
    if seed % 3 == 2:                                         # orthonormal directions -> all ties
        U = np.concatenate([np.eye(3), np.eye(3)[: max(q - 3, 0) % 4]])
        q = U.shape[0]
    D = po.cosine_distance_matrix(U)
    rho = po.density(D, 2.0)
    order = po.density_order(rho)
    assert list(order) == brute.order_by_definition(rho)
    for d_c in (0.0, 0.05, 0.3, 0.8, 1.0, 1.5, 2.0):
        got = list(po.select_centers(D, order, d_c))
        fixed = brute.centers_fixed_point_enumeration(D, order, d_c)
        assert fixed == [got], (seed, d_c, fixed, got)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("T", [0, 1, 10, 10 ** 9])
def test_recursive_centre_identification_equals_sequential(seed, T):
    r = rng(200 + seed)
    q = 70
    blobs = r.normal(size=(6, 8))
    U = blobs[r.integers(0, 6, q)] + 0.25 * r.normal(size=(q, 8))
    if seed % 2:
        U[10] = U[3]
        U[40] = U[3]
    D = po.cosine_distance_matrix(U)
    rho = po.density(D, 2.0)
    order = po.density_order(rho)
    for d_c in (0.02, 0.1, 0.4):
        a = po.select_centers(D, order, d_c)
        b = brute.recursive_centers(D, rho, d_c, T)
        assert np.array_equal(a, b), (seed, T, d_c)


@pytest.mark.parametrize("name,seed", [("tiny_f32", 0), ("tiny_bf16", 1), ("img_0p5b", 2)])
def test_dbdpc_guarantees_of_appendix_b(name, seed):
    s = gen.make_sample(name, seed)
    U = s.keys.reshape(s.n, -1).astype(np.float64)
    for d_c in (0.005, 0.015, 0.05, 0.5):
        out = po.dbdpc(U, d_c, 2.0)
        D, c, lab = out["D"], out["centers"], out["labels"]
        assert np.all(D[np.arange(s.n), c[lab]] <= d_c)                       # member within d_c of its centre
        Dcc = D[np.ix_(c, c)] + np.eye(c.size) * 10
        assert np.all(Dcc > d_c)                                             # centres pairwise farther than d_c
        assert np.array_equal(lab[c], np.arange(c.size))                     # a centre belongs to itself
        bound = 2 * d_c * (2 - d_c)
        for k in range(c.size):
            mem = np.flatnonzero(lab == k)
            assert np.all(D[np.ix_(mem, mem)] <= bound + 1e-12)              # intra-cluster bound
        assert np.array_equal(lab, np.argmin(D[:, c], axis=1))


def test_dbdpc_special_cases():
    r = rng(17)
    U = r.normal(size=(20, 5))
    out = po.dbdpc(U, 2.0, 2.0)                               # cutoff >= 2: one centre, the densest
    assert list(out["centers"]) == [int(np.argmax(out["rho"]))] and np.all(out["labels"] == 0)
    out = po.dbdpc(U, 0.0, 2.0)                               # cutoff 0, distinct directions: all centres
    assert list(out["centers"]) == list(range(20)) and list(out["labels"]) == list(range(20))
    V = np.array([[1.0, 2.0, 2.0], [0.0, 3.0, 4.0], [2.0, 4.0, 4.0], [1.0, 2.0, 2.0], [0.0, 6.0, 8.0]])
    out = po.dbdpc(V, 0.0, 2.0)                               # exact duplicates merge into the lowest copy
    assert list(out["centers"]) == [0, 1] and list(out["labels"]) == [0, 1, 0, 0, 1]


# ------------------------------------------------------------------ assignment, recovery (Eq. 8/9)

def test_assignment_bruteforce_and_tie_break():
    Dc = rng(21).random(size=(40, 7))
    lab = po.assign_to_centers(Dc)
    for i in range(40):
        best = min(range(7), key=lambda c: (Dc[i, c], c))
        assert lab[i] == best
    # token (1,1) is exactly equidistant from centres (1,0) and (0,1): the lower index wins
    D = po.cosine_distance_cross(np.array([[1.0, 1.0]]), np.array([[1.0, 0.0], [0.0, 1.0]]))
    assert D[0, 0] == D[0, 1] and po.assign_to_centers(D)[0] == 0


def test_reincorporation_threshold_is_strict_and_alpha_limits():
    P = np.array([[0.0, 1.0], [1.0, 1.0], [-1.0, 0.0]])
    Cn = np.array([[1.0, 0.0]])
    D = po.cosine_distance_cross(P, Cn)                      # [1, 1-sqrt(.5), 2]
    assert D[0, 0] == 1.0 and D[2, 0] == 2.0
    assert list(po.reincorporate(D, 0.5, 2.0)) == [-1, 0, -1]                # 1 < 1 false
    assert list(po.reincorporate(D, 0.5, np.nextafter(2.0, 3))) == [0, 0, -1]
    assert list(po.reincorporate(D, 0.5, 0.0)) == [-1, -1, -1]               # alpha = 0: no recovery
    assert list(po.reincorporate(D, 1.0, 2.0000001)) == [0, 0, 0]            # alpha d_c > 2: everything
    Dr = rng(22).random(size=(30, 5))
    lab = po.reincorporate(Dr, 0.2, 1.5)
    for i in range(30):
        c = min(range(5), key=lambda k: (Dr[i, k], k))
        assert lab[i] == (c if Dr[i, c] < 0.3 else -1)
    assert po.reincorporate(np.zeros((0, 3)), 0.2, 1.5).size == 0


def test_fig1_membership_bookkeeping():
    """Fig. 1's picture with its centres {2,6,10} forced: Euclidean distance, radius 0.45,
    alpha = 1.  Kept points go to the nearest centre, pruned 12 and 13 are re-added,
    14 and 15 stay out; the merged token is the members' mean."""
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "fig1_points.txt")) if not ln.startswith("#")]
    ids = np.array([int(r[0]) for r in rows])
    P = np.array([[float(r[1]), float(r[2])] for r in rows])
    kept_flag = np.array([int(r[3]) for r in rows]) == 1
    want_centre = np.array([int(r[4]) for r in rows])
    centres = np.array([2, 6, 10]) - 1
    kept = np.flatnonzero(kept_flag)
    pruned = np.flatnonzero(~kept_flag)
    E = ssd.cdist(P, P)
    cluster_id = np.full(15, -1)
    cluster_id[kept] = po.assign_to_centers(E[np.ix_(kept, centres)])
    assert np.all(E[kept, centres[cluster_id[kept]]] <= 0.45)
    cluster_id[pruned] = po.reincorporate(E[np.ix_(pruned, centres)], 0.45, 1.0)
    got_centre = np.where(cluster_id >= 0, ids[centres][np.maximum(cluster_id, 0)], 0)
    assert np.array_equal(got_centre, want_centre)
    merged, counts = po.merge(P, cluster_id, 3)
    assert list(counts) == [4, 5, 4]
    assert np.allclose(merged[1], P[[4, 5, 6, 7, 11]].mean(axis=0), rtol=1e-15)


# ------------------------------------------------------------------ Eq. 10 and the whole of Alg. 3

def test_merge_identities():
    r = rng(31)
    H = r.normal(size=(50, 6)).astype(np.float32)
    cid = r.integers(-1, 8, 50)
    cid[7] = 8                                                # singleton cluster
    merged, counts = po.merge(H, cid, 9)
    ref, cnt = brute.merge_loops(H, cid, 9)
    assert np.allclose(merged, ref, rtol=1e-14) and np.array_equal(counts, cnt)
    assert counts.sum() == (cid >= 0).sum()
    assert np.allclose((merged * counts[:, None]).sum(0), H[cid >= 0].astype(np.float64).sum(0), atol=1e-12)
    assert np.array_equal(merged[8], H[7].astype(np.float64))


def test_no_merging_variant_keeps_the_centre_rows():
    # the ablation that lets the centre stand for its cluster: rows of H at the centres, bit for bit,
    # in the order of the centres; everything but the rows is the full method's
    r = rng(33)
    H = r.normal(size=(20, 5)).astype(np.float32)
    centres = np.array([2, 7, 11, 19])
    rows = po.centre_representatives(H, centres)
    assert rows.shape == (4, 5) and all(np.array_equal(rows[k], H[c].astype(np.float64)) for k, c in enumerate(centres))
    rows[0, 0] = 99.0
    assert H[2, 0] != 99.0                                     # a copy, not a view
    s = gen.make_sample("tiny_f32", 4)
    d_c = 0.02
    a = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, d_c, 2.0, 1.5)
    b = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, d_c, 2.0, 1.5, merge_clusters=False)
    for k in ("kept_idx", "center_idx", "cluster_id", "counts"):
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(b["merged"], s.hidden[b["center_idx"]].astype(np.float64))
    single = a["counts"] == 1                                  # a cluster of one: mean and centre row coincide
    assert single.any() and np.array_equal(a["merged"][single], b["merged"][single])
    assert not np.array_equal(a["merged"][~single], b["merged"][~single])


@pytest.mark.parametrize("name,seed", [("tiny_f32", 5), ("tiny_bf16", 6)])
def test_pact_pipeline_conservation_and_limits(name, seed):
    s = gen.make_sample(name, seed)
    n = s.n
    U = s.keys.reshape(n, -1).astype(np.float64)
    d_c, alpha = 0.015, 1.5
    out = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, d_c, 2.0, alpha)
    d_c32, thr = float(np.float32(d_c)), float(np.float32(alpha)) * float(np.float32(d_c))
    cid, cidx = out["cluster_id"], out["center_idx"]
    C = cidx.size
    assert n == out["counts"].sum() + out["n_dropped"]
    assert out["counts"].sum() == out["kept_idx"].size + out["n_reincorporated"]
    assert np.all(cid[out["kept_idx"]] >= 0)                                  # every kept token is assigned
    assert set(np.flatnonzero(cid < 0)) <= set(out["pruned_idx"])             # only pruned tokens drop
    assert np.array_equal(cid[cidx], np.arange(C)) and list(cidx) == sorted(cidx)
    Dall = po.cosine_distance_cross(U, U[cidx])
    for i in out["kept_idx"]:
        assert Dall[i, cid[i]] <= d_c32 and cid[i] == np.argmin(Dall[i])
    for i in out["pruned_idx"]:
        if cid[i] >= 0:
            assert Dall[i, cid[i]] < thr and cid[i] == np.argmin(Dall[i])
        else:
            assert Dall[i].min() >= thr
    H = s.hidden.astype(np.float64)
    assert np.allclose((out["merged"] * out["counts"][:, None]).sum(0), H[cid >= 0].sum(0), atol=1e-9)
    # lambda = 0: PACT is DBDPC on all tokens
    o0 = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, 0.0, d_c, 2.0, alpha)
    cl = po.dbdpc(U, d_c32, 2.0)
    assert np.array_equal(o0["center_idx"], cl["centers"]) and np.array_equal(o0["cluster_id"], cl["labels"])
    # d_c = 0 with distinct directions: pruning only, merged = the kept rows, alpha irrelevant
    oz = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, 0.0, 2.0, alpha)
    assert np.array_equal(oz["center_idx"], oz["kept_idx"]) and oz["n_reincorporated"] == 0
    assert np.array_equal(oz["merged"], H[oz["kept_idx"]])
    # alpha = 0: no recovery; C unchanged
    oa = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, d_c, 2.0, 0.0)
    assert oa["n_reincorporated"] == 0 and np.array_equal(oa["center_idx"], cidx)


def test_generator_casts_are_exact_and_seeded():
    a = gen.make_sample("tiny_bf16", 3)
    b = gen.make_sample("tiny_bf16", 3)
    assert np.array_equal(a.keys, b.keys) and np.array_equal(a.hidden, b.hidden)
    assert not np.array_equal(a.keys, gen.make_sample("tiny_bf16", 4).keys)
    bits = gen.bf16_bits(a.keys)                               # raises if not representable
    back = (bits.astype(np.uint32) << 16).view(np.float32)
    assert np.array_equal(back, a.keys)
    x = np.array([1.0, 1.00390625, 1.005859375, 1.001953125, -3.3895313892515355e38], dtype=np.float32)
    assert np.array_equal(gen.round_to_bf16(x)[:4], np.array([1.0, 1.0, 1.0078125, 1.0], dtype=np.float32))


def test_attention_handoff_positions_and_weights():
    # Eq. 11 / Alg. 3: positions are the centres' own, log-weights are logs of cluster sizes
    cen = np.array([2, 5, 11])
    cnt = np.array([1, 4, 7])
    P = np.arange(100, 120) * 3
    pos, lw = po.attention_handoff(cen, cnt, P)
    assert list(pos) == [102 * 3, 105 * 3, 111 * 3]
    assert lw[0] == 0.0 and abs(lw[1] - 2 * math.log(2.0)) < 1e-15 and abs(math.exp(lw[2]) - 7.0) < 1e-12
    pos0, _ = po.attention_handoff(cen, cnt)
    assert list(pos0) == [2, 5, 11]
    # on a real reduction: weights sum to the number of tokens that survive in some cluster,
    # positions ascend (cluster ids follow the centres' token order)
    s = gen.make_sample("tiny_f32", 3)
    r = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, 0.05, 2.0, 1.5)
    pos, lw = po.attention_handoff(r["center_idx"], r["counts"])
    assert np.all(np.diff(pos) > 0)
    assert round(float(np.exp(lw).sum())) == s.n - r["n_dropped"]


def test_max_pairwise_distance_against_scipy_and_closed_forms():
    r = np.random.default_rng(11)
    U = r.normal(size=(40, 16))
    assert abs(po.max_pairwise_distance(U) - ssd.pdist(U, "cosine").max()) < 1e-13
    assert po.max_pairwise_distance(np.eye(5)) == 1.0                       # orthonormal: every pair at 1
    assert po.max_pairwise_distance(np.array([[1.0, 0.0], [-2.0, 0.0]])) == 2.0   # opposite directions
    assert po.max_pairwise_distance(np.tile(U[:1], (4, 1))) < 1e-15             # copies of one vector
    assert po.max_pairwise_distance(U[:1]) == 0.0

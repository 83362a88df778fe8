"""Second routes to the same answers, used only to pin oracle/pact_oracle.py.

TEST INFRASTRUCTURE ONLY (imported by tests/ alone).  Nothing here is shared with
pact_oracle.py beyond numpy: each function re-derives its quantity from the
definition with explicit Python loops, or follows a different algorithm the paper
proves equivalent.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


def distance_loops(U) -> np.ndarray:
    """Eq. 5 written out with scalar loops (dot, two norms, one division)."""
    U = np.asarray(U, dtype=np.float64)
    q, d = U.shape
    D = np.zeros((q, q))
    for i in range(q):
        for j in range(q):
            if i == j:
                continue
            dot = 0.0
            ni = 0.0
            nj = 0.0
            for k in range(d):
                dot += U[i, k] * U[j, k]
                ni += U[i, k] * U[i, k]
                nj += U[j, k] * U[j, k]
            den = math.sqrt(ni) * math.sqrt(nj)
            c = dot / den if den > 0 else 0.0
            D[i, j] = min(max(1.0 - c, 0.0), 2.0)
    return D


def density_loops(D, d_n) -> np.ndarray:
    """Eq. 6 with a scalar loop per row, j = i included."""
    q = D.shape[0]
    rho = np.zeros(q)
    for i in range(q):
        acc = 0.0
        for j in range(q):
            acc += math.exp(-D[i, j] / d_n)
        rho[i] = acc
    return rho


def order_by_definition(rho) -> list:
    """Density order as a total order: i precedes j iff rho_i > rho_j, or they are
    equal and i < j.  Built by counting predecessors, not by sorting."""
    q = len(rho)
    pos = [0] * q
    for i in range(q):
        pos[i] = sum(1 for j in range(q) if rho[j] > rho[i] or (rho[j] == rho[i] and j < i))
    order = [0] * q
    for i, p in enumerate(pos):
        order[p] = i
    return order


def centers_fixed_point_enumeration(D, order, d_c) -> list:
    """All subsets S of {0..q-1} such that, for every i: i in S  <=>  no j in S that
    precedes i in `order` has d_ij <= d_c.  Alg. 2's greedy set is the unique such S;
    exhaustive over 2^q subsets, so q <= ~14."""
    q = D.shape[0]
    pos = {int(i): k for k, i in enumerate(order)}
    found = []
    for bits in itertools.product((False, True), repeat=q):
        ok = True
        for i in range(q):
            blocked = any(bits[j] and pos[j] < pos[i] and D[i, j] <= d_c for j in range(q))
            if bits[i] == blocked:
                ok = False
                break
        if ok:
            found.append([i for i in range(q) if bits[i]])
    return found


def recursive_centers(D, rho, d_c, T) -> np.ndarray:
    """Centres by peeling (the scheme appendix D proves equal to Alg. 2's loop), stated with
    sets rather than as the printed procedure.  Let `before(i)` be the vectors that precede i
    in the density order and N(i) the vectors within d_c of i.  While vectors remain:
      * a remaining vector with no remaining vector of before(i) in N(i) has nothing left that
        could ever exclude it: all such vectors become centres together;
      * the new centres and every remaining vector in the N(.) of one of them leave;
      * once a peel yields fewer than T centres, what remains is taken one vector at a time in
        density order (a centre iff no centre so far is in its N(.)).
    T = 0 never leaves the peeling, T = infinity leaves it after the first peel."""
    D = np.asarray(D, dtype=np.float64)
    q = D.shape[0]
    order = order_by_definition(rho)
    position = {int(i): k for k, i in enumerate(order)}
    near = [set(int(j) for j in np.flatnonzero(D[i] <= d_c)) - {i} for i in range(q)]
    before = [set(int(j) for j in range(q) if position[j] < position[i]) for i in range(q)]
    remaining = set(range(q))
    centers = set()
    while remaining:
        peel = {i for i in remaining if not (near[i] & before[i] & remaining)}
        centers |= peel
        remaining -= peel
        remaining -= set().union(*(near[i] for i in peel)) if peel else set()
        if len(peel) < T:
            for i in sorted(remaining, key=position.get):
                if not (near[i] & centers):
                    centers.add(i)
            break
    return np.array(sorted(centers), dtype=np.int64)


def merge_loops(H, cluster_id, C):
    """Eq. 10 with explicit accumulation."""
    H = np.asarray(H, dtype=np.float64)
    out = np.zeros((C, H.shape[1]))
    cnt = np.zeros(C, dtype=np.int64)
    for i, c in enumerate(cluster_id):
        if c >= 0:
            out[c] += H[i]
            cnt[c] += 1
    for c in range(C):
        if cnt[c]:
            out[c] /= cnt[c]
    return out, cnt

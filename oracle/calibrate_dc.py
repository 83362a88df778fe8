"""Writes pact_synth/manifest.json: the cutoff distance d_c for every seeded synthetic
sample, chosen with the oracle so that the total reduction 1 - C/n hits the
configuration's target.

TEST INFRASTRUCTURE ONLY: calls oracle/ and the input generator, nothing else.
Run from the repository root:   python -m oracle.calibrate_dc [--missing] [group ...]
(--missing: only the samples that have no entry yet)

For each sample: scores, percentile split and the kept tokens' distance matrix and
density order are computed once; d_c is bisected on the number of centres Alg. 2
selects; the result is then moved to the middle of the widest gap between
consecutive pairwise distances in a +-0.2% window around it (so that no kept pair
sits on the threshold) and rounded to float32, the type it crosses the library
boundary in.  The entry records what the oracle then obtains (q, C, recovered,
dropped) and how close any decision-relevant distance comes to a threshold.
"""
from __future__ import annotations

import hashlib
import json
import os
import sys
import time

import numpy as np

from oracle import pact_oracle as po
from pact_synth import gen

D_N = 2.0
ALPHA = 1.5
MANIFEST = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                        "pact_synth", "manifest.json")


def sample_key(s: gen.Sample) -> str:
    grids = s.n // (s.config.gh * s.config.gw)
    heads = "" if s.queries.shape[1] == s.config.n_kv else f":q{s.queries.shape[1]}"      # query heads, if not one per key head
    return f"{s.config.name}:s{s.seed}:g{grids}:l{s.lam:.2f}{heads}"


def digest(a) -> str:
    """Fingerprint of an integer array (values as int64, in order): what the GPU tests compare where the
    oracle is not run again."""
    return hashlib.sha256(np.ascontiguousarray(a, dtype=np.int64).tobytes()).hexdigest()[:24]


def oracle_digests(s: gen.Sample, d_c: float) -> dict:
    """Fingerprints of the oracle's discrete results for the whole of Alg. 3 on sample s."""
    o = po.pact_reduce(s.hidden, s.keys, s.queries, s.keys, s.lam, d_c, D_N, ALPHA)
    return {"kept_idx": digest(o["kept_idx"]), "center_idx": digest(o["center_idx"]),
            "cluster_id": digest(o["cluster_id"]), "counts": digest(o["counts"])}


def calibrate(s: gen.Sample, target: float) -> dict:
    n = s.n
    U = np.asarray(s.keys, dtype=np.float64).reshape(n, -1)
    scores = po.euti_scores(s.hidden, s.keys, s.queries)
    kept, pruned, _ = po.percentile_split(scores.astype(np.float32), float(np.float32(s.lam)))
    D = po.cosine_distance_matrix(U[kept])
    rho = po.density(D, D_N)
    order = po.density_order(rho)
    want_c = max(1, int(round((1.0 - target) * n)))

    lo, hi = 0.0, 2.0
    for _ in range(40):
        mid = 0.5 * (lo + hi)
        if po.select_centers(D, order, mid).size > want_c:
            lo = mid
        else:
            hi = mid
        if hi - lo < 1e-7:
            break
    d0 = hi

    iu = np.triu_indices(D.shape[0], 1)
    allp = np.sort(D[iu])
    w = 0.002 * max(d0, 1e-3)
    a = max(min(int(np.searchsorted(allp, d0 - w, "left")),
                int(np.searchsorted(allp, d0, "right")) - 1), 0)
    b = min(max(int(np.searchsorted(allp, d0 + w, "right")),
                int(np.searchsorted(allp, d0, "right")) + 1), allp.size)
    dd = allp[a:b]
    if dd.size >= 2:
        k = int(np.argmax(np.diff(dd)))
        d_c = 0.5 * (dd[k] + dd[k + 1])
    else:
        d_c = d0
    d_c = float(np.float32(d_c))

    centers = po.select_centers(D, order, d_c)
    center_idx = kept[centers]
    D_pc = po.cosine_distance_cross(U[pruned], U[center_idx])
    rl = po.reincorporate(D_pc, d_c, ALPHA)
    thr = float(np.float32(ALPHA)) * d_c
    logits = po.euti_logits(s.keys, po.q_global(s.queries))
    p = po.softmax_over_tokens(logits)
    return {
        "d_c": d_c, "d_c_hex": float(d_c).hex(), "d_n": D_N, "alpha": ALPHA, "lambda": s.lam,
        "n": n, "q": int(kept.size), "C": int(centers.size),
        "n_reincorporated": int((rl >= 0).sum()), "n_dropped": int((rl < 0).sum()),
        "reduction": 1.0 - centers.size / n,
        "min_gap_to_dc": float(np.abs(D[iu] - d_c).min()) if iu[0].size else None,
        "min_gap_to_alpha_dc": float(np.abs(D_pc - thr).min()) if D_pc.size else None,
        "softmax_effective_support": [float(v) for v in 1.0 / (p * p).sum(axis=0)],
    }


def calibrate_vectors(U, target: float) -> dict:
    """DBDPC alone on the rows of U (nothing pruned, no recovery): d_c for a reduction 1 - C/n of
    `target`, moved to the middle of the widest nearby gap of pair distances like calibrate()."""
    U = np.asarray(U, dtype=np.float64)
    n = U.shape[0]
    D = po.cosine_distance_matrix(U)
    order = po.density_order(po.density(D, D_N))
    want_c = max(1, int(round((1.0 - target) * n)))
    lo, hi = 0.0, 2.0
    for _ in range(40):
        mid = 0.5 * (lo + hi)
        if po.select_centers(D, order, mid).size > want_c:
            lo = mid
        else:
            hi = mid
        if hi - lo < 1e-7:
            break
    d0 = hi
    allp = np.sort(D[np.triu_indices(n, 1)])
    w = 0.002 * max(d0, 1e-3)
    a = max(int(np.searchsorted(allp, d0 - w, "left")), 0)
    b = min(max(int(np.searchsorted(allp, d0 + w, "right")), a + 2), allp.size)
    dd = allp[a:b]
    k = int(np.argmax(np.diff(dd)))
    d_c = float(np.float32(0.5 * (dd[k] + dd[k + 1])))
    centers = po.select_centers(D, order, d_c)
    return {"d_c": d_c, "d_c_hex": float(d_c).hex(), "d_n": D_N, "n": n, "q": n, "C": int(centers.size),
            "reduction": 1.0 - centers.size / n, "min_gap_to_dc": float(np.abs(allp - d_c).min())}


def groups():
    g = {
        "tiny_f32": lambda: [gen.make_sample("tiny_f32", s) for s in range(10)],
        "tiny_bf16": lambda: [gen.make_sample("tiny_bf16", s) for s in range(10)],
        "img_0p5b": lambda: [gen.make_sample("img_0p5b", s) for s in range(10)],
        "img_7b": lambda: [gen.make_sample("img_7b", s) for s in range(10)],
        "vid_7b": lambda: [s for b in range(3) for s in gen.make_batch("vid_7b", b)],
        "varlen": lambda: [s for b in range(3) for s in gen.make_varlen_batch(b)],
        "vid_long": lambda: [gen.make_sample("vid_long", s) for s in range(3)],
        # the 7B-shaped image with the model's 28 query heads on its 4 key heads (scores, hence the kept set, differ)
        "img_7b_q28": lambda: [gen.make_sample("img_7b", s, n_q=28) for s in range(2)],
        # the long video with nothing pruned: all 16384 tokens are clustered
        "vid_long_all": lambda: [gen.make_sample("vid_long", 0, lam=0.0)],
        # further long videos, stored with fingerprints of the oracle's results (DIGEST_GROUPS)
        "vid_long_more": lambda: [gen.make_sample("vid_long", s) for s in range(3, 10)],
    }
    return g


DIGEST_GROUPS = ("vid_long_more",)


def main(argv):
    only_missing = "--missing" in argv
    argv = [a for a in argv if a != "--missing"]
    want = argv or list(groups().keys()) + ["img_7b_hidden"]
    manifest = {}
    if os.path.exists(MANIFEST):
        with open(MANIFEST) as f:
            manifest = json.load(f)
    if "img_7b_hidden" in want:
        # clustering on the hidden states instead of the keys (the ablation of Sec. "Ablation study"): the
        # 3584-wide hidden states of the benchmark image, 60% reduction as in the paper's DBDPC-only tables
        want = [w for w in want if w != "img_7b_hidden"]
        key = "img_7b:s0:g10:hidden"
        if not (only_missing and key in manifest):
            t = time.time()
            entry = calibrate_vectors(gen.make_sample("img_7b", 0).hidden, 0.60)
            if os.path.exists(MANIFEST):
                with open(MANIFEST) as f:
                    manifest = json.load(f)
            manifest[key] = entry
            print(f"{key}: d_c={entry['d_c']:.6f} C={entry['C']} reduction={entry['reduction']:.4f} "
                  f"gap={entry['min_gap_to_dc']:.2e} ({time.time() - t:.1f}s)", flush=True)
            with open(MANIFEST, "w") as f:
                json.dump(manifest, f, indent=1, sort_keys=True)
    for name in want:
        for s in groups()[name]():
            if only_missing and sample_key(s) in manifest:
                continue
            t = time.time()
            entry = calibrate(s, s.config.target_reduction)
            if name in DIGEST_GROUPS:
                entry["digest"] = oracle_digests(s, entry["d_c"])
            if os.path.exists(MANIFEST):           # (another run may have added entries meanwhile)
                with open(MANIFEST) as f:
                    manifest = json.load(f)
            manifest[sample_key(s)] = entry
            print(f"{sample_key(s)}: d_c={entry['d_c']:.6f} q={entry['q']} C={entry['C']} "
                  f"reduction={entry['reduction']:.4f} gap={entry['min_gap_to_dc']:.2e} "
                  f"({time.time() - t:.1f}s)", flush=True)
            with open(MANIFEST, "w") as f:
                json.dump(manifest, f, indent=1, sort_keys=True)


if __name__ == "__main__":
    main(sys.argv[1:])

"""Helpers for the GPU parity tests: move seeded samples to the device, call the library
through its binding, bring trimmed results back as numpy.  No method arithmetic."""
from __future__ import annotations

import json
import os

import numpy as np
import torch

import paper_2504_08966_amd as P
from pact_synth import gen

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_MANIFEST = None


def manifest():
    global _MANIFEST
    if _MANIFEST is None:
        with open(os.path.join(ROOT, "pact_synth", "manifest.json")) as f:
            _MANIFEST = json.load(f)
    return _MANIFEST


def sample_key(s: gen.Sample) -> str:
    grids = s.n // (s.config.gh * s.config.gw)
    heads = "" if s.queries.shape[1] == s.config.n_kv else f":q{s.queries.shape[1]}"      # query heads, if not one per key head
    return f"{s.config.name}:s{s.seed}:g{grids}:l{s.lam:.2f}{heads}"


def d_c_of(s: gen.Sample) -> float:
    return manifest()[sample_key(s)]["d_c"]


def dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def sample_to_dev(s: gen.Sample):
    n = s.n
    cfg = s.config
    return dict(hidden=dev(s.hidden, cfg.hidden_dtype),
                keys=dev(s.keys.reshape(n, -1), cfg.key_dtype),
                q=dev(s.queries.reshape(n, -1), cfg.key_dtype))


def trim(o, n, base=0, b=0):
    """Device outputs of one sample -> numpy, cut to the lengths the report gives."""
    rep = P.read_report(o["rep"])
    rep = rep[b] if isinstance(rep, list) else rep
    sl = slice(base, base + n)
    q, npr, C = rep["n_kept"], rep["n_pruned"], rep["n_centers"]
    return dict(
        rep=rep,
        scores=o["scores"][sl].cpu().numpy(),
        kept_idx=o["kept_idx"][base:base + q].cpu().numpy().astype(np.int64),
        pruned_idx=o["pruned_idx"][base:base + npr].cpu().numpy().astype(np.int64),
        center_idx=o["center_idx"][base:base + C].cpu().numpy().astype(np.int64),
        cluster_id=o["cluster_id"][sl].cpu().numpy().astype(np.int64),
        merged=o["merged"][base:base + C].float().cpu().numpy(),
        counts=o["cluster_counts"][base:base + C].cpu().numpy().astype(np.int64),
    )


def gpu_reduce(s: gen.Sample, d_c, d_n=2.0, alpha=1.5, lam=None, out_dtype=torch.float32, flags=0,
               fallback_T=10, ws=None):
    cfg = s.config
    d = sample_to_dev(s)
    prm = P.PactParams(s.lam if lam is None else lam, d_c, d_n, alpha, fallback_T, flags)
    o = P.pact_reduce(d["hidden"], d["keys"], d["keys"], d["q"], cfg.n_kv, cfg.d_h, cfg.n_kv, prm,
                      out_dtype=out_dtype, ws=ws)
    torch.cuda.synchronize()
    return trim(o, s.n)

"""Seeded synthetic inputs shaped like LLaVA-OneVision visual tokens.

Serves the oracle-side tests and the GPU-side tests/benchmark alike and holds none of
the method's arithmetic: it only draws random tensors.  Everything is generated in
float64 from numpy's PCG64 and cast ONCE to the configuration's storage type; the
cast values are the inputs for both sides.  bf16 tensors are returned as float32
arrays whose values are exactly bf16-representable.

Recipe (one image crop or video frame is a gh x gw grid of tokens):
  1. B blob centres, uniform on the unit sphere of R^Dk.
  2. Each grid gets a random Voronoi partition (sites at random grid cells, each site
     labelled with a random blob), so neighbouring tokens tend to share a blob.
     direction_i = normalise(centre_b + sigma * g / sqrt(Dk)), g ~ N(0, I), sigma 0.15.
  3. A random 30% of the tokens are overwritten, in raster order, by
     normalise(direction_nb + 0.02 * g / sqrt(Dk)), nb a random 4-neighbour.
  4. key_i = r_i * direction_i with log-normal r_i (mu 0, s 0.5).
     hidden_i: direction = fixed random projection of direction_i to R^H plus
     N(0, 0.1^2 / H) noise, norm log-normal(0, 0.5), independent of r_i.
     query_i (head j) = sqrt(d_h) * m_j + N(0, I), m_j a fixed unit vector per head.
  5. Video: frame t = frame t-1 + N(0, 0.03^2 / Dk) drift on the directions
     (re-normalised), 20% of the positions of each frame resampled from the mixture.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def round_to_bf16(x) -> np.ndarray:
    """float -> float32 array whose values are bf16-representable (round to nearest even)."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(f.shape)


def bf16_bits(x_f32) -> np.ndarray:
    """uint16 bit patterns of a float32 array that already holds bf16-representable values."""
    f = np.ascontiguousarray(x_f32, dtype=np.float32)
    u = f.view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(f.shape)


@dataclass(frozen=True)
class Config:
    name: str
    grids: int            # crops (image) or frames (video) per sample
    gh: int
    gw: int
    hidden: int
    n_kv: int
    d_h: int
    key_dtype: str        # "f32" | "bf16"
    hidden_dtype: str
    blobs: int            # per sample; 0 = n // 24
    lam: float
    target_reduction: float
    video: bool = False
    batch: int = 1

    @property
    def n(self) -> int:
        return self.grids * self.gh * self.gw

    @property
    def dk(self) -> int:
        return self.n_kv * self.d_h


CONFIGS = {
    # LLaVA-OV-0.5B-shaped single image
    "img_0p5b": Config("img_0p5b", 1, 27, 27, 896, 2, 64, "f32", "f32", 40, 0.30, 0.50),
    # LLaVA-OV-7B-shaped anyres image (10 crops x 729): the headline workload
    "img_7b": Config("img_7b", 10, 27, 27, 3584, 4, 128, "bf16", "bf16", 300, 0.45, 0.71),
    # LLaVA-OV-7B-shaped video, 32 frames x 14x14, batch of 8 independent videos
    "vid_7b": Config("vid_7b", 32, 14, 14, 3584, 4, 128, "bf16", "bf16", 300, 0.45, 0.71,
                     video=True, batch=8),
    # long video stress: 64 frames x 16x16, fp32 keys, bf16 hidden
    "vid_long": Config("vid_long", 64, 16, 16, 3584, 4, 128, "f32", "bf16", 800, 0.50, 0.80,
                       video=True),
    # small shapes for fast CPU/GPU parity sweeps (not in the benchmark list)
    "tiny_f32": Config("tiny_f32", 1, 12, 12, 256, 2, 32, "f32", "f32", 10, 0.30, 0.50),
    "tiny_bf16": Config("tiny_bf16", 2, 14, 14, 512, 2, 64, "bf16", "bf16", 20, 0.45, 0.70),
}

VARLEN_CROPS = (1, 2, 4, 5, 10)      # x 729 tokens
VARLEN_LAMBDAS = (0.5, 0.6, 0.7)


@dataclass
class Sample:
    config: Config
    seed: int
    hidden: np.ndarray      # [n, hidden]  float32 container
    keys: np.ndarray        # [n, n_kv, d_h]; used for EUTI and DBDPC alike
    queries: np.ndarray     # [n, n_q, d_h], n_q == n_kv unless asked otherwise
    lam: float
    extra: dict = field(default_factory=dict)

    @property
    def n(self) -> int:
        return self.hidden.shape[0]


def _cast(x, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    return np.ascontiguousarray(x, dtype=np.float32)


def _unit(x):
    return x / np.linalg.norm(x, axis=-1, keepdims=True)


def _voronoi_blobs(rng, gh, gw, n_sites, n_blobs):
    sites = np.stack([rng.integers(0, gh, n_sites), rng.integers(0, gw, n_sites)], axis=1)
    site_blob = rng.integers(0, n_blobs, n_sites)
    yy, xx = np.meshgrid(np.arange(gh), np.arange(gw), indexing="ij")
    cells = np.stack([yy.ravel(), xx.ravel()], axis=1)
    d2 = ((cells[:, None, :] - sites[None, :, :]) ** 2).sum(-1)
    return site_blob[np.argmin(d2, axis=1)]


def _grid_directions(rng, centres, gh, gw, n_sites, sigma=0.15):
    dk = centres.shape[1]
    blob = _voronoi_blobs(rng, gh, gw, n_sites, centres.shape[0])
    g = rng.standard_normal((gh * gw, dk))
    return _unit(centres[blob] + sigma * g / np.sqrt(dk))


def _near_duplicates(rng, dirs, gh, gw, frac=0.30, sigma=0.02):
    """Overwrite a random `frac` of the grid's tokens by a jittered copy of a random
    4-neighbour, in raster order (so chains of copies can form)."""
    n, dk = dirs.shape
    pick = rng.random(n) < frac
    nb_choice = rng.integers(0, 4, n)
    noise = rng.standard_normal((n, dk)) * (sigma / np.sqrt(dk))
    steps = ((-1, 0), (1, 0), (0, -1), (0, 1))
    for i in np.flatnonzero(pick):
        y, x = divmod(int(i), gw)
        dy, dx = steps[nb_choice[i]]
        yy, xx = y + dy, x + dx
        if not (0 <= yy < gh and 0 <= xx < gw):
            yy, xx = y - dy, x - dx
        src = yy * gw + xx
        v = dirs[src] + noise[i]
        dirs[i] = v / np.linalg.norm(v)
    return dirs


def _directions(rng, cfg: Config, n_blobs: int, grids: int):
    dk = cfg.dk
    centres = _unit(rng.standard_normal((n_blobs, dk)))
    per_grid_sites = max(2, n_blobs // max(grids, 1)) if not cfg.video else max(2, n_blobs // 8)
    out = []
    if not cfg.video:
        for _ in range(grids):
            d = _grid_directions(rng, centres, cfg.gh, cfg.gw, per_grid_sites)
            out.append(_near_duplicates(rng, d, cfg.gh, cfg.gw))
    else:
        m = cfg.gh * cfg.gw
        frame = _near_duplicates(rng, _grid_directions(rng, centres, cfg.gh, cfg.gw, per_grid_sites),
                                 cfg.gh, cfg.gw)
        out.append(frame)
        for _ in range(1, grids):
            frame = _unit(frame + rng.standard_normal((m, dk)) * (0.03 / np.sqrt(dk)))
            fresh = _grid_directions(rng, centres, cfg.gh, cfg.gw, per_grid_sites)
            resample = rng.random(m) < 0.20
            frame = np.where(resample[:, None], fresh, frame)
            out.append(frame)
    return np.concatenate(out, axis=0)


def make_sample(cfg: Config | str, seed: int, *, grids: int | None = None,
                lam: float | None = None, n_q: int | None = None) -> Sample:
    """One image / video of configuration `cfg` from `seed`.  n_q: number of query heads (a
    multiple of the key heads, as in grouped-query models; default: as many as key heads).
    Hidden states and keys do not depend on it."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    grids = cfg.grids if grids is None else grids
    n = grids * cfg.gh * cfg.gw
    n_blobs = cfg.blobs if cfg.blobs > 0 else max(2, n // 24)
    rng = np.random.Generator(np.random.PCG64([seed, grids, cfg.dk, cfg.hidden]))
    dirs = _directions(rng, cfg, n_blobs, grids)

    r = np.exp(rng.normal(0.0, 0.5, n))
    keys = (dirs * r[:, None]).reshape(n, cfg.n_kv, cfg.d_h)

    proj = rng.standard_normal((cfg.dk, cfg.hidden)) / np.sqrt(cfg.dk)
    hdir = dirs @ proj + rng.standard_normal((n, cfg.hidden)) * (0.1 / np.sqrt(cfg.hidden))
    hnorm = np.exp(rng.normal(0.0, 0.5, n))
    hidden = _unit(hdir) * hnorm[:, None]

    n_q = cfg.n_kv if n_q is None else n_q
    assert n_q % cfg.n_kv == 0
    m = _unit(rng.standard_normal((n_q, cfg.d_h)))
    queries = np.sqrt(cfg.d_h) * m[None, :, :] + rng.standard_normal((n, n_q, cfg.d_h))

    return Sample(cfg, seed, _cast(hidden, cfg.hidden_dtype), _cast(keys, cfg.key_dtype),
                  _cast(queries, cfg.key_dtype), cfg.lam if lam is None else lam)


def make_batch(cfg: Config | str, seed: int):
    """`cfg.batch` independent samples (seeds seed*1000 + b)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    return [make_sample(cfg, seed * 1000 + b) for b in range(cfg.batch)]


def make_varlen_batch(seed: int, batch: int = 16, base: str = "img_7b"):
    """Ragged batch: each sample has 729 x {1,2,4,5,10} tokens, one blob per 24 tokens,
    lambda drawn from {0.5, 0.6, 0.7}."""
    cfg = CONFIGS[base]
    cfg = Config(**{**cfg.__dict__, "name": "varlen", "blobs": 0})
    rng = np.random.Generator(np.random.PCG64([seed, 0x7A11]))
    crops = rng.choice(VARLEN_CROPS, batch)
    lams = rng.choice(VARLEN_LAMBDAS, batch)
    return [make_sample(cfg, seed * 1000 + b, grids=int(crops[b]), lam=float(lams[b]))
            for b in range(batch)]

"""Seeded synthetic inputs: pruned-LLM-shaped FP16 weight matrices and FP16 input vectors.

These stand in for the SparseGPT-pruned LLaMA2 / OPT matrices the paper evaluates on
(Section 8, dataset paragraph), which are not available here.  The module holds no part
of the method (no sparse format, no products, no block logic): it only draws random
masks, values and vectors.  Both the CPU oracle's tests and the HIP path's tests and
bench draw their inputs from here.

All randomness comes from numpy's PCG64 seeded by a SeedSequence over
(base seed, config id, shape id, copy id), so every matrix is reproducible on its own.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


@dataclass(frozen=True)
class Config:
    """One synthetic workload: a list of (name, m, n) shapes sharing one mask recipe."""
    cid: int
    name: str
    shapes: Tuple[Tuple[str, int, int], ...]
    density: float                      # rho = 1 - sparsity
    beta: Optional[Tuple[float, float]] # column keep-probability law; None = i.i.d. Bernoulli(rho)
    planted_frac: float = 0.0           # share of nnz inside planted dense blocks
    planted_count: int = 0              # fixed number of planted blocks (config 0); 0 = use planted_frac
    planted_h: Tuple[int, int] = (0, 0) # inclusive height range (rows)
    planted_w: Tuple[int, int] = (0, 0) # inclusive width range (columns)
    rotation_bytes: int = 0             # cold-cache rotation set size the bench aims for


CONFIGS: Tuple[Config, ...] = (
    Config(0, "opt125m-768-s50", (("w", 768, 768),), 0.5, (2.0, 2.0),
           planted_count=8, planted_h=(16, 16), planted_w=(32, 32)),
    Config(1, "llama7b-attn-s50", (("attn", 4096, 4096),), 0.5, (2.0, 2.0),
           planted_frac=0.10, planted_h=(4, 32), planted_w=(8, 64), rotation_bytes=512 << 20),
    Config(2, "llama7b-mlp-s60", (("up", 11008, 4096), ("down", 4096, 11008)), 0.4, (2.0, 2.0),
           planted_frac=0.10, planted_h=(4, 32), planted_w=(8, 64), rotation_bytes=512 << 20),
    Config(3, "llama13b-layer-s70",
           (("q", 5120, 5120), ("k", 5120, 5120), ("v", 5120, 5120), ("o", 5120, 5120),
            ("gate", 13824, 5120), ("up", 13824, 5120), ("down", 5120, 13824)),
           0.3, (0.5, 0.5), planted_frac=0.15, planted_h=(4, 32), planted_w=(8, 64),
           rotation_bytes=1 << 30),
    Config(4, "opt13b-ffn-s80", (("fc1", 20480, 5120), ("fc2", 5120, 20480)), 0.2, None,
           rotation_bytes=1 << 30),
)


def config(cid: int) -> Config:
    return CONFIGS[cid]


def scaled(cfg: Config, div: int) -> Config:
    """Same recipe on shapes divided by `div` (kept a multiple of 8): for fast tests."""
    shapes = tuple((nm, max(8, (m // div) // 8 * 8), max(8, (n // div) // 8 * 8)) for nm, m, n in cfg.shapes)
    return Config(cfg.cid, f"{cfg.name}/div{div}", shapes, cfg.density, cfg.beta, cfg.planted_frac,
                  cfg.planted_count, cfg.planted_h, cfg.planted_w, cfg.rotation_bytes)


def _rng(seed: int, cid: int, shape_id: int, copy: int, stream: int) -> np.random.Generator:
    ss = np.random.SeedSequence([int(seed), int(cid), int(shape_id), int(copy), int(stream)])
    return np.random.Generator(np.random.PCG64(ss))


def _column_keep_probs(rng: np.random.Generator, n: int, beta: Tuple[float, float], target: float) -> np.ndarray:
    """p_j = clip(s * q_j, 0.02, 0.98), q_j ~ Beta(a, b), s chosen so that mean(p) = target."""
    q = rng.beta(beta[0], beta[1], size=n)
    lo, hi = 0.0, 1.0
    while np.mean(np.clip(hi * q, 0.02, 0.98)) < target and hi < 1e6:
        hi *= 2.0
    for _ in range(60):
        mid = 0.5 * (lo + hi)
        if np.mean(np.clip(mid * q, 0.02, 0.98)) < target:
            lo = mid
        else:
            hi = mid
    return np.clip(0.5 * (lo + hi) * q, 0.02, 0.98)


def _planted_blocks(rng: np.random.Generator, cfg: Config, m: int, n: int):
    """Row sets and column sets (both scattered, drawn without replacement) of the planted blocks."""
    blocks = []
    if cfg.planted_count > 0:
        target_cells, count = None, cfg.planted_count
    elif cfg.planted_frac > 0.0:
        target_cells, count = cfg.planted_frac * cfg.density * m * n, None
    else:
        return blocks
    cells = 0
    while (count is not None and len(blocks) < count) or (target_cells is not None and cells < target_cells):
        h = int(rng.integers(cfg.planted_h[0], cfg.planted_h[1] + 1))
        w = int(rng.integers(cfg.planted_w[0], cfg.planted_w[1] + 1))
        h, w = min(h, m), min(w, n)
        rows = np.sort(rng.choice(m, size=h, replace=False))
        cols = np.sort(rng.choice(n, size=w, replace=False))
        blocks.append((rows, cols))
        cells += h * w
    return blocks


def make_mask(cfg: Config, m: int, n: int, seed: int = 0, shape_id: int = 0, copy: int = 0) -> np.ndarray:
    """Boolean keep-mask of shape (m, n) with overall density cfg.density."""
    rng_b = _rng(seed, cfg.cid, shape_id, copy, 1)
    blocks = _planted_blocks(rng_b, cfg, m, n)
    planted = sum(len(r) * len(c) for r, c in blocks)
    total = float(m) * float(n)
    bg = (cfg.density * total - planted) / max(total - planted, 1.0)
    bg = min(max(bg, 0.0), 1.0)
    rng_m = _rng(seed, cfg.cid, shape_id, copy, 2)
    if cfg.beta is None:
        p = np.full(n, bg, dtype=np.float32)
    else:
        p = _column_keep_probs(rng_m, n, cfg.beta, bg).astype(np.float32)
    mask = np.empty((m, n), dtype=bool)
    step = max(1, (1 << 24) // max(n, 1))
    for r0 in range(0, m, step):
        r1 = min(m, r0 + step)
        u = rng_m.random((r1 - r0, n), dtype=np.float32)
        np.less(u, p[None, :], out=mask[r0:r1])
    for rows, cols in blocks:
        mask[np.ix_(rows, cols)] = True
    return mask


def make_matrix(cfg: Config, shape_id: int = 0, seed: int = 0, copy: int = 0) -> np.ndarray:
    """Dense masked FP16 weight matrix (m, n): kept entries ~ N(0, 0.02^2) rounded to FP16, rest +0."""
    _, m, n = cfg.shapes[shape_id]
    mask = make_mask(cfg, m, n, seed, shape_id, copy)
    rng_v = _rng(seed, cfg.cid, shape_id, copy, 3)
    w = np.zeros((m, n), dtype=np.float16)
    step = max(1, (1 << 24) // max(n, 1))
    for r0 in range(0, m, step):
        r1 = min(m, r0 + step)
        v = rng_v.standard_normal((r1 - r0, n), dtype=np.float32)
        v *= np.float32(0.02)
        np.copyto(w[r0:r1], v.astype(np.float16), where=mask[r0:r1])
    return w


def make_vector(n: int, seed: int = 0, cid: int = 0, shape_id: int = 0, copy: int = 0) -> np.ndarray:
    """Input vector x ~ N(0, 1) rounded to FP16."""
    rng_x = _rng(seed, cid, shape_id, copy, 4)
    return rng_x.standard_normal(n, dtype=np.float32).astype(np.float16)


def make_case(cfg: Config, shape_id: int = 0, seed: int = 0, copy: int = 0):
    """(W, x) for one shape of a config."""
    w = make_matrix(cfg, shape_id, seed, copy)
    x = make_vector(w.shape[1], seed, cfg.cid, shape_id, copy)
    return w, x


def small_random(m: int, n: int, density: float, seed: int, scale: float = 0.02):
    """Tiny i.i.d.-masked case for unit tests: (W fp16, x fp16)."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, m, n])))
    mask = rng.random((m, n)) < density
    w = np.where(mask, (rng.standard_normal((m, n)) * scale), 0.0).astype(np.float16)
    x = rng.standard_normal(n).astype(np.float16)
    return w, x

"""Seeded synthetic inputs for the five benchmark configurations.

Serves both the CPU oracle and the HIP path and holds none of the method's
arithmetic: it only draws matrices, vectors and segment lengths.  The shapes
stand in for the LLM-decode layers the paper evaluates on (weights times
activations, KV cache times query), using only the structural values the paper
states: batch sizes 1 to 8, I/O blocks of 4/8/16 KB, 8 KB slots, a 64-request
ragged batch and a 64K-token context (Sections 5, 6.1, 6.2, 6.3).
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    seed: int
    rows: int
    K: int
    B: int
    tile_bytes: int
    slot_bytes: int
    dist: str = "uniform"           # "uniform": U[0,1);  "lognormal": exp(N(0, 2^2))
    n_seg: int = 0                  # > 0: ragged batch of n_seg row segments (then B is 1 per segment)
    zipf_s: float = 0.0


CONFIGS = {
    "cfg1": Config("cfg1", seed=0, rows=128, K=128, B=1, tile_bytes=4096, slot_bytes=4096),
    "cfg2": Config("cfg2", seed=1, rows=1024, K=1024, B=1, tile_bytes=4096, slot_bytes=4096),
    "cfg3": Config("cfg3", seed=2, rows=8192, K=8192, B=1, tile_bytes=8192, slot_bytes=8192),
    "cfg4": Config("cfg4", seed=3, rows=1 << 19, K=128, B=1, tile_bytes=8192, slot_bytes=8192,
                   dist="lognormal", n_seg=64, zipf_s=1.1),
    "cfg5": Config("cfg5", seed=4, rows=32768, K=65536, B=8, tile_bytes=16384, slot_bytes=8192),
    "cfg5_b1": Config("cfg5_b1", seed=4, rows=32768, K=65536, B=1, tile_bytes=16384, slot_bytes=8192),
}


def _draw(shape, dist, gen, device):
    if dist == "uniform":
        return torch.rand(shape, generator=gen, device=device, dtype=torch.float32)
    if dist == "lognormal":
        t = torch.empty(shape, device=device, dtype=torch.float32)
        return t.log_normal_(mean=0.0, std=2.0, generator=gen)
    if dist == "normal":
        return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    raise ValueError(dist)


def zipf_segments(total_rows, n_seg, s, seed, min_rows=16):
    """Segment lengths L_r = max(min_rows, round(c * r**-s)), r = 1..n_seg, with c chosen so the
    lengths sum to total_rows (the remainder goes to the longest segment); the order of the
    segments is shuffled with the seed.  Returns row_off (int64, n_seg + 1)."""
    ranks = np.arange(1, n_seg + 1, dtype=np.float64)
    w = ranks ** (-s)
    lo, hi = 0.0, float(total_rows) * 4
    for _ in range(200):
        c = 0.5 * (lo + hi)
        tot = np.maximum(min_rows, np.rint(c * w)).sum()
        if tot > total_rows:
            hi = c
        else:
            lo = c
    L = np.maximum(min_rows, np.rint(lo * w)).astype(np.int64)
    L[0] += total_rows - L.sum()
    assert L.sum() == total_rows and L.min() >= 1
    order = np.random.default_rng(seed).permutation(n_seg)
    L = L[order]
    row_off = np.zeros(n_seg + 1, dtype=np.int64)
    np.cumsum(L, out=row_off[1:])
    return row_off


@dataclass
class Workload:
    cfg: Config
    M: torch.Tensor                 # [rows, K] fp32
    X: torch.Tensor                 # [B, K] (dense) or [n_seg, K] (ragged) fp32
    row_off: Optional[np.ndarray] = None


def make(cfg, device="cpu", rows=None, K=None, B=None, dist=None):
    """Draw the inputs of a configuration (optionally with overridden sizes) on `device`."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    rows = cfg.rows if rows is None else rows
    K = cfg.K if K is None else K
    B = cfg.B if B is None else B
    dist = cfg.dist if dist is None else dist
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed)
    M = _draw((rows, K), dist, gen, device)
    if cfg.n_seg:
        row_off = zipf_segments(rows, cfg.n_seg, cfg.zipf_s, cfg.seed)
        X = _draw((cfg.n_seg, K), dist, gen, device)
        return Workload(cfg, M, X, row_off)
    X = _draw((B, K), dist, gen, device)
    return Workload(cfg, M, X, None)

"""Benchmark configurations and seeded synthetic inputs.

This module holds no arithmetic of the attention method: only the shapes of the
five workloads and a random-tensor recipe.  Both the CPU oracle's tests and the
HIP path's tests/benchmark draw their inputs from here, so the two sides see
bit-identical Q, K, V.

Recipe (stands in for video latents, whose data and weights are not available):
for every (head, channel) a white-noise image on the token grid is blurred with
a separable Gaussian (sigma in tokens, reflect padding) and normalised to unit
variance -> a spatially smooth field F.  Tensors are white noise plus F, so that
neighbouring tokens are correlated and pooled block scores carry spatial
structure.  Values are rounded to the workload's dtype and returned as float32
(a bf16 value widened to float32 is exact).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
from scipy.ndimage import gaussian_filter1d

SEED_BASE = 12747 * 1000


@dataclass(frozen=True)
class Workload:
    name: str
    index: int            # position in the benchmark's config list (enters the seed)
    heads: int
    head_dim: int
    dtype: str            # "fp32" | "bf16"
    grid_h: int           # latent tokens per frame, rows x cols
    grid_w: int
    tile_h: int           # block = tile_h x tile_w tokens of one frame
    tile_w: int
    q_frames: int         # frames per chunk
    cache_frames: int     # sliding-window capacity in frames, current chunk included
    radius: int           # locality radius in tokens between block centres
    topk: int
    sigma: float          # blur of the smooth field, in tokens
    field_on_v: bool      # Tiny: field on Q,K only with weight 1; others: 0.5*F on Q,K,V
    field_weight: float
    drift_rho: float = 1.0   # F_{c+1} = rho F_c + sqrt(1-rho^2) F'  (1.0 = static scene)
    n_layers: int = 1
    n_chunks: int = 1        # chunks timed once the cache is primed

    @property
    def tokens_per_frame(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def prime_chunks(self) -> int:
        """Chunks appended before the measured one so that the cache is full."""
        return (self.cache_frames - self.q_frames) // self.q_frames


WORKLOADS = {
    "tiny": Workload("tiny", 0, 1, 32, "fp32", 6, 8, 4, 4, 2, 4, 4, 4, 2.0, False, 1.0),
    "small": Workload("small", 1, 12, 128, "bf16", 24, 44, 8, 16, 2, 6, 16, 16, 3.0, True, 0.5),
    "paper": Workload("paper", 2, 12, 128, "bf16", 48, 88, 8, 16, 2, 6, 24, 32, 3.0, True, 0.5, n_layers=30),
    "ultra": Workload("ultra", 3, 12, 128, "bf16", 90, 160, 8, 16, 2, 6, 24, 32, 3.0, True, 0.5),
    "4k": Workload("4k", 4, 12, 128, "bf16", 135, 240, 8, 16, 1, 6, 24, 32, 3.0, True, 0.5,
                   drift_rho=0.9, n_chunks=16),
}


def with_overrides(w: Workload, **kw) -> Workload:
    return replace(w, **kw)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result is float32."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an array that already holds bf16-representable float32 values."""
    return (np.ascontiguousarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def _rng(w: Workload, layer: int, stream: int, chunk: int) -> np.random.Generator:
    seed = SEED_BASE + 100 * w.index + layer
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, stream, chunk])))


def _smooth_field(w: Workload, rng: np.random.Generator) -> np.ndarray:
    """[H][W][heads][d] unit-variance blurred field."""
    g = rng.standard_normal((w.grid_h, w.grid_w, w.heads, w.head_dim), dtype=np.float32)
    g = gaussian_filter1d(g, w.sigma, axis=0, mode="reflect", truncate=3.0)
    g = gaussian_filter1d(g, w.sigma, axis=1, mode="reflect", truncate=3.0)
    g /= g.std(axis=(0, 1), keepdims=True)
    return g.astype(np.float32)


class ChunkStream:
    """Seeded stream of chunks for one layer call: next() -> (q, k, v), each
    float32 [q_frames*H*W][heads][d] holding dtype-rounded values."""

    def __init__(self, w: Workload, layer: int = 0):
        self.w, self.layer, self.chunk = w, layer, 0
        self.field = _smooth_field(w, _rng(w, layer, 0, 0))

    def next(self):
        w = self.w
        if self.chunk > 0 and w.drift_rho < 1.0:
            fresh = _smooth_field(w, _rng(w, self.layer, 0, self.chunk))
            self.field = (w.drift_rho * self.field
                          + np.float32(np.sqrt(1.0 - w.drift_rho ** 2)) * fresh).astype(np.float32)
        rng = _rng(w, self.layer, 1, self.chunk)
        shape = (w.q_frames, w.grid_h, w.grid_w, w.heads, w.head_dim)
        f = (np.float32(w.field_weight) * self.field)[None]
        out = []
        for name in ("q", "k", "v"):
            x = rng.standard_normal(shape, dtype=np.float32)
            if name != "v" or w.field_on_v:
                x += f
            x = x.reshape(w.q_frames * w.tokens_per_frame, w.heads, w.head_dim)
            out.append(round_to_bf16(x) if w.dtype == "bf16" else x)
        self.chunk += 1
        return tuple(out)

"""Seeded synthetic inputs for the GraphKV eviction pass.

This module only draws random tensors and rounds them to the storage type.  It
holds none of the method's arithmetic (no scores, no similarities, no
selection), so both the CPU oracle's tests and the HIP path's tests may use it
without sharing any computation.

The recipes stand in for the key/value/query tensors a Llama-3-8B prefill would
produce (the paper evaluates on LongBench and Needle-in-a-Haystack prompts,
Experiment section / Appendix "Implementation Details"; neither the prompts nor
the weights are available here).  Keys come from a mixture of Gaussians so that
near-duplicate tokens exist, which is the situation the paper's Observation
section describes (important tokens with highly similar keys).

Storage types: "fp32" arrays are numpy float32; "bf16" arrays are numpy uint16
holding the upper 16 bits of the float32 value after round-to-nearest-even.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Tuple

import numpy as np

BASE_SEED = 250900388


@dataclass(frozen=True)
class Config:
    """One workload: shapes follow the paper's problem statement (Methodology,
    "Problem Formulation": per-layer K, V of n x d and a layer budget k_l),
    extended with the head structure of grouped-query attention."""

    name: str
    n_layers: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    n_tokens: int          # N: rows of the key cache, observation window included
    window: int            # w: the last w tokens are the observation window
    pool_kernel: int
    budget: int            # B: retained tokens per head, window included
    n_sources: int         # S: source nodes (Eq. 2's k)
    n_neighbors: int       # m: neighbours per source (Eq. 3)
    rounds: int            # T
    dtype: str             # "fp32" | "bf16"
    n_centroids: int
    centroid_unit_norm: bool
    noise_sigma: float     # per-coordinate sigma (after the unit-norm rescale if any)
    n_outlier_channels: int = 0
    outlier_scale: float = 8.0
    dup_fraction: float = 0.0
    dup_noise: float = 0.01
    decay: float = 1.0
    reselect: int = 1
    pool_mode: int = 0
    key_scale: float = 1.0  # multiplies every key (cosines unchanged)

    @property
    def n_prefix(self) -> int:
        return self.n_tokens - self.window

    def budget_for_layer(self, layer: int) -> int:
        return self.budget


@dataclass(frozen=True)
class PyramidConfig(Config):
    budget_first: int = 4096
    budget_last: int = 512

    def budget_for_layer(self, layer: int) -> int:
        if self.n_layers == 1:
            return self.budget_first
        span = self.budget_first - self.budget_last
        return self.budget_first - (span * layer) // (self.n_layers - 1)


CONFIGS: Dict[str, Config] = {
    # Tiny: fp32, GQA 1:1.  sigma = 0.3/sqrt(d) per coordinate so that the noise
    # vector has norm ~0.3 around a unit-norm centroid (same-cluster cosine ~0.92).
    "c1": Config("c1", 1, 4, 4, 64, 512, 16, 5, 64, 8, 4, 1, "fp32",
                 n_centroids=16, centroid_unit_norm=True, noise_sigma=0.3 / 8.0),
    # Llama-3-8B-shaped single layer.
    "c2": Config("c2", 1, 8, 32, 128, 4096, 32, 7, 512, 32, 8, 1, "bf16",
                 n_centroids=256, centroid_unit_norm=False, noise_sigma=0.3,
                 n_outlier_channels=4),
    # Llama-3-8B full model shape, 32K prompt: the headline workload.
    "c3": Config("c3", 32, 8, 32, 128, 32768, 32, 7, 2048, 64, 32, 2, "bf16",
                 n_centroids=256, centroid_unit_norm=False, noise_sigma=0.3,
                 n_outlier_channels=4),
    # Per-layer (pyramid-shaped) budgets 4096 .. 512.
    "c4": PyramidConfig("c4", 32, 8, 32, 128, 32768, 32, 7, 4096, 64, 32, 3, "bf16",
                        n_centroids=256, centroid_unit_norm=False, noise_sigma=0.3,
                        n_outlier_channels=4, budget_first=4096, budget_last=512),
    # Long context with 10% near-duplicate tokens.
    "c5": Config("c5", 32, 8, 32, 128, 131072, 64, 7, 4096, 128, 128, 3, "bf16",
                 n_centroids=1024, centroid_unit_norm=False, noise_sigma=0.3,
                 n_outlier_channels=4, dup_fraction=0.10, dup_noise=0.01),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a config with some fields replaced (smaller N for tests...)."""
    return replace(cfg, **kw)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bits to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "fp32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """The exact values of a stored tensor, widened to float64."""
    if dtype == "fp32":
        return x.astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    raise ValueError(dtype)


def make_layer(cfg: Config, layer: int = 0, seed: int = BASE_SEED
               ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Draw (Kc, Vc, Qw) for one layer in the config's storage type.

    Kc, Vc: [H_kv, N, d];  Qw: [H_q, w, d].  The per-layer stream is
    ``seed + layer`` so any layer can be regenerated on its own.
    """
    rng = np.random.Generator(np.random.PCG64(seed + layer))
    H, Hq, d, N, w = cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.n_tokens, cfg.window
    G = Hq // H
    K = np.empty((H, N, d), dtype=np.float32)
    for h in range(H):
        cent = rng.standard_normal((cfg.n_centroids, d), dtype=np.float32)
        if cfg.centroid_unit_norm:
            cent /= np.linalg.norm(cent, axis=1, keepdims=True)
        assign = rng.integers(0, cfg.n_centroids, size=N)
        k = cent[assign]
        k += cfg.noise_sigma * rng.standard_normal((N, d), dtype=np.float32)
        if cfg.n_outlier_channels:
            ch = rng.choice(d, size=cfg.n_outlier_channels, replace=False)
            k[:, ch] *= np.float32(cfg.outlier_scale)
        if cfg.dup_fraction > 0.0:
            n_dup = int(cfg.dup_fraction * N)
            dst = rng.choice(N, size=n_dup, replace=False)
            src = (dst + rng.integers(1, N, size=n_dup)) % N   # some other position
            norms = np.linalg.norm(k[src], axis=1, keepdims=True)
            noise = rng.standard_normal((n_dup, d), dtype=np.float32)
            k[dst] = k[src] + np.float32(cfg.dup_noise) * (norms / np.sqrt(np.float32(d))) * noise
        K[h] = k * np.float32(cfg.key_scale)
    V = rng.standard_normal((H, N, d), dtype=np.float32)
    Q = rng.standard_normal((Hq, w, d), dtype=np.float32)
    for q in range(Hq):
        pick = rng.integers(0, N, size=w)
        Q[q] += np.float32(0.5) * K[q // G, pick]
    Ks = to_storage(K, cfg.dtype)
    # queries see the keys as stored, values likewise
    return Ks, to_storage(V, cfg.dtype), to_storage(Q, cfg.dtype)


def random_scores(cfg: Config, seed: int = BASE_SEED) -> np.ndarray:
    """Positive float32 scores [H_kv, P] for tests that feed the propagation
    stage directly (any importance indicator may initialise the nodes: Sparse
    Graph Building section)."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5C0235))
    return rng.random((cfg.n_kv_heads, cfg.n_prefix), dtype=np.float32) + np.float32(1e-3)

"""Seeded node features and layer weights (inputs only; no binarisation here)."""

from __future__ import annotations

from typing import List, Sequence

import numpy as np


def make_features(kind: str, n: int, d: int, density: float, rng: np.random.Generator) -> np.ndarray:
    """fp32 node-feature matrix, row-major (n, d).

    bernoulli: 0/1 bag-of-words with the given density of ones.
    tfidf:     non-negative, ``density`` of the entries non-zero, each lognormal(mu=-3, sigma=1),
               rows then divided by their L1 norm (rows without a non-zero stay zero).
    normal:    dense N(0, 1).
    """
    if kind == "bernoulli":
        x = np.empty((n, d), dtype=np.float32)
        step = max(1, (1 << 24) // max(d, 1))
        for r0 in range(0, n, step):
            r1 = min(n, r0 + step)
            x[r0:r1] = rng.random((r1 - r0, d), dtype=np.float32) < density
        return x
    if kind == "tfidf":
        mask = rng.random((n, d)) < density
        vals = rng.lognormal(mean=-3.0, sigma=1.0, size=(n, d))
        x = np.where(mask, vals, 0.0)
        norm = x.sum(axis=1, keepdims=True)
        norm[norm == 0.0] = 1.0
        return (x / norm).astype(np.float32)
    if kind == "normal":
        return rng.standard_normal((n, d), dtype=np.float32)
    raise ValueError(f"unknown feature kind {kind!r}")


def glorot_uniform(d_in: int, d_out: int, rng: np.random.Generator) -> np.ndarray:
    """fp32 (d_in, d_out) matrix, uniform in +-sqrt(6 / (d_in + d_out))."""
    limit = np.sqrt(6.0 / (d_in + d_out))
    return rng.uniform(-limit, limit, size=(d_in, d_out)).astype(np.float32)


def make_weights(dims: Sequence[int], rng: np.random.Generator) -> List[np.ndarray]:
    return [glorot_uniform(dims[l], dims[l + 1], rng) for l in range(len(dims) - 1)]

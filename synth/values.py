"""Seeded synthetic VALUES: features, weights, perturbation noise, upstream gradients.

Pure random draws with stated distributions; none of the method's arithmetic lives here.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


def normal(seed: int, stream: int, shape, std: float = 1.0) -> np.ndarray:
    """fp32 N(0, std^2)."""
    out = _rng(seed, stream).standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def half_normal(seed: int, stream: int, shape) -> np.ndarray:
    """fp32 |N(0,1)|: non-negative, like a post-ReLU embedding."""
    return np.abs(normal(seed, stream, shape))


def glorot_uniform(seed: int, stream: int, d_in: int, d_out: int) -> np.ndarray:
    """fp32 U(-s, s), s = sqrt(6 / (d_in + d_out)); layout [d_in, d_out] row-major."""
    s = np.sqrt(6.0 / (d_in + d_out))
    return _rng(seed, stream).uniform(-s, s, size=(d_in, d_out)).astype(np.float32)


def permutation(seed: int, stream: int, k: int) -> np.ndarray:
    """A chunk processing order (chunk shuffling, Section 3.4 technique 1)."""
    return _rng(seed, stream).permutation(k).astype(np.int32)


def group_features(seed: int, stream: int, group: np.ndarray, d: int, signal: float) -> np.ndarray:
    """fp32 features of a synthetic classification task: a fixed random +-1 pattern per group, scaled by
    ``signal``, under N(0,1) noise."""
    rng = _rng(seed, stream)
    n_groups = int(group.max()) + 1
    pattern = rng.integers(0, 2, size=(n_groups, d)).astype(np.float32) * 2.0 - 1.0
    return (signal * pattern[group] + rng.standard_normal((group.shape[0], d), dtype=np.float32)).astype(np.float32)


def bernoulli_mask(seed: int, stream: int, n: int, p: float) -> np.ndarray:
    """uint8 [n], 1 with probability p (which vertices carry a training label)."""
    return (_rng(seed, stream).random(n) < p).astype(np.uint8)

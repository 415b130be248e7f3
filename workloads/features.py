"""Seeded dense operands: node features X and GCN weights W (inputs only)."""
from __future__ import annotations

import numpy as np

FEATURE_SEED_OFFSET = 1000


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def gaussian_features(n: int, k: int, seed: int) -> np.ndarray:
    """X ~ N(0, 1), fp32, row-major n x k."""
    return _rng(seed + FEATURE_SEED_OFFSET).standard_normal((n, k), dtype=np.float32)


def integer_features(n: int, k: int, seed: int, lo: int = -8, hi: int = 8) -> np.ndarray:
    """Integer-valued fp32 features, uniform in [lo, hi] (both inclusive)."""
    x = _rng(seed + FEATURE_SEED_OFFSET).integers(lo, hi + 1, size=(n, k))
    return x.astype(np.float32)


def glorot_uniform(fan_in: int, fan_out: int, seed: int) -> np.ndarray:
    """Glorot/Xavier-uniform weight matrix fan_in x fan_out, fp32."""
    a = np.sqrt(6.0 / (fan_in + fan_out))
    w = _rng(seed + FEATURE_SEED_OFFSET + 7 * fan_in + fan_out).uniform(-a, a, size=(fan_in, fan_out))
    return w.astype(np.float32)

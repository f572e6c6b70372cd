"""Seeded synthetic inputs shared by the GPU library's tests and the CPU oracle.

Holds no arithmetic of the method itself: only the data sets the configurations
are stated on.  The Gaussian-mixture set stands in, by shape (32x32x3 = 3072
features, 10 classes, 50 000 samples) for the image data of Sec. 5.1, which is
not available here.
"""
from __future__ import annotations

import numpy as np


def lsq_data(N: int, d: int, seed: int = 0, noise: float = 0.1):
    """x ~ N(0, I), w* ~ N(0, I), y = x.w* + noise * N(0, 1); all stored as fp32."""
    rng = np.random.default_rng([seed, 0x15C])
    X = rng.standard_normal((N, d)).astype(np.float32)
    w_star = rng.standard_normal(d).astype(np.float32)
    y = (X.astype(np.float64) @ w_star.astype(np.float64) + noise * rng.standard_normal(N)).astype(np.float32)
    return X, y, w_star


def mixture_data(N: int, d: int, classes: int = 10, seed: int = 0):
    """Labels uniform on [0, classes); class means ~ N(0, I/d); x = mean + N(0, I), fp32."""
    rng = np.random.default_rng([seed, 0xC1F])
    means = (rng.standard_normal((classes, d)) / np.sqrt(d)).astype(np.float32)
    y = rng.integers(0, classes, size=N).astype(np.int32)
    X = np.empty((N, d), dtype=np.float32)
    step = 4096
    for n0 in range(0, N, step):
        n1 = min(N, n0 + step)
        X[n0:n1] = rng.standard_normal((n1 - n0, d), dtype=np.float32)
        X[n0:n1] += means[y[n0:n1]]
    return X, y

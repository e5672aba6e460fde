"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random tensors; it holds none of the method's arithmetic
(no pruning, quantisation, decomposition or lifting).  Both the GPU tests and the
CPU oracle take their inputs from here so the two sides see identical bits.

The paper measures on pruned W8A8 / FP8 checkpoints of Llama-3.2 and Qwen2.5
(App. E); those weights are not available, so Gaussian tensors with the same
layer shapes stand in: weights ~ N(0, 0.02^2), activations ~ N(0, 1) with a few
whole columns scaled by 20 to mimic outlier channels."""
from __future__ import annotations

import numpy as np

# (name, K, O) of the four linear layers per transformer block ("model mode", App. D.3)
QWEN25_7B = (("qkv", 3584, 4608), ("o", 3584, 3584), ("gate_up", 3584, 37888), ("down", 18944, 3584))
LLAMA3_8B = (("qkv", 4096, 6144), ("o", 4096, 4096), ("gate_up", 4096, 28672), ("down", 14336, 4096))
# pattern sweep: (N, K, O)
PATTERN_SWEEP = ((3, 6144, 4096), (4, 4096, 14336), (5, 5120, 4096))


def n_outlier_columns(K: int) -> int:
    """0.1 % of the channels, at least one."""
    return max(1, int(round(0.001 * K)))


def activations(M: int, K: int, seed: int, n_outliers: int | None = None,
                outlier_scale: float = 20.0) -> np.ndarray:
    """fp32 [M, K] ~ N(0, 1); `n_outliers` distinct columns multiplied by 20."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K), dtype=np.float32)
    if n_outliers is None:
        n_outliers = n_outlier_columns(K)
    if n_outliers > 0:
        cols = rng.choice(K, size=n_outliers, replace=False)
        X[:, cols] *= np.float32(outlier_scale)
    return X


def weights(O: int, K: int, seed: int, sigma: float = 0.02) -> np.ndarray:
    """fp32 [O, K] ~ N(0, sigma^2)."""
    rng = np.random.default_rng(1_000_003 + seed)
    W = rng.standard_normal((O, K), dtype=np.float32)
    W *= np.float32(sigma)
    return W


def config1(seed: int = 0):
    """The small anchor case: M=16, K=512, O=512, 4 outlier columns."""
    return activations(16, 512, seed, n_outliers=4), weights(512, 512, seed)

"""CPU fp64 oracle for the sequence-tiled linear layer.

TEST INFRASTRUCTURE ONLY: the plain definition of what the tiled linear path computes, used to
check the HIP library, never a fallback for it.  Imports nothing from the HIP package.

Paper, section "Sequence Tiling for Reducing Activation Memory Footprint": a linear layer has no
cross-sequence dependency, so running it tile by tile along the sequence gives exactly the untiled
result:

    y[n, m]  = sum_k x[n, k] * W[m, k]
    dx[n, k] = sum_m dy[n, m] * W[m, k]
    dW[m, k] = sum_n dy[n, m] * x[n, k]

numpy float64; np.matmul is the only library primitive.  Pinned by tests/test_linear_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

__all__ = ["forward", "backward"]


def _f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:      # bfloat16 bit patterns: exact widening
        return (np.ascontiguousarray(a).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return np.asarray(a, dtype=np.float64)


def forward(x, W) -> np.ndarray:
    return np.matmul(_f64(x), _f64(W).T)


def backward(x, W, dy):
    """(dx [N, K], dW [M, K])."""
    dyf = _f64(dy)
    return np.matmul(dyf, _f64(W)), np.matmul(dyf.T, _f64(x))

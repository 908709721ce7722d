"""CPU fp64 oracle for the sequence-tiled MLP block (gate / up / down projections with SiLU gating).

TEST INFRASTRUCTURE ONLY.  Plain definition of what the tiled MLP path computes; it exists to
check the HIP library and is never a fallback for it.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import it.  It imports nothing from the HIP package and shares no
code, table or constant with it.

What is computed (paper, subsection "TiledMLP" of "Sequence Tiling for Reducing Activation Memory
Footprint": the MLP of a transformer layer has no cross-sequence dependency, so its forward and
backward are run on tiles of the sequence and the [tile, intermediate] activations exist only per
tile; the result is exactly the untiled MLP.  The paper's example is the Llama-8B MLP layer, i.e.
the gated form below with SiLU, on a [256 000, 4096] bf16 input, tile = hidden size):

    g[t, i] = sum_k x[t, k] * Wg[i, k]            gate projection        Wg [I, H]
    u[t, i] = sum_k x[t, k] * Wu[i, k]            up projection          Wu [I, H]
    a[t, i] = silu(g[t, i]) * u[t, i]             silu(z) = z / (1 + exp(-z))
    y[t, h] = sum_i a[t, i] * Wd[h, i]            down projection        Wd [H, I]

    da = dy Wd                                     [N, I]
    dg = da * u * silu'(g),   silu'(z) = s (1 + z (1 - s)),  s = 1 / (1 + exp(-z))
    du = da * silu(g)
    dx = dg Wg + du Wu                             [N, H]
    dWg = dg^T x,  dWu = du^T x                    [I, H]
    dWd = dy^T a                                   [H, I]

All arithmetic is numpy float64; the only library primitive is np.matmul.  Rows are handled in
blocks of `row_block` rows purely to bound host memory; rows are independent, so the blocking
cannot change what is computed.

Every function here is pinned by tests/test_mlp_oracle_pins.py (closed forms, finite differences,
invariants, torch autograd of the same expression).
"""
from __future__ import annotations

import numpy as np

__all__ = ["bf16_bits_to_f64", "silu", "silu_grad", "forward", "backward", "forward_rows",
           "dx_rows", "dwd_columns", "dwgu_rows"]


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64."""
    bits = np.ascontiguousarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("expected uint16 bfloat16 bit patterns")
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _f64(x: np.ndarray) -> np.ndarray:
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    return np.asarray(x, dtype=np.float64)


def _sigmoid(z: np.ndarray) -> np.ndarray:
    # evaluated on the side where exp cannot overflow
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    e = np.exp(z[~pos])
    out[~pos] = e / (1.0 + e)
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z * _sigmoid(z)


def silu_grad(z: np.ndarray) -> np.ndarray:
    s = _sigmoid(z)
    return s * (1.0 + z * (1.0 - s))


def _blocks(n: int, row_block):
    rb = n if not row_block or row_block <= 0 else int(row_block)
    for lo in range(0, n, max(rb, 1)):
        yield lo, min(n, lo + rb)


def forward(x, Wg, Wu, Wd, row_block=None) -> np.ndarray:
    """y [N, H] (float64)."""
    Wg, Wu, Wd = _f64(Wg), _f64(Wu), _f64(Wd)
    N = x.shape[0]
    y = np.zeros((N, Wd.shape[0]), dtype=np.float64)
    for lo, hi in _blocks(N, row_block):
        xb = _f64(x[lo:hi])
        a = silu(np.matmul(xb, Wg.T)) * np.matmul(xb, Wu.T)
        y[lo:hi] = np.matmul(a, Wd.T)
    return y


def backward(x, Wg, Wu, Wd, dy, row_block=None):
    """(dx [N, H], dWg [I, H], dWu [I, H], dWd [H, I]), all float64."""
    Wg, Wu, Wd = _f64(Wg), _f64(Wu), _f64(Wd)
    N, H = x.shape
    dx = np.zeros((N, H), dtype=np.float64)
    dWg, dWu, dWd = np.zeros_like(Wg), np.zeros_like(Wu), np.zeros_like(Wd)
    for lo, hi in _blocks(N, row_block):
        xb, dyb = _f64(x[lo:hi]), _f64(dy[lo:hi])
        g, u = np.matmul(xb, Wg.T), np.matmul(xb, Wu.T)
        sg = silu(g)
        da = np.matmul(dyb, Wd)
        dg = da * u * silu_grad(g)
        du = da * sg
        dx[lo:hi] = np.matmul(dg, Wg) + np.matmul(du, Wu)
        dWg += np.matmul(dg.T, xb)
        dWu += np.matmul(du.T, xb)
        dWd += np.matmul(dyb.T, sg * u)
    return dx, dWg, dWu, dWd


def forward_rows(x, Wg, Wu, Wd, rows) -> np.ndarray:
    """y for the listed rows only (a row of y needs only that row of x)."""
    rows = np.asarray(rows, dtype=np.int64)
    return forward(x[rows], Wg, Wu, Wd)


def dx_rows(x, Wg, Wu, Wd, dy, rows) -> np.ndarray:
    """dx for the listed rows only (needs only those rows of x and dy)."""
    rows = np.asarray(rows, dtype=np.int64)
    Wg, Wu, Wd = _f64(Wg), _f64(Wu), _f64(Wd)
    xb, dyb = _f64(x[rows]), _f64(dy[rows])
    g, u = np.matmul(xb, Wg.T), np.matmul(xb, Wu.T)
    da = np.matmul(dyb, Wd)
    return np.matmul(da * u * silu_grad(g), Wg) + np.matmul(da * silu(g), Wu)


def dwd_columns(x, Wg, Wu, dy, cols, row_block=None) -> np.ndarray:
    """dWd[:, cols]  ([H, len(cols)]): needs a[:, i] only at the listed intermediate indices i."""
    cols = np.asarray(cols, dtype=np.int64)
    Wg, Wu = _f64(Wg[cols]), _f64(Wu[cols])
    N = x.shape[0]
    out = np.zeros((dy.shape[1], len(cols)), dtype=np.float64)
    for lo, hi in _blocks(N, row_block):
        xb = _f64(x[lo:hi])
        a = silu(np.matmul(xb, Wg.T)) * np.matmul(xb, Wu.T)
        out += np.matmul(_f64(dy[lo:hi]).T, a)
    return out


def dwgu_rows(x, Wg, Wu, Wd, dy, rows, row_block=None):
    """(dWg[rows, :], dWu[rows, :]) for the listed intermediate indices."""
    rows = np.asarray(rows, dtype=np.int64)
    Wgr, Wur, Wdc = _f64(Wg[rows]), _f64(Wu[rows]), _f64(Wd)[:, rows]
    N, H = x.shape
    og = np.zeros((len(rows), H), dtype=np.float64)
    ou = np.zeros((len(rows), H), dtype=np.float64)
    for lo, hi in _blocks(N, row_block):
        xb = _f64(x[lo:hi])
        g, u = np.matmul(xb, Wgr.T), np.matmul(xb, Wur.T)
        da = np.matmul(_f64(dy[lo:hi]), Wdc)
        og += np.matmul((da * u * silu_grad(g)).T, xb)
        ou += np.matmul((da * silu(g)).T, xb)
    return og, ou

"""CPU fp64 oracle for the LM-head projection + cross-entropy loss, forward and backward.

TEST INFRASTRUCTURE ONLY.  This module is the plain definition of what the sequence-tiled
LM-head + loss path computes; it exists to check the HIP library and is never a fallback for
it.  Only tests, the smoke check and the benchmark's cpu_baseline leg may import it.  It
imports nothing from the HIP package and shares no code, table or constant with it.

What is computed (paper, section "Sequence Tiling for Reducing Activation Memory Footprint":
the logits of the LM head are produced and consumed shard by shard along the sequence, forward
and backward of each shard independently; rows have no cross-sequence dependency, so the
result is exactly the unsharded projection + per-token cross-entropy; section "Loss Sharding in
Hugging Face Transformers": labels arrive already shifted to line up with the hidden rows, and
the label value -100 marks a token that is left out of the loss):

    z[i, v]  = sum_k hidden[i, k] * W[v, k]                       (logits, all V columns)
    lse[i]   = max_v z[i, v] + log(sum_v exp(z[i, v] - max_v z[i, v]))
    valid[i] = labels[i] != ignore_index,       M = sum_i valid[i]
    l[i]     = lse[i] - z[i, labels[i]]         for valid rows, 0 otherwise
    L        = (sum_i l[i]) / M                 (mean over the non-ignored tokens)
    dz[i, v] = (g / M) * valid[i] * (exp(z[i, v] - lse[i]) - [v == labels[i]])
    dH[i, k] = sum_v dz[i, v] * W[v, k]
    dW[v, k] = sum_i dz[i, v] * hidden[i, k]

Readings where the paper is silent: the reduction is the mean over non-ignored tokens of the
whole sequence (a sum over all shards divided by the global count, not a mean of shard means);
reduction="sum" leaves out the division, and loss_rows is the unreduced per-token loss;
M == 0 gives L = 0 and zero gradients; a label outside [0, V) that is not ignore_index is an
error; g is a scalar upstream gradient.

All arithmetic is numpy float64.  The only library primitive is np.matmul.  Rows are handled
in blocks of `row_block` rows purely to bound host memory: each block still materialises all V
logits of its rows, and because rows are independent the blocking cannot change what is
computed.  With `ordered=True` the contraction over k is done by an explicit loop in index
order instead of np.matmul, so that every row's bits are independent of the blocking.

Every function here is pinned by tests/test_oracle_pins.py (closed forms, finite differences,
invariants, the library routine torch.nn.functional.cross_entropy under autograd).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "bf16_bits_to_f64",
    "logits",
    "row_lse",
    "forward",
    "backward",
    "dhidden_rows",
    "dw_rows",
]


class LabelRangeError(ValueError):
    """A label is neither ignore_index nor inside [0, V)."""


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float64.

    A bfloat16 is the upper 16 bits of an IEEE binary32, so shifting left by 16 gives the
    binary32 with the same value; binary32 -> binary64 is exact.
    """
    bits = np.ascontiguousarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("expected uint16 bfloat16 bit patterns")
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _as_f64(x: np.ndarray) -> np.ndarray:
    if x.dtype == np.uint16:
        return bf16_bits_to_f64(x)
    return np.asarray(x, dtype=np.float64)


def _contract(a: np.ndarray, b: np.ndarray, ordered: bool) -> np.ndarray:
    """a[r, k] , b[k, c] -> out[r, c] = sum_k a[r, k] b[k, c]  (a and b may be transposed views)."""
    if not ordered:
        return np.matmul(a, b)
    out = np.zeros((a.shape[0], b.shape[1]), dtype=np.float64)
    for k in range(a.shape[1]):
        out += a[:, k : k + 1] * b[k : k + 1, :]
    return out


def logits(hidden: np.ndarray, W: np.ndarray, ordered: bool = False) -> np.ndarray:
    """z = hidden @ W^T with all V columns materialised (the LM-head projection)."""
    return _contract(_as_f64(hidden), _as_f64(W).T, ordered)


def row_lse(z: np.ndarray) -> np.ndarray:
    """log(sum_v exp(z[i, v])) per row, evaluated around the row maximum."""
    m = z.max(axis=1)
    s = np.exp(z - m[:, None]).sum(axis=1)
    return m + np.log(s)


def _check_labels(labels: np.ndarray, V: int, ignore_index: int) -> np.ndarray:
    labels = np.asarray(labels).astype(np.int64)
    valid = labels != ignore_index
    bad = valid & ((labels < 0) | (labels >= V))
    if bad.any():
        raise LabelRangeError(f"label out of range at row {int(np.flatnonzero(bad)[0])}")
    return valid


def _blocks(n: int, row_block: int | None):
    rb = n if not row_block or row_block <= 0 else int(row_block)
    rb = max(rb, 1)
    for lo in range(0, n, rb):
        yield lo, min(n, lo + rb)


def forward(hidden, W, labels, ignore_index: int = -100, row_block: int | None = None,
            ordered: bool = False, reduction: str = "mean") -> dict:
    """Cross-entropy over non-ignored tokens (their mean, or their sum with reduction="sum"),
    plus the per-row pieces; loss_rows is the unreduced loss.

    Returns dict(loss=float, lse=[N] f64, loss_rows=[N] f64 (0 on ignored rows),
    zlabel=[N] f64 (0 on ignored rows), n_valid=int).
    """
    Wd = _as_f64(W)
    N, V = hidden.shape[0], Wd.shape[0]
    valid = _check_labels(labels, V, ignore_index)
    labels = np.asarray(labels).astype(np.int64)
    lse = np.zeros(N, dtype=np.float64)
    zlab = np.zeros(N, dtype=np.float64)
    for lo, hi in _blocks(N, row_block):
        z = _contract(_as_f64(hidden[lo:hi]), Wd.T, ordered)
        lse[lo:hi] = row_lse(z)
        vb = valid[lo:hi]
        idx = np.flatnonzero(vb)
        zlab[lo + idx] = z[idx, labels[lo:hi][idx]]
    loss_rows = np.where(valid, lse - zlab, 0.0)
    M = int(valid.sum())
    # one fixed-order reduction over the whole [N] vector, whatever row_block was
    total = 0.0
    for x in loss_rows.tolist():
        total += x
    if reduction not in ("mean", "sum"):
        raise ValueError("reduction must be 'mean' or 'sum'")
    loss = (total if reduction == "sum" else total / M) if M > 0 else 0.0
    return dict(loss=loss, lse=lse, loss_rows=loss_rows, zlabel=zlab, n_valid=M)


def backward(hidden, W, labels, ignore_index: int = -100, grad_loss: float = 1.0,
             row_block: int | None = None, ordered: bool = False, reduction: str = "mean"):
    """Gradients of the mean (or, with reduction="sum", the summed) loss: returns
    (dHidden [N, H] f64, dW [V, H] f64)."""
    Wd = _as_f64(W)
    N, H = hidden.shape
    V = Wd.shape[0]
    valid = _check_labels(labels, V, ignore_index)
    labels = np.asarray(labels).astype(np.int64)
    M = int(valid.sum())
    dH = np.zeros((N, H), dtype=np.float64)
    dW = np.zeros((V, H), dtype=np.float64)
    if M == 0:
        return dH, dW
    if reduction not in ("mean", "sum"):
        raise ValueError("reduction must be 'mean' or 'sum'")
    coef = float(grad_loss) if reduction == "sum" else float(grad_loss) / M
    for lo, hi in _blocks(N, row_block):
        hb = _as_f64(hidden[lo:hi])
        z = _contract(hb, Wd.T, ordered)
        p = np.exp(z - row_lse(z)[:, None])
        vb = valid[lo:hi]
        idx = np.flatnonzero(vb)
        p[idx, labels[lo:hi][idx]] -= 1.0
        dz = coef * vb[:, None].astype(np.float64) * p
        dH[lo:hi] = _contract(dz, Wd, ordered)
        dW += _contract(dz.T, hb, ordered)
    return dH, dW


def dhidden_rows(hidden, W, labels, rows, n_valid: int, ignore_index: int = -100,
                 grad_loss: float = 1.0):
    """Exact dHidden for the listed rows only (a row's gradient needs only that row's logits).

    `n_valid` is the global count M of non-ignored labels.  Returns (dH_rows [len(rows), H],
    lse_rows, loss_rows) for those rows.
    """
    Wd = _as_f64(W)
    rows = np.asarray(rows, dtype=np.int64)
    labels = np.asarray(labels).astype(np.int64)
    V = Wd.shape[0]
    lab = labels[rows]
    valid = _check_labels(lab, V, ignore_index)
    hb = _as_f64(hidden[rows])
    z = np.matmul(hb, Wd.T)
    lse = row_lse(z)
    p = np.exp(z - lse[:, None])
    idx = np.flatnonzero(valid)
    zl = np.zeros(len(rows))
    zl[idx] = z[idx, lab[idx]]
    p[idx, lab[idx]] -= 1.0
    coef = float(grad_loss) / n_valid if n_valid > 0 else 0.0
    dz = coef * valid[:, None].astype(np.float64) * p
    return np.matmul(dz, Wd), lse, np.where(valid, lse - zl, 0.0)


def dw_rows(hidden, W, labels, lse, vocab_ids, ignore_index: int = -100,
            grad_loss: float = 1.0, row_block: int | None = None):
    """Exact dW rows for the listed vocabulary ids, given lse[N] of ALL rows (from forward()).

    dW[v, :] = (g / M) * sum_i valid[i] * (exp(z[i, v] - lse[i]) - [labels[i] == v]) * hidden[i, :]
    needs z[i, v] only at the listed v, so it costs 2*N*H flops per id.
    """
    vocab_ids = np.asarray(vocab_ids, dtype=np.int64)
    Wd = _as_f64(W[vocab_ids])
    N, H = hidden.shape
    labels = np.asarray(labels).astype(np.int64)
    valid = labels != ignore_index
    M = int(valid.sum())
    out = np.zeros((len(vocab_ids), H), dtype=np.float64)
    if M == 0:
        return out
    coef = float(grad_loss) / M
    for lo, hi in _blocks(N, row_block):
        hb = _as_f64(hidden[lo:hi])
        z = np.matmul(hb, Wd.T)                       # [rows, len(ids)]
        dz = np.exp(z - np.asarray(lse[lo:hi], dtype=np.float64)[:, None])
        dz -= (labels[lo:hi, None] == vocab_ids[None, :])
        dz *= coef * valid[lo:hi, None]
        out += np.matmul(dz.T, hb)
    return out

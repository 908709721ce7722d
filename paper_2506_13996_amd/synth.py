"""Seeded synthetic inputs for the tiled LM-head + cross-entropy path.

This module holds NO arithmetic of the method itself: it only draws hidden states, LM-head
weights and labels of the shapes and value laws of the benchmark workloads, as bfloat16 bit
patterns (uint16) and int32 labels.  Both the HIP path and the CPU oracle consume the very same
bits.  Stand-ins for the Llama-3.1-8B / Qwen-32B LM heads named in the paper's evaluation
section, whose weights are not needed: only the shapes matter to this path.

Generator: numpy Philox, keyed by (seed, stream) with the counter's top word set to the row-block
index, so any block of 1024 rows can be drawn on its own and in parallel, and a tensor's values
do not depend on how many rows are requested after it.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

IGNORE_INDEX = -100
_ROWS_PER_BLOCK = 1024
STREAM_HIDDEN, STREAM_W, STREAM_LABEL, STREAM_IGNORE = 1, 2, 3, 4


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    H: int
    V: int
    tile: int
    label_law: str      # "uniform" | "zipf"
    ignore_law: str     # "iid" | "runs" | "docs"
    ignore_frac: float
    seed: int = 0


WORKLOADS = {
    "tiny": Workload("tiny", 512, 256, 4096, 128, "uniform", "iid", 0.05),
    "llama8b_32k": Workload("llama8b_32k", 32768, 4096, 128256, 2048, "uniform", "iid", 0.02),
    "llama8b_128k": Workload("llama8b_128k", 131072, 4096, 128256, 4096, "uniform", "runs", 0.10),
    "llama8b_512k": Workload("llama8b_512k", 524288, 4096, 128256, 4096, "uniform", "runs", 0.10),
    "qwen32b_256k": Workload("qwen32b_256k", 262144, 5120, 152064, 4096, "zipf", "docs", 0.30),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (finite inputs only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def _rng(seed: int, stream: int, block: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream], counter=[0, 0, 0, block]))


def normal_bf16(rows: int, cols: int, std: float, seed: int, stream: int,
                row_lo: int = 0, threads: int = 8) -> np.ndarray:
    """bf16 bits of N(0, std^2) for rows [row_lo, row_lo + rows) of a [*, cols] tensor."""
    if row_lo % _ROWS_PER_BLOCK:
        raise ValueError("row_lo must be a multiple of the generator's row block")
    out = np.empty((rows, cols), dtype=np.uint16)
    nblk = (rows + _ROWS_PER_BLOCK - 1) // _ROWS_PER_BLOCK

    def fill(b: int) -> None:
        lo = b * _ROWS_PER_BLOCK
        hi = min(rows, lo + _ROWS_PER_BLOCK)
        g = _rng(seed, stream, row_lo // _ROWS_PER_BLOCK + b)
        x = g.standard_normal((_ROWS_PER_BLOCK, cols), dtype=np.float32)[: hi - lo]
        if std != 1.0:
            x *= np.float32(std)
        out[lo:hi] = f32_to_bf16_bits(x)

    if nblk <= 1 or threads <= 1:
        for b in range(nblk):
            fill(b)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(nblk)))
    return out


def _label_ids(N: int, V: int, law: str, seed: int) -> np.ndarray:
    g = _rng(seed, STREAM_LABEL)
    if law == "uniform":
        return g.integers(0, V, size=N, dtype=np.int64).astype(np.int32)
    if law == "zipf":
        # inverse CDF on the exactly normalised weights k^-1.1, k = 1..V; vocabulary id = rank - 1
        w = np.arange(1, V + 1, dtype=np.float64) ** -1.1
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        u = g.random(N)
        return np.minimum(np.searchsorted(cdf, u, side="left"), V - 1).astype(np.int32)
    raise ValueError(law)


def _ignore_mask(N: int, law: str, frac: float, seed: int) -> np.ndarray:
    g = _rng(seed, STREAM_IGNORE)
    mask = np.zeros(N, dtype=bool)
    if frac <= 0.0:
        return mask
    if law == "iid":
        return g.random(N) < frac
    if law == "runs":
        # masked prompt spans: kept gap, then an ignored run of 64..512 tokens (mean 288);
        # gap length uniform with mean 288 * (1 - frac) / frac
        mean_gap = 288.0 * (1.0 - frac) / frac
        glo, ghi = int(mean_gap * 0.5), int(mean_gap * 1.5)
        pos = 0
        while pos < N:
            pos += int(g.integers(glo, ghi + 1))
            run = int(g.integers(64, 513))
            mask[pos : pos + run] = True
            pos += run
        return mask
    if law == "docs":
        # packed documents, length log-uniform in [512, 32768]; the first ceil(frac * len)
        # tokens of each document (its prompt / boundary span) carry no loss
        pos = 0
        while pos < N:
            ln = int(round(math.exp(g.uniform(math.log(512.0), math.log(32768.0)))))
            ln = min(ln, N - pos)
            mask[pos : pos + int(math.ceil(frac * ln))] = True
            pos += ln
        return mask
    raise ValueError(law)


def make_labels(wl: Workload) -> np.ndarray:
    """int32 labels [N], already aligned with the hidden rows, IGNORE_INDEX where masked."""
    ids = _label_ids(wl.N, wl.V, wl.label_law, wl.seed)
    ids[_ignore_mask(wl.N, wl.ignore_law, wl.ignore_frac, wl.seed)] = IGNORE_INDEX
    return ids


def make_hidden(wl: Workload, row_lo: int = 0, rows: int | None = None) -> np.ndarray:
    rows = wl.N - row_lo if rows is None else rows
    return normal_bf16(rows, wl.H, 1.0, wl.seed, STREAM_HIDDEN, row_lo)


def make_weight(wl: Workload) -> np.ndarray:
    return normal_bf16(wl.V, wl.H, 0.02, wl.seed, STREAM_W)


def make_inputs(wl: Workload):
    """(hidden bf16 bits [N, H], W bf16 bits [V, H], labels int32 [N])."""
    return make_hidden(wl), make_weight(wl), make_labels(wl)


def custom(name: str, N: int, H: int, V: int, tile: int, ignore_frac: float = 0.05,
           seed: int = 0, label_law: str = "uniform", ignore_law: str = "iid") -> Workload:
    return Workload(name, N, H, V, tile, label_law, ignore_law, ignore_frac, seed)


# ---------------------------------------------------------------------------------------------
# tiled MLP workloads (the Llama-8B MLP layer of the paper's TiledMLP example)
# ---------------------------------------------------------------------------------------------
STREAM_MLP_X, STREAM_MLP_WG, STREAM_MLP_WU, STREAM_MLP_WD, STREAM_MLP_DY = 11, 12, 13, 14, 15


@dataclass(frozen=True)
class MlpWorkload:
    name: str
    N: int
    H: int
    I: int
    tile: int
    seed: int = 0


MLP_WORKLOADS = {
    "mlp_tiny": MlpWorkload("mlp_tiny", 512, 256, 768, 128),
    # the paper's example: a bf16 [1, 256 000, 4096] input through one Llama-8B MLP layer
    # (intermediate size 14336 from that model's configuration), tile = hidden size -> 63 tiles
    "mlp_llama8b_256k": MlpWorkload("mlp_llama8b_256k", 256000, 4096, 14336, 4096),
}


def make_mlp_inputs(wl: MlpWorkload):
    """bf16 bits of (x [N,H] ~ N(0,1), Wg [I,H], Wu [I,H], Wd [H,I] ~ N(0, 0.02^2), dy [N,H] ~ N(0,1))."""
    x = normal_bf16(wl.N, wl.H, 1.0, wl.seed, STREAM_MLP_X)
    Wg = normal_bf16(wl.I, wl.H, 0.02, wl.seed, STREAM_MLP_WG)
    Wu = normal_bf16(wl.I, wl.H, 0.02, wl.seed, STREAM_MLP_WU)
    Wd = normal_bf16(wl.H, wl.I, 0.02, wl.seed, STREAM_MLP_WD)
    dy = normal_bf16(wl.N, wl.H, 1.0, wl.seed, STREAM_MLP_DY)
    return x, Wg, Wu, Wd, dy

"""CPU oracle for the label handling of a sharded causal loss.

TEST INFRASTRUCTURE ONLY: only tests may import it; it shares nothing with the HIP library.

Paper, section "Loss Sharding in Hugging Face Transformers": the loss at position i compares the
prediction there with the token at position i + 1, so the labels are moved one place to the left
and the last position, which has no next token, gets the ignore value (-100).  If every
sequence-parallel shard does that move on its own piece, the first label of every shard but the
first is lost (its predecessor sits on another rank) and every shard ends in an ignored position;
moving the labels on the whole sequence first and cutting afterwards keeps all of them.

Pinned by tests/test_labels_oracle.py against the example the paper prints
(tests/golden/shift_labels_example.txt) and by counting arguments.
"""
from __future__ import annotations

import numpy as np

IGNORE = -100


def shift_labels(labels, ignore_index: int = IGNORE) -> np.ndarray:
    """out[i] = labels[i + 1] for i < N - 1, out[N - 1] = ignore_index."""
    labels = np.asarray(labels)
    out = np.empty_like(labels)
    for i in range(len(labels)):
        out[i] = labels[i + 1] if i + 1 < len(labels) else ignore_index
    return out


def shard(seq, sp: int) -> list:
    """Cut a sequence whose length is a multiple of sp into sp equal consecutive pieces."""
    seq = np.asarray(seq)
    if len(seq) % sp != 0:
        raise ValueError("sequence length must be a multiple of the sequence-parallel degree")
    n = len(seq) // sp
    return [seq[r * n:(r + 1) * n] for r in range(sp)]


def shard_then_shift(labels, sp: int, ignore_index: int = IGNORE) -> list:
    """What goes wrong: every rank shifts its own piece."""
    return [shift_labels(piece, ignore_index) for piece in shard(labels, sp)]


def shift_then_shard(labels, sp: int, ignore_index: int = IGNORE) -> list:
    """The paper's fix: shift the whole sequence, then cut."""
    return shard(shift_labels(labels, ignore_index), sp)

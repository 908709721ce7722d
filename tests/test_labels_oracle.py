"""Pins of oracle/labels_oracle.py: the example the paper prints and counting arguments."""
import os

import numpy as np

from oracle import labels_oracle as lab

FIXTURE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "shift_labels_example.txt")


def _fixture():
    out = {}
    for line in open(FIXTURE):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, rest = line.split(None, 1)
        out[name] = [[int(t) for t in piece.split()] for piece in rest.split("|")]
    return out


def test_paper_example():
    fx = _fixture()
    labels = fx["labels"][0]
    assert lab.shift_labels(labels).tolist() == fx["shift_labels_unsharded"][0]
    assert [p.tolist() for p in lab.shard_then_shift(labels, 2)] == fx["shift_labels_naive_sp2"]
    assert [p.tolist() for p in lab.shift_then_shard(labels, 2)] == fx["shift_labels_preshifted_sp2"]
    # the naive way drops token id 5 entirely, as the paper says; the fix keeps it
    assert 5 not in np.concatenate(lab.shard_then_shift(labels, 2))
    assert 5 in np.concatenate(lab.shift_then_shard(labels, 2))


def test_counting_arguments():
    g = np.random.default_rng(0)
    for N, sp in ((64, 1), (64, 4), (96, 8), (8, 8)):
        labels = g.integers(0, 1000, N)
        whole = lab.shift_labels(labels)
        # a left shift: everything but the last position is the next label, one ignored position
        assert (whole[:-1] == labels[1:]).all() and whole[-1] == lab.IGNORE
        assert int((whole == lab.IGNORE).sum()) == 1
        fixed = np.concatenate(lab.shift_then_shard(labels, sp))
        naive = np.concatenate(lab.shard_then_shift(labels, sp))
        assert (fixed == whole).all()                                   # cutting loses nothing
        assert int((naive == lab.IGNORE).sum()) == sp                   # one lost label per shard
        kept = naive != lab.IGNORE
        assert (naive[kept] == whole[kept]).all()                       # what survives is unchanged
    assert lab.shift_labels([7], ignore_index=-1).tolist() == [-1]
    assert lab.shift_labels([], ignore_index=-1).tolist() == []

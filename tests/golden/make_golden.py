#!/usr/bin/env python3
"""Writes tests/golden/<workload>.json: expected values for the full-size workloads, computed by
the CPU fp64 oracle ALONE (nothing here touches the HIP library).

The full-size checks need lse of every row (2*N*H*V fp64 flop: minutes to an hour of CPU time), too
slow to recompute inside a GPU test, so they are computed once here from the seeded inputs and
stored: the loss, the number of valid tokens, lse at sampled rows, the sum of lse over all rows and
over the rows with a valid label (the library skips the rows of ignored tokens), and exact dW entries for a sample
of vocabulary ids (always including id 0, V-1, ids at 256-column block edges, the most frequent
labels, ids that never occur as a label) at a sample of hidden columns, plus each sampled dW row's
max |.| for the normaliser.  dHidden rows are cheap and are computed by the test itself.

usage: python tests/golden/make_golden.py llama8b_32k [llama8b_128k ...]
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import tiled_ce_oracle as orc          # noqa: E402
from paper_2506_13996_amd import synth             # noqa: E402


def sample_ids(wl, labels):
    V = wl.V
    g = np.random.default_rng(1234)
    lab = labels[labels != synth.IGNORE_INDEX]
    counts = np.bincount(lab, minlength=V)
    top = np.argsort(-counts, kind="stable")[:4]
    unused = np.flatnonzero(counts == 0)[:3]
    fixed = [0, 1, 127, 128, 255, 256, V // 2, V - 257, V - 256, V - 1]
    rnd = g.integers(0, V, size=8)
    ids = []
    for v in list(fixed) + top.tolist() + unused.tolist() + rnd.tolist():
        if 0 <= v < V and v not in ids:
            ids.append(int(v))
    return np.array(ids, dtype=np.int64), counts


def main():
    for name in sys.argv[1:]:
        wl = synth.WORKLOADS[name]
        t0 = time.time()
        h, W, y = synth.make_inputs(wl)
        print(name, "inputs", round(time.time() - t0, 1), "s", flush=True)
        f = orc.forward(h, W, y, ignore_index=synth.IGNORE_INDEX, row_block=1024)
        print(name, "forward", round(time.time() - t0, 1), "s loss", f["loss"], flush=True)
        ids, counts = sample_ids(wl, y)
        dw = orc.dw_rows(h, W, y, f["lse"], ids, ignore_index=synth.IGNORE_INDEX, row_block=4096)
        g = np.random.default_rng(99)
        cols = np.unique(np.concatenate([np.arange(0, wl.H, wl.H // 32), g.integers(0, wl.H, 32),
                                         [wl.H - 1]]))
        rows = np.unique(np.concatenate([g.integers(0, wl.N, 60), [0, wl.N - 1, wl.tile - 1, wl.tile]]))
        out = {
            "_about": "written by tests/golden/make_golden.py from oracle/tiled_ce_oracle.py only; "
                      "inputs = paper_2506_13996_amd.synth.WORKLOADS[name], seed 0",
            "workload": name, "N": wl.N, "H": wl.H, "V": wl.V,
            "loss": f["loss"], "n_valid": f["n_valid"],
            "lse_sum": float(np.sum(f["lse"])),
            "lse_sum_valid": float(np.sum(f["lse"][y != synth.IGNORE_INDEX])),
            "lse_rows": rows.tolist(), "lse_values": [float(x) for x in f["lse"][rows]],
            "dw_ids": ids.tolist(), "dw_label_counts": [int(counts[v]) for v in ids],
            "dw_cols": cols.tolist(),
            "dw_values": [[float(x) for x in dw[j, cols]] for j in range(len(ids))],
            "dw_row_maxabs": [float(np.abs(dw[j]).max()) for j in range(len(ids))],
            "oracle_seconds": round(time.time() - t0, 1),
        }
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), name + ".json")
        with open(path, "w") as fh:
            json.dump(out, fh, indent=0)
        print(name, "written", path, out["oracle_seconds"], "s", flush=True)


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the sequence-tiled LM-head + cross-entropy path on one MI355X.

One "step" = one fused forward+backward pass (alst_tiled_ce_forward_backward) over the whole
synthetic batch of the workload: every tile's logits GEMM, online log-sum-exp, dZ, dHidden GEMM and
dW GEMM, plus the final loss and dW reductions.  Inputs are resident in HBM before the timed region.
Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this path is measured on one GPU only.

The headline (llama8b_128k unless --workload says otherwise) is timed over exactly --steps steps.
With the default workload the line also carries `others`: the remaining LM-head workloads, the
split entry points on the headline workload and the tiled MLP, each timed the same way over a few
steps (median and min of the per-step times), and `memory_scan`: peak device memory at three
sequence lengths with the O(N) terms taken out.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MI355X_BF16_MFMA_PEAK_TFLOPS = 2500.0      # dense bf16, vendor figure
# Memory-side bytes per launch (calibrated FETCH_SIZE + WRITE_SIZE) are not measurable from inside
# this script: they come from two `rocprofv3 --pmc` runs of this very command, whose summary is
# committed under profiles/.  The line below repeats that file's figures for the headline workload
# and says so in `traffic_source`; for any other workload or tile the field is null.
TRAFFIC_PROFILE = "profiles/bench_llama8b_128k_hbm_traffic.txt"
PROFILED_TRAFFIC_BYTES_PER_LAUNCH = {
    "llama8b_128k": {"logits_gemm": 6.806e9, "dhidden_gemm": 5.916e9, "dw_gemm": 25.573e9},
}
OTHER_STEPS, OTHER_WARMUP = 3, 1


def mfma_sustained(B) -> dict:
    """Sustained TFLOP/s of the bf16 matrix instruction on this device right now, from a loop that
    touches no memory (alst_debug_mfma_rate): context for `roofline.frac`, which stays priced on
    the published peak.  The clock under matrix load follows the power drawn, hence the operand bits."""
    return {"random_operands_tflops": B.alst_debug_mfma_rate(1, 60000),
            "small_integer_operands_tflops": B.alst_debug_mfma_rate(0, 60000),
            "random_operands_16x16x32_tflops": B.alst_debug_mfma_rate(3, 60000),
            "how": "256 workgroups x 4 wavefronts x 60000 x 64 v_mfma_f32_32x32x16_bf16 (or 128 "
                   "v_mfma_f32_16x16x32_bf16), register resident"}


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_threads() -> int:
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1]))
    except Exception:
        return os.cpu_count() or 1


def cpu_baseline(wl, h_bits, W_bits, labels, rows: int) -> dict:
    """The CPU fp64 oracle, as it stands, timed on a bounded sample of the same workload: forward
    and backward of the first `rows` rows against all V columns.  Also quoted: what the whole
    workload would take at the sample's forward rate (3 x the forward time, since forward is one
    of the three contractions) -- an extrapolation, labelled as such."""
    from oracle import tiled_ce_oracle as orc
    hs, ys = h_bits[:rows], labels[:rows]
    t0 = time.perf_counter()
    f = orc.forward(hs, W_bits, ys, ignore_index=-100, row_block=512)
    t1 = time.perf_counter()
    orc.backward(hs, W_bits, ys, ignore_index=-100, row_block=512)
    t2 = time.perf_counter()
    fwd_s, dt = t1 - t0, t2 - t0
    return {"value": rows / dt, "unit": "tokens/s", "cores": cpu_threads(), "kind": "oracle",
            "cpu_model": cpu_model(),
            "sample": f"full fp64 oracle forward + backward on the first {rows} rows of the "
                      f"workload (all V={wl.V} columns), {dt:.1f} s; loss of the sample {f['loss']:.6f}",
            "sample_rows": rows, "sample_forward_s": fwd_s, "sample_forward_backward_s": dt,
            "full_oracle_equivalent_s_extrapolated": 3.0 * fwd_s * wl.N / rows,
            "extrapolation": "3 x the sample's forward time x N / sample rows (not measured)"}


def timed_steps(torch, run_step, steps: int, warmup: int):
    """`warmup` untimed steps, then exactly `steps` steps between two synchronisations; an event
    after every step gives the per-step times without any extra synchronisation.  Returns
    (mean ms per step from the first to the last event, list of per-step ms, wall seconds)."""
    for _ in range(warmup):
        run_step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(steps):
        run_step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    return ev[0].elapsed_time(ev[steps]) / steps, per, wall


def spread(per_step_ms) -> dict:
    return {"median": statistics.median(per_step_ms), "min": min(per_step_ms), "max": max(per_step_ms)}


class CeRun:
    """One LM-head workload resident on the device, ready to step."""

    def __init__(self, torch, B, synth, name: str, tile: int = 0, split: bool = False, flags: int = 0):
        import numpy as np
        self.torch, self.B, self.split, self.flags = torch, B, split, flags
        self.wl = wl = synth.WORKLOADS[name]
        self.tile = tile or wl.tile
        N, H, V = wl.N, wl.H, wl.V
        t0 = time.perf_counter()
        self.h_bits, self.W_bits, self.labels = synth.make_inputs(wl)
        self.t_gen = time.perf_counter() - t0
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        self.base_bytes = torch.cuda.memory_allocated()
        self.hd = torch.from_numpy(self.h_bits.view(np.int16)).cuda().view(torch.bfloat16)
        self.Wd = torch.from_numpy(self.W_bits.view(np.int16)).cuda().view(torch.bfloat16)
        self.yd = torch.from_numpy(self.labels).cuda()
        self.ws = B.alloc_workspace(N, H, V, self.tile, flags)
        self.loss = torch.zeros(1, device="cuda")
        self.lse = torch.zeros(N, device="cuda")
        self.nv = torch.zeros(1, dtype=torch.int64, device="cuda")
        self.dH = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
        self.dW = torch.empty((V, H), dtype=torch.bfloat16, device="cuda")

    def step(self):
        B = self.B
        if self.split:
            B.alst_tiled_ce_forward(self.hd, self.Wd, self.yd, self.tile, -100, loss_out=self.loss,
                                    lse_out=self.lse, n_valid_out=self.nv, workspace=self.ws, flags=self.flags)
            B.alst_tiled_ce_backward(self.hd, self.Wd, self.yd, self.lse, self.tile, -100, 1.0,
                                     dHidden=self.dH, dW=self.dW, workspace=self.ws, flags=self.flags)
        else:
            B.alst_tiled_ce_forward_backward(self.hd, self.Wd, self.yd, self.tile, -100, 1.0,
                                             loss_out=self.loss, lse_out=self.lse, n_valid_out=self.nv,
                                             dHidden=self.dH, dW=self.dW, workspace=self.ws, flags=self.flags)

    def peak_bytes(self) -> int:
        return int(self.torch.cuda.max_memory_allocated() - self.base_bytes)

    def figures(self, ms_per_step: float, prof: dict, prof_steps: int) -> dict:
        """Throughput and utilisation figures of a timed run.  Rows of ignored tokens are skipped
        by the library: the flop it has to execute are 6 M H V for the M valid tokens (8 M H V for
        the split entry points, which compute the logits twice).  Utilisation is priced on those;
        the figure on 6 N H V, which also counts the skipped rows, is given beside it."""
        wl, split = self.wl, self.split
        N, H, V = wl.N, wl.H, wl.V
        M = int(self.nv.item())
        sec = ms_per_step * 1e-3
        tflops_useful = 6.0 * N * H * V / sec / 1e12
        tflops_exec = (8.0 if split else 6.0) * M * H * V / sec / 1e12
        # dominant kernel = the block GEMM kind with the largest summed time.  Over one step the
        # launches of a kind together contract 2 M H V flop (each launch its tile's, or its group
        # of tiles', valid rows), so the mean algorithmic flop per launch are 2 M H V * steps / launches.
        gemm = {k: v for k, v in prof.items() if k.endswith("_gemm") and v[1] > 0}
        dom = max(gemm, key=lambda k: gemm[k][0])
        dom_ms, dom_n = gemm[dom]
        flop_per_launch = (4.0 if split and dom == "logits_gemm" else 2.0) * M * H * V * prof_steps / dom_n
        achieved = flop_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
        known = PROFILED_TRAFFIC_BYTES_PER_LAUNCH.get(wl.name, {}).get(dom)
        profiled = known is not None and self.tile == wl.tile and not split and self.flags == 0
        roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved,
                    "peak": MI355X_BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / MI355X_BF16_MFMA_PEAK_TFLOPS,
                    "traffic": known if profiled else None,
                    "traffic_source": (TRAFFIC_PROFILE + " (rocprofv3 --pmc runs of this command; "
                                       "not measured in this run)") if profiled else None,
                    "avg_launch_ms": dom_ms / dom_n, "launches": dom_n,
                    "flop_per_launch": flop_per_launch,
                    "per_kind_ms_per_step": {k: v[0] / prof_steps for k, v in prof.items() if v[1]},
                    "per_kind_frac": {k: (4.0 if split and k == "logits_gemm" else 2.0) * M * H * V * prof_steps
                                      / (v[0] * 1e-3) / 1e12 / MI355X_BF16_MFMA_PEAK_TFLOPS
                                      for k, v in gemm.items()}}
        return {
            "value": N / sec, "ms_per_step": ms_per_step,
            "tflops_executed": tflops_exec, "executed_flop": "8MHV" if split else "6MHV",
            "mfma_peak_frac": tflops_exec / MI355X_BF16_MFMA_PEAK_TFLOPS,
            "tflops_useful_6NHV": tflops_useful,
            "mfma_peak_frac_counting_skipped_rows": tflops_useful / MI355X_BF16_MFMA_PEAK_TFLOPS,
            "peak_device_bytes": self.peak_bytes(), "would_be_fp32_logits_bytes": 4 * N * V,
            "loss": float(self.loss.item()), "n_valid": M, "roofline": roofline,
        }

    def config(self, graph: bool = False) -> dict:
        wl = self.wl
        return {"workload": wl.name, "N": wl.N, "H": wl.H, "V": wl.V, "tile": self.tile,
                "ignore_frac": wl.ignore_frac,
                "entry": "alst_tiled_ce_forward + alst_tiled_ce_backward" if self.split
                else "alst_tiled_ce_forward_backward",
                "launch": "hip graph replay" if graph else "eager"}


def run_other_ce(torch, B, synth, name: str, split: bool = False, tile: int = 0) -> dict:
    """A workload of the `others` list: OTHER_WARMUP + OTHER_STEPS steps under the per-kernel timer."""
    run = CeRun(torch, B, synth, name, tile=tile, split=split)
    B.alst_profile_enable(True)
    for _ in range(OTHER_WARMUP):
        run.step()
    torch.cuda.synchronize()
    B.alst_profile_read()
    mean_ms, per, _ = timed_steps(torch, run.step, OTHER_STEPS, 0)
    prof = B.alst_profile_read()
    B.alst_profile_enable(False)
    status = B.alst_last_device_status(run.ws)
    out = {"config": run.config(), "steps": OTHER_STEPS, "warmup": OTHER_WARMUP, "unit": "tokens/s",
           "ms_per_step_spread": spread(per), "device_status": status}
    out.update(run.figures(mean_ms, prof, OTHER_STEPS))
    out["workspace_bytes"] = int(run.ws.numel())
    return out


def memory_scan(torch, B, others: dict, headline: dict) -> dict:
    """Peak device memory at three sequence lengths of the Llama-8B shape, tile 4096, with the
    terms that must grow with N taken out: hidden and dHidden (4 N H bytes) and labels, lse and
    the workspace's per-row state (4 + 4 + 12 bytes per row).  What is left is the same at every N."""
    rows = []
    for d in (others.get("llama8b_32k@tile4096"), headline, others.get("llama8b_512k")):
        if not d:
            continue
        c = d["config"]
        N, H = c["N"], c["H"]
        rows.append({"N": N, "tile": c["tile"], "peak_device_bytes": d["peak_device_bytes"],
                     "peak_minus_4NH_minus_12N": d["peak_device_bytes"] - 4 * N * H - 12 * N,
                     "peak_minus_4NH_minus_20N": d["peak_device_bytes"] - 4 * N * H - 20 * N})
    rest = [r["peak_minus_4NH_minus_20N"] for r in rows]
    return {"shape": "H=4096 V=128256 tile=4096", "rows": rows,
            "max_difference_bytes": (max(rest) - min(rest)) if rest else None}


def bench_mlp(args, torch=None, B=None, synth=None, steps=None, warmup=None, with_cpu=True) -> dict:
    """The tiled MLP (next row after the LM-head path): one step = forward + backward over the
    whole synthetic [N, H] input of the workload.  Same JSON shape as the headline benchmark."""
    import numpy as np
    steps = args.steps if steps is None else steps
    warmup = args.warmup if warmup is None else warmup
    wl = synth.MLP_WORKLOADS[args.workload if args.workload.startswith("mlp_") else "mlp_llama8b_256k"]
    tile = (args.tile if args.workload.startswith("mlp_") else 0) or wl.tile
    N, H, I = wl.N, wl.H, wl.I
    t0 = time.perf_counter()
    bits = synth.make_mlp_inputs(wl)
    t_gen = time.perf_counter() - t0
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    base = torch.cuda.memory_allocated()
    x, Wg, Wu, Wd, dy = [torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16) for b in bits]
    ws_f = B.alloc_mlp_workspace(N, H, I, tile, False)
    ws_b = B.alloc_mlp_workspace(N, H, I, tile, True)
    y = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    dx = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    gW = [torch.empty(sh, dtype=torch.bfloat16, device="cuda") for sh in ((I, H), (I, H), (H, I))]

    def step():
        B.alst_tiled_mlp_forward(x, Wg, Wu, Wd, tile, y=y, workspace=ws_f)
        B.alst_tiled_mlp_backward(x, Wg, Wu, Wd, dy, tile, dx=dx, dWg=gW[0], dWu=gW[1], dWd=gW[2],
                                  workspace=ws_b)

    B.alst_profile_enable(True)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    B.alst_profile_read()
    ms_per_step, per, wall = timed_steps(torch, step, steps, 0)
    prof = B.alst_profile_read()
    B.alst_profile_enable(False)
    peak_bytes = torch.cuda.max_memory_allocated() - base
    # forward 3 projections (6 N H I flop); backward recomputes 2, plus dy Wd, the K = 2I product for
    # dx (4 N H I) and three weight gradients: 22 N H I in all, 16 of them in the projection kind
    flop = 22.0 * N * H * I
    tflops = flop / (ms_per_step * 1e-3) / 1e12
    kind_flop = {"mlp_linear_gemm": 16.0 * N * H * I, "mlp_wgrad_gemm": 6.0 * N * H * I}
    gemm = {k: v for k, v in prof.items() if k in kind_flop and v[1] > 0}
    dom = max(gemm, key=lambda k: gemm[k][0])
    dom_ms, dom_n = gemm[dom]
    flop_per_launch = kind_flop[dom] * steps / dom_n
    achieved = flop_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
    out = {
        "metric": "tokens/sec, tiled MLP fwd+bwd, H=%d I=%d" % (H, I),
        "value": N / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": steps,
        "warmup": warmup, "ms_per_step": ms_per_step, "ms_per_step_spread": spread(per),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "N": N, "H": H, "I": I, "tile": tile,
                   "entry": "alst_tiled_mlp_forward + alst_tiled_mlp_backward"},
        "tflops_22NHI": tflops, "mfma_peak_frac": tflops / MI355X_BF16_MFMA_PEAK_TFLOPS,
        "peak_device_bytes": int(peak_bytes),
        "untiled_intermediate_bytes": 2 * 3 * N * I,     # g, u and a of the whole sequence in bf16
        "wall_s_timed_region": wall, "input_gen_s": t_gen,
        "roofline": {"bound": "mfma", "kernel": dom, "achieved": achieved,
                     "peak": MI355X_BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MI355X_BF16_MFMA_PEAK_TFLOPS, "traffic": None,
                     "avg_launch_ms": dom_ms / dom_n, "launches": dom_n,
                     "flop_per_launch": flop_per_launch,
                     "per_kind_ms_per_step": {k: v[0] / steps for k, v in prof.items() if v[1]},
                     "per_kind_frac": {k: kind_flop[k] * steps / (v[0] * 1e-3) / 1e12
                                       / MI355X_BF16_MFMA_PEAK_TFLOPS for k, v in gemm.items()}},
    }
    if with_cpu:
        out["mfma_sustained"] = mfma_sustained(B)
        out["roofline"]["frac_of_sustained_random"] = achieved / out["mfma_sustained"]["random_operands_tflops"]
    if with_cpu and not args.no_cpu_baseline:
        from oracle import tiled_mlp_oracle as morc
        rows = min(args.cpu_rows, N)
        t0 = time.perf_counter()
        morc.forward(bits[0][:rows], bits[1], bits[2], bits[3], row_block=512)
        morc.backward(bits[0][:rows], bits[1], bits[2], bits[3], bits[4][:rows], row_block=512)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": rows / dt, "unit": "tokens/s", "cores": cpu_threads(),
                               "kind": "oracle", "cpu_model": cpu_model(),
                               "sample": f"fp64 MLP oracle forward + backward on the first {rows} rows, {dt:.1f} s"}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="llama8b_128k",
                    help="an LM-head workload (headline metric) or an mlp_* workload (tiled MLP)")
    ap.add_argument("--tile", type=int, default=0, help="override the workload's tile size")
    ap.add_argument("--entry", choices=["fused", "split"], default="fused",
                    help="fused: alst_tiled_ce_forward_backward (the headline); split: "
                         "alst_tiled_ce_forward then alst_tiled_ce_backward, which computes the "
                         "logits twice (8 M H V executed flop)")
    ap.add_argument("--tile-scratch", action="store_true",
                    help="ALST_FLAG_TILE_SCRATCH: dZ scratch of one tile, dW sums updated after every tile")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays of it (the per-kind "
                         "times and the roofline then come from one extra, eagerly launched step)")
    ap.add_argument("--others", choices=["auto", "on", "off"], default="auto",
                    help="also time the other workloads, the split entry points and the tiled MLP "
                         "(auto: with the default workload, entry, tile and launch)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=4096)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device-to-device copy before the timed region, so "
                         "that a rocprofv3 --pmc run holds a kernel of known traffic to scale "
                         "FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures the one-GPU path only; run with --gpus 1 "
              "(the path shards along the sequence; the exchanges between GPUs are not built)",
              file=sys.stderr)
        return 2

    import torch
    from paper_2506_13996_amd import binding as B
    from paper_2506_13996_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.load_library()                       # fails loudly if the HIP library is not built
    if args.workload.startswith("mlp_"):
        print(json.dumps(bench_mlp(args, torch, B, synth)))
        return 0

    split = args.entry == "split"
    flags = B.ALST_FLAG_TILE_SCRATCH if args.tile_scratch else 0
    run = CeRun(torch, B, synth, args.workload, tile=args.tile, split=split, flags=flags)
    wl = run.wl

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        run.step()
    torch.cuda.synchronize()
    run_step, prof_steps, graph = run.step, args.steps, None
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run.step()
        run_step, prof_steps = graph.replay, 1
        graph.replay()
        torch.cuda.synchronize()
    else:
        B.alst_profile_enable(True)
        B.alst_profile_read()
    ms_per_step, per, wall = timed_steps(torch, run_step, args.steps, 0)
    if args.graph:                      # one eager step under the per-kernel timer
        B.alst_profile_enable(True)
        B.alst_profile_read()
        run.step()
        torch.cuda.synchronize()
    prof = B.alst_profile_read()
    B.alst_profile_enable(False)
    status = B.alst_last_device_status(run.ws)

    fig = run.figures(ms_per_step, prof, prof_steps)
    sustained = mfma_sustained(B)
    fig["roofline"]["frac_of_sustained_random"] = fig["roofline"]["achieved"] / sustained["random_operands_tflops"]
    out = {
        "metric": "tokens/sec, tiled LM-head+CE fwd+bwd, H=%d V=%d" % (wl.H, wl.V),
        "value": fig.pop("value"), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": fig.pop("ms_per_step"), "ms_per_step_spread": spread(per),
        "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": run.config(args.graph),
    }
    out["config"]["flags"] = flags
    out.update(fig)
    out.update({"device_status": status, "workspace_bytes": int(run.ws.numel()),
                "wall_s_timed_region": wall, "input_gen_s": run.t_gen, "mfma_sustained": sustained})
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, run.h_bits, run.W_bits, run.labels, min(args.cpu_rows, wl.N))

    default_line = (args.workload == "llama8b_128k" and not split and not args.graph and not args.tile
                    and not flags)
    if args.others == "on" or (args.others == "auto" and default_line):
        run = run_step = graph = None    # frees the headline's tensors before the next workload
        t0 = time.perf_counter()
        others = {}
        others["llama8b_128k@split"] = run_other_ce(torch, B, synth, "llama8b_128k", split=True)
        others["llama8b_32k"] = run_other_ce(torch, B, synth, "llama8b_32k")
        others["llama8b_32k@tile4096"] = run_other_ce(torch, B, synth, "llama8b_32k", tile=4096)
        others["llama8b_512k"] = run_other_ce(torch, B, synth, "llama8b_512k")
        others["qwen32b_256k"] = run_other_ce(torch, B, synth, "qwen32b_256k")
        mlp = bench_mlp(args, torch, B, synth, steps=OTHER_STEPS, warmup=OTHER_WARMUP, with_cpu=False)
        others["mlp_llama8b_256k"] = {k: mlp[k] for k in (
            "config", "steps", "warmup", "value", "unit", "ms_per_step", "ms_per_step_spread", "tflops_22NHI",
            "mfma_peak_frac", "peak_device_bytes", "untiled_intermediate_bytes", "roofline")}
        out["memory_scan"] = memory_scan(torch, B, others, out)
        out["others"] = others
        out["others_wall_s"] = time.perf_counter() - t0
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

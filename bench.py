#!/usr/bin/env python3
"""Benchmark of the sequence-tiled LM-head + cross-entropy path on one MI355X.

One "step" = one fused forward+backward pass (alst_tiled_ce_forward_backward) over the whole
synthetic batch of the workload: every tile's logits GEMM, online log-sum-exp, dZ, dHidden GEMM and
dW GEMM, plus the final loss and dW reductions.  Inputs are resident in HBM before the timed region.
Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this path is measured on one GPU only.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MI355X_BF16_MFMA_PEAK_TFLOPS = 2500.0      # dense bf16, vendor figure
# Memory-side bytes per launch (calibrated FETCH_SIZE + WRITE_SIZE from two `rocprofv3 --pmc` runs of
# this script on llama8b_128k, see profiles/bench_llama8b_128k_hbm_traffic.txt); other workloads: None.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {
    "llama8b_128k": {"logits_gemm": 6.806e9, "dhidden_gemm": 5.843e9, "dw_gemm": 25.259e9},
}


def mfma_sustained(B) -> dict:
    """Sustained TFLOP/s of the bf16 matrix instruction on this device right now, from a loop that
    touches no memory (alst_debug_mfma_rate): context for `roofline.frac`, which stays priced on
    the published peak.  The clock under matrix load follows the power drawn, hence the operand bits."""
    return {"random_operands_tflops": B.alst_debug_mfma_rate(1, 60000),
            "small_integer_operands_tflops": B.alst_debug_mfma_rate(0, 60000),
            "how": "256 workgroups x 4 wavefronts x 60000 x 64 v_mfma_f32_32x32x16_bf16, register resident"}


def cpu_baseline(wl, h_bits, W_bits, labels, rows: int) -> dict:
    """The CPU fp64 oracle, as it stands, timed on a bounded sample of the same workload."""
    import numpy as np
    from oracle import tiled_ce_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    hs, ys = h_bits[:rows], labels[:rows]
    t0 = time.perf_counter()
    f = orc.forward(hs, W_bits, ys, ignore_index=-100, row_block=512)
    orc.backward(hs, W_bits, ys, ignore_index=-100, row_block=512)
    dt = time.perf_counter() - t0
    return {"value": rows / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"full fp64 oracle forward + backward on the first {rows} rows of the "
                      f"workload (all V={wl.V} columns), {dt:.1f} s; loss of the sample {f['loss']:.6f}"}


def bench_mlp(args) -> int:
    """The tiled MLP (next row after the LM-head path): one step = forward + backward over the
    whole synthetic [N, H] input of the workload.  Same JSON shape as the headline benchmark."""
    import numpy as np
    import torch
    from paper_2506_13996_amd import binding as B
    from paper_2506_13996_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.load_library()
    wl = synth.MLP_WORKLOADS[args.workload]
    tile = args.tile or wl.tile
    N, H, I = wl.N, wl.H, wl.I
    t0 = time.perf_counter()
    bits = synth.make_mlp_inputs(wl)
    t_gen = time.perf_counter() - t0
    torch.cuda.reset_peak_memory_stats()
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

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.alst_profile_enable(True)
    B.alst_profile_read()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    prof = B.alst_profile_read()
    B.alst_profile_enable(False)
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    peak_bytes = torch.cuda.max_memory_allocated()
    # forward 3 projections (6 N H I flop); backward recomputes 2, plus dy Wd, the K = 2I product for
    # dx (4 N H I) and three weight gradients: 22 N H I in all, 16 of them in the projection kind
    flop = 22.0 * N * H * I
    tflops = flop / (ms_per_step * 1e-3) / 1e12
    kind_flop = {"mlp_linear_gemm": 16.0 * N * H * I, "mlp_wgrad_gemm": 6.0 * N * H * I}
    gemm = {k: v for k, v in prof.items() if k in kind_flop and v[1] > 0}
    dom = max(gemm, key=lambda k: gemm[k][0])
    dom_ms, dom_n = gemm[dom]
    flop_per_launch = kind_flop[dom] * args.steps / dom_n
    achieved = flop_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
    out = {
        "metric": "tokens/sec, tiled MLP fwd+bwd, H=%d I=%d" % (H, I),
        "value": N / (ms_per_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
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
                     "per_kind_ms_per_step": {k: v[0] / args.steps for k, v in prof.items() if v[1]}},
    }
    out["mfma_sustained"] = mfma_sustained(B)
    out["roofline"]["frac_of_sustained_random"] = achieved / out["mfma_sustained"]["random_operands_tflops"]
    if not args.no_cpu_baseline:
        from oracle import tiled_mlp_oracle as morc
        rows = min(args.cpu_rows, N)
        t0 = time.perf_counter()
        morc.forward(bits[0][:rows], bits[1], bits[2], bits[3], row_block=512)
        morc.backward(bits[0][:rows], bits[1], bits[2], bits[3], bits[4][:rows], row_block=512)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": rows / dt, "unit": "tokens/s", "cores": os.cpu_count() or 1,
                               "kind": "oracle",
                               "sample": f"fp64 MLP oracle forward + backward on the first {rows} rows, {dt:.1f} s"}
    print(json.dumps(out))
    return 0


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
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays of it (the per-kind "
                         "times and the roofline then come from one extra, eagerly launched step)")
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
    if args.workload.startswith("mlp_"):
        return bench_mlp(args)

    import numpy as np
    import torch
    from paper_2506_13996_amd import binding as B
    from paper_2506_13996_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    B.load_library()                       # fails loudly if the HIP library is not built
    wl = synth.WORKLOADS[args.workload]
    tile = args.tile or wl.tile
    N, H, V = wl.N, wl.H, wl.V

    t0 = time.perf_counter()
    h_bits, W_bits, labels = synth.make_inputs(wl)
    t_gen = time.perf_counter() - t0
    torch.cuda.reset_peak_memory_stats()
    hd = torch.from_numpy(h_bits.view(np.int16)).cuda().view(torch.bfloat16)
    Wd = torch.from_numpy(W_bits.view(np.int16)).cuda().view(torch.bfloat16)
    yd = torch.from_numpy(labels).cuda()
    flags = 0
    ws = B.alloc_workspace(N, H, V, tile, flags)
    loss = torch.zeros(1, device="cuda")
    lse = torch.zeros(N, device="cuda")
    nv = torch.zeros(1, dtype=torch.int64, device="cuda")
    dH = torch.empty((N, H), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((V, H), dtype=torch.bfloat16, device="cuda")

    split = args.entry == "split"

    def step():
        if split:
            B.alst_tiled_ce_forward(hd, Wd, yd, tile, -100, loss_out=loss, lse_out=lse, n_valid_out=nv,
                                    workspace=ws, flags=flags)
            B.alst_tiled_ce_backward(hd, Wd, yd, lse, tile, -100, 1.0, dHidden=dH, dW=dW, workspace=ws,
                                     flags=flags)
        else:
            B.alst_tiled_ce_forward_backward(hd, Wd, yd, tile, -100, 1.0, loss_out=loss, lse_out=lse,
                                             n_valid_out=nv, dHidden=dH, dW=dW, workspace=ws, flags=flags)

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    run_step, prof_steps = step, args.steps
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run_step, prof_steps = graph.replay, 1
        graph.replay()
        torch.cuda.synchronize()
    else:
        B.alst_profile_enable(True)
        B.alst_profile_read()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        run_step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if args.graph:                      # one eager step under the per-kernel timer
        B.alst_profile_enable(True)
        B.alst_profile_read()
        step()
        torch.cuda.synchronize()
    prof = B.alst_profile_read()
    B.alst_profile_enable(False)
    status = B.alst_last_device_status(ws)
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    peak_bytes = torch.cuda.max_memory_allocated()

    tokens_per_s = N / (ms_per_step * 1e-3)
    useful_flop = 6.0 * N * H * V
    tflops = useful_flop / (ms_per_step * 1e-3) / 1e12
    # Rows of ignored tokens are skipped by the library: the flop it has to execute are 6 M H V for
    # the M valid tokens.  Utilisation figures are priced on those, not on the skipped rows.
    M = int(nv.item())
    exec_gemms = 8.0 if split else 6.0      # the split entry points compute the logits twice
    tflops_exec = exec_gemms * M * H * V / (ms_per_step * 1e-3) / 1e12

    # dominant kernel = the block GEMM kind with the largest summed time.  Over one step the
    # launches of a kind together contract 2 M H V flop (each launch its tile's, or its group of
    # tiles', valid rows), so the mean algorithmic flop per launch are 2 M H V * steps / launches.
    gemm = {k: v for k, v in prof.items() if k.endswith("_gemm") and v[1] > 0}
    dom = max(gemm, key=lambda k: gemm[k][0])
    dom_ms, dom_n = gemm[dom]
    flop_per_launch = (4.0 if split and dom == "logits_gemm" else 2.0) * M * H * V * prof_steps / dom_n
    achieved = flop_per_launch / (dom_ms / dom_n * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dom, "achieved": achieved,
                "peak": MI355X_BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MI355X_BF16_MFMA_PEAK_TFLOPS,
                "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(wl.name, {}).get(dom) if tile == wl.tile else None,
                "avg_launch_ms": dom_ms / dom_n, "launches": dom_n,
                "flop_per_launch": flop_per_launch,
                "per_kind_ms_per_step": {k: v[0] / prof_steps for k, v in prof.items() if v[1]}}
    sustained = mfma_sustained(B)
    roofline["frac_of_sustained_random"] = achieved / sustained["random_operands_tflops"]

    out = {
        "metric": "tokens/sec, tiled LM-head+CE fwd+bwd, H=%d V=%d" % (H, V),
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "N": N, "H": H, "V": V, "tile": tile,
                   "ignore_frac": wl.ignore_frac,
                   "entry": "alst_tiled_ce_forward + alst_tiled_ce_backward" if split
                   else "alst_tiled_ce_forward_backward",
                   "launch": "hip graph replay" if args.graph else "eager"},
        "tflops_useful_6NHV": tflops,
        "mfma_peak_frac": tflops / MI355X_BF16_MFMA_PEAK_TFLOPS,
        ("tflops_executed_8MHV" if split else "tflops_executed_6MHV"): tflops_exec,
        "mfma_peak_frac_executed": tflops_exec / MI355X_BF16_MFMA_PEAK_TFLOPS,
        "peak_device_bytes": int(peak_bytes),
        "would_be_fp32_logits_bytes": 4 * N * V,
        "loss": float(loss.item()), "n_valid": M, "device_status": status,
        "wall_s_timed_region": wall, "input_gen_s": t_gen,
        "roofline": roofline,
        "mfma_sustained": sustained,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, h_bits, W_bits, labels, args.cpu_rows)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

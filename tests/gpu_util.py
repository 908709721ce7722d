"""Helpers for the GPU parity tests: run the library through its binding, fetch results to numpy."""
from __future__ import annotations

import numpy as np
import torch

from paper_2506_13996_amd import binding as B


def bits_to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bf16_dev_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class Result:
    pass


def run_fused(h_bits, W_bits, labels, tile, ignore_index=-100, grad_loss=1.0, flags=0, dW_init=None,
              dev_inputs=None):
    N, H = h_bits.shape
    V = W_bits.shape[0]
    if dev_inputs is None:
        dev_inputs = (bits_to_dev(h_bits), bits_to_dev(W_bits), torch.from_numpy(labels).cuda())
    hd, Wd, yd = dev_inputs
    ws = B.alloc_workspace(N, H, V, tile, flags)
    loss = torch.full((1,), float("nan"), device="cuda")
    lse = torch.full((N,), float("nan"), device="cuda")
    nv = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    dH = torch.full((N, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    dw_dtype = torch.float32 if flags & B.ALST_FLAG_DW_FP32 else torch.bfloat16
    if dW_init is None:
        dW = torch.full((V, H), float("nan"), dtype=dw_dtype, device="cuda")
    else:
        dW = dW_init.clone()
    B.alst_tiled_ce_forward_backward(hd, Wd, yd, tile, ignore_index, grad_loss, loss_out=loss,
                                     lse_out=lse, n_valid_out=nv, dHidden=dH, dW=dW, workspace=ws,
                                     flags=flags)
    r = Result()
    r.status = B.alst_last_device_status(ws)
    torch.cuda.synchronize()
    r.loss = float(loss.item())
    r.loss_bits = loss.cpu().numpy().view(np.uint32)[0]
    r.lse = lse.cpu().numpy()
    r.n_valid = int(nv.item())
    r.dH_t, r.dW_t = dH, dW
    r.dH = bf16_dev_to_f64(dH)
    r.dW = dW.float().cpu().numpy().astype(np.float64)
    return r


def run_split(h_bits, W_bits, labels, tile, ignore_index=-100, grad_loss=1.0, flags=0):
    N, H = h_bits.shape
    V = W_bits.shape[0]
    hd, Wd, yd = bits_to_dev(h_bits), bits_to_dev(W_bits), torch.from_numpy(labels).cuda()
    ws = B.alloc_workspace(N, H, V, tile, flags)
    loss = torch.full((1,), float("nan"), device="cuda")
    lse = torch.full((N,), float("nan"), device="cuda")
    nv = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    B.alst_tiled_ce_forward(hd, Wd, yd, tile, ignore_index, loss_out=loss, lse_out=lse,
                            n_valid_out=nv, workspace=ws, flags=flags)
    r = Result()
    r.status = B.alst_last_device_status(ws)
    dH = torch.full((N, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    dw_dtype = torch.float32 if flags & B.ALST_FLAG_DW_FP32 else torch.bfloat16
    dW = torch.full((V, H), float("nan"), dtype=dw_dtype, device="cuda")
    B.alst_tiled_ce_backward(hd, Wd, yd, lse, tile, ignore_index, grad_loss, dHidden=dH, dW=dW,
                             workspace=ws, flags=flags)
    r.status_bwd = B.alst_last_device_status(ws)
    torch.cuda.synchronize()
    r.loss = float(loss.item())
    r.loss_bits = loss.cpu().numpy().view(np.uint32)[0]
    r.lse = lse.cpu().numpy()
    r.n_valid = int(nv.item())
    r.dH = bf16_dev_to_f64(dH)
    r.dW = dW.float().cpu().numpy().astype(np.float64)
    return r


def grad_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| (0/0 -> max |got|)."""
    den = np.abs(ref).max()
    num = np.abs(got - ref).max()
    return float(num / den) if den > 0 else float(num)

"""Thin ctypes binding of libalst.so (include/alst.h).  Argument marshalling only.

torch is used for device memory and the current HIP stream; every step of the path runs inside
the library's kernels.  There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libalst.so")

ALST_OK = 0
ALST_ERR_NULL, ALST_ERR_SHAPE, ALST_ERR_ALIGN, ALST_ERR_WORKSPACE = 1, 2, 3, 4
ALST_ERR_LABEL_RANGE, ALST_ERR_HIP, ALST_ERR_UNSUPPORTED, ALST_ERR_NONFINITE = 5, 6, 7, 8
ALST_ERR_NOALLOC_LIMIT = 9
ALST_NOALLOC_SCRATCH_BYTES = 64 << 20
ALST_FLAG_DW_FP32 = 1
ALST_FLAG_DW_ACCUMULATE = 2
ALST_FLAG_REDUCE_SUM = 4
ALST_FLAG_TILE_SCRATCH = 8
ALST_FLAG_FORWARD_ONLY = 16

EXPORTS = (
    "alst_status_string", "alst_version", "alst_tiled_ce_workspace_bytes", "alst_tiled_ce_forward",
    "alst_tiled_ce_backward", "alst_tiled_ce_forward_backward",
    "alst_tiled_ce_forward_backward_noalloc", "alst_last_device_status",
    "alst_shift_labels", "alst_tiled_ce_token_losses",
    "alst_profile_enable", "alst_profile_read", "alst_debug_block_tile", "alst_debug_mfma_rate",
    "alst_tiled_mlp_workspace_bytes", "alst_tiled_mlp_forward", "alst_tiled_mlp_backward",
    "alst_tiled_linear_workspace_bytes", "alst_tiled_linear_forward", "alst_tiled_linear_backward",
)

_lib = None


class AlstError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({alst_status_string(status)})")


def load_library() -> ctypes.CDLL:
    """Load libalst.so (built by `python -m paper_2506_13996_amd.build`); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2506_13996_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    c = ctypes
    vp, i64, i32, u32, f32, sz = c.c_void_p, c.c_int64, c.c_int32, c.c_uint32, c.c_float, c.c_size_t
    lib.alst_status_string.restype = c.c_char_p
    lib.alst_status_string.argtypes = [c.c_int]
    lib.alst_version.restype = c.c_int
    lib.alst_version.argtypes = []
    lib.alst_tiled_ce_workspace_bytes.restype = sz
    lib.alst_tiled_ce_workspace_bytes.argtypes = [i64, i64, i64, i64, u32]
    lib.alst_tiled_ce_forward.restype = c.c_int
    lib.alst_tiled_ce_forward.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, vp, vp, vp, vp, sz, u32, vp]
    lib.alst_tiled_ce_backward.restype = c.c_int
    lib.alst_tiled_ce_backward.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i32, f32, vp, vp, vp, sz, u32, vp]
    lib.alst_tiled_ce_forward_backward.restype = c.c_int
    lib.alst_tiled_ce_forward_backward.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, f32, vp, vp, vp, vp, vp, vp, sz, u32, vp]
    lib.alst_tiled_ce_forward_backward_noalloc.restype = c.c_int
    lib.alst_tiled_ce_forward_backward_noalloc.argtypes = [vp, vp, vp, i64, i64, i64, i64, i32, f32, vp, vp, vp,
                                                           vp, vp, vp, u32, vp]
    lib.alst_last_device_status.restype = c.c_int
    lib.alst_last_device_status.argtypes = [vp, vp]
    lib.alst_shift_labels.restype = c.c_int
    lib.alst_shift_labels.argtypes = [vp, vp, i64, i32, vp]
    lib.alst_tiled_ce_token_losses.restype = c.c_int
    lib.alst_tiled_ce_token_losses.argtypes = [vp, sz, i64, i64, i64, i64, u32, vp, vp]
    lib.alst_tiled_mlp_workspace_bytes.restype = sz
    lib.alst_tiled_mlp_workspace_bytes.argtypes = [i64, i64, i64, i64, c.c_int, u32]
    lib.alst_tiled_mlp_forward.restype = c.c_int
    lib.alst_tiled_mlp_forward.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, sz, u32, vp]
    lib.alst_tiled_mlp_backward.restype = c.c_int
    lib.alst_tiled_mlp_backward.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, vp, vp, vp, vp, vp,
                                            sz, u32, vp]
    lib.alst_tiled_linear_workspace_bytes.restype = sz
    lib.alst_tiled_linear_workspace_bytes.argtypes = [i64, i64, i64, i64, c.c_int, u32]
    lib.alst_tiled_linear_forward.restype = c.c_int
    lib.alst_tiled_linear_forward.argtypes = [vp, vp, i64, i64, i64, i64, vp, vp, sz, u32, vp]
    lib.alst_tiled_linear_backward.restype = c.c_int
    lib.alst_tiled_linear_backward.argtypes = [vp, vp, vp, i64, i64, i64, i64, vp, vp, vp, sz, u32, vp]
    lib.alst_profile_enable.restype = c.c_int
    lib.alst_profile_enable.argtypes = [c.c_int]
    lib.alst_profile_read.restype = c.c_int
    lib.alst_profile_read.argtypes = [c.POINTER(c.c_double), c.POINTER(c.c_int64)]
    lib.alst_debug_mfma_rate.restype = c.c_int
    lib.alst_debug_mfma_rate.argtypes = [c.c_int, c.c_int, c.c_void_p, c.POINTER(c.c_double), c.c_void_p]
    lib.alst_debug_block_tile.restype = c.c_int
    lib.alst_debug_block_tile.argtypes = [c.c_int] * 4 + [c.POINTER(c.c_int)] * 3
    _lib = lib
    return lib


def alst_status_string(status: int) -> str:
    return load_library().alst_status_string(int(status)).decode()


def alst_version() -> int:
    return load_library().alst_version()


def alst_tiled_ce_workspace_bytes(N: int, H: int, V: int, tile: int, flags: int = 0) -> int:
    return int(load_library().alst_tiled_ce_workspace_bytes(N, H, V, tile, flags))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _want(t, name: str, dtype, shape=None, optional: bool = False):
    """The C ABI sees only addresses: a tensor of another dtype, a strided view or a host tensor
    would be reinterpreted silently, so the binding refuses them here."""
    if t is None and optional:
        return
    why = None
    if t is None:
        why = "a tensor is required"
    elif not isinstance(t, torch.Tensor):
        why = f"expected a torch.Tensor, got {type(t).__name__}"
    elif t.dtype != dtype:
        why = f"must be {dtype}, got {t.dtype}"
    elif not t.is_contiguous():
        why = "must be contiguous (dense row-major, no strides)"
    elif shape is not None and tuple(t.shape) != tuple(shape):
        why = f"expected shape {tuple(shape)}, got {tuple(t.shape)}"
    if why:
        raise TypeError(f"{name}: {why}")


def _on_device(**tensors) -> None:
    """Last check of a wrapper, after every dtype / shape / contiguity check has passed: all the
    tensors it hands to the library live on a GPU."""
    for name, t in tensors.items():
        if t is not None and not t.is_cuda:
            raise TypeError(f"{name}: must be a device tensor, got device {t.device}")


def _want_ce_inputs(hidden, W, labels):
    _want(hidden, "hidden", torch.bfloat16)
    _want(W, "W", torch.bfloat16)
    if hidden.dim() != 2 or W.dim() != 2 or hidden.shape[1] != W.shape[1]:
        raise TypeError(f"hidden [N,H] and W [V,H] must share H, got {tuple(hidden.shape)} and {tuple(W.shape)}")
    N, H = hidden.shape
    _want(labels, "labels", torch.int32, (N,))
    return N, H, W.shape[0]


def _want_dw(dW, V: int, H: int, flags: int, name: str = "dW"):
    _want(dW, name, torch.float32 if flags & ALST_FLAG_DW_FP32 else torch.bfloat16, (V, H))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str) -> None:
    if status != ALST_OK:
        raise AlstError(status, where)


def alloc_workspace(N: int, H: int, V: int, tile: int, flags: int = 0, device="cuda") -> torch.Tensor:
    nbytes = alst_tiled_ce_workspace_bytes(N, H, V, tile, flags)
    if nbytes == 0:
        raise AlstError(ALST_ERR_SHAPE, "alst_tiled_ce_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def alst_tiled_ce_forward(hidden, W, labels, tile: int, ignore_index: int = -100, *, loss_out,
                          lse_out=None, n_valid_out=None, workspace, flags: int = 0) -> None:
    """hidden [N,H] bf16, W [V,H] bf16, labels [N] int32 (device tensors); results are written
    into loss_out [1] f32, lse_out [N] f32, n_valid_out [1] int64.  Asynchronous on the current
    stream."""
    N, H, V = _want_ce_inputs(hidden, W, labels)
    _want(loss_out, "loss_out", torch.float32, (1,))
    _want(lse_out, "lse_out", torch.float32, (N,), optional=True)
    _want(n_valid_out, "n_valid_out", torch.int64, (1,), optional=True)
    _want(workspace, "workspace", torch.uint8)
    _on_device(hidden=hidden, W=W, labels=labels, loss_out=loss_out, lse_out=lse_out, n_valid_out=n_valid_out, workspace=workspace)
    st = load_library().alst_tiled_ce_forward(
        _ptr(hidden), _ptr(W), _ptr(labels), N, H, V, tile, ignore_index, _ptr(loss_out),
        _ptr(lse_out), _ptr(n_valid_out), _ptr(workspace), workspace.numel(), flags, _stream())
    _check(st, "alst_tiled_ce_forward")


def alst_tiled_ce_backward(hidden, W, labels, lse, tile: int, ignore_index: int = -100,
                           grad_loss: float = 1.0, *, dHidden, dW, workspace, flags: int = 0) -> None:
    N, H, V = _want_ce_inputs(hidden, W, labels)
    _want(lse, "lse", torch.float32, (N,))
    _want(dHidden, "dHidden", torch.bfloat16, (N, H))
    _want_dw(dW, V, H, flags)
    _want(workspace, "workspace", torch.uint8)
    _on_device(hidden=hidden, W=W, labels=labels, lse=lse, dHidden=dHidden, dW=dW, workspace=workspace)
    st = load_library().alst_tiled_ce_backward(
        _ptr(hidden), _ptr(W), _ptr(labels), _ptr(lse), N, H, V, tile, ignore_index, grad_loss,
        _ptr(dHidden), _ptr(dW), _ptr(workspace), workspace.numel(), flags, _stream())
    _check(st, "alst_tiled_ce_backward")


def alst_tiled_ce_forward_backward(hidden, W, labels, tile: int, ignore_index: int = -100,
                                   grad_loss: float = 1.0, *, loss_out, lse_out=None,
                                   n_valid_out=None, dHidden, dW, workspace, flags: int = 0) -> None:
    N, H, V = _want_ce_inputs(hidden, W, labels)
    _want(loss_out, "loss_out", torch.float32, (1,))
    _want(lse_out, "lse_out", torch.float32, (N,), optional=True)
    _want(n_valid_out, "n_valid_out", torch.int64, (1,), optional=True)
    _want(dHidden, "dHidden", torch.bfloat16, (N, H))
    _want_dw(dW, V, H, flags)
    _want(workspace, "workspace", torch.uint8)
    _on_device(hidden=hidden, W=W, labels=labels, loss_out=loss_out, lse_out=lse_out, n_valid_out=n_valid_out,
               dHidden=dHidden, dW=dW, workspace=workspace)
    st = load_library().alst_tiled_ce_forward_backward(
        _ptr(hidden), _ptr(W), _ptr(labels), N, H, V, tile, ignore_index, grad_loss,
        _ptr(loss_out), _ptr(lse_out), _ptr(n_valid_out), _ptr(dHidden), _ptr(dW),
        _ptr(workspace), workspace.numel(), flags, _stream())
    _check(st, "alst_tiled_ce_forward_backward")


def alst_tiled_ce_forward_backward_noalloc(hidden, W, labels, tile: int, ignore_index: int = -100,
                                           grad_loss: float = 1.0, *, loss_out, lse_out=None,
                                           n_valid_out=None, dHidden, dW, device_status_out=None,
                                           flags: int = 0) -> None:
    """alst_tiled_ce_forward_backward on the library's own static scratch (no workspace argument);
    device_status_out [1] int32 receives the device status word."""
    N, H, V = _want_ce_inputs(hidden, W, labels)
    _want(loss_out, "loss_out", torch.float32, (1,))
    _want(lse_out, "lse_out", torch.float32, (N,), optional=True)
    _want(n_valid_out, "n_valid_out", torch.int64, (1,), optional=True)
    _want(dHidden, "dHidden", torch.bfloat16, (N, H))
    _want_dw(dW, V, H, flags)
    _want(device_status_out, "device_status_out", torch.int32, (1,), optional=True)
    _on_device(hidden=hidden, W=W, labels=labels, loss_out=loss_out, lse_out=lse_out, n_valid_out=n_valid_out,
               dHidden=dHidden, dW=dW, device_status_out=device_status_out)
    st = load_library().alst_tiled_ce_forward_backward_noalloc(
        _ptr(hidden), _ptr(W), _ptr(labels), N, H, V, tile, ignore_index, grad_loss,
        _ptr(loss_out), _ptr(lse_out), _ptr(n_valid_out), _ptr(dHidden), _ptr(dW),
        _ptr(device_status_out), flags, _stream())
    _check(st, "alst_tiled_ce_forward_backward_noalloc")


def alst_last_device_status(workspace) -> int:
    return int(load_library().alst_last_device_status(_ptr(workspace), _stream()))


def alst_shift_labels(labels, shift_labels, ignore_index: int = -100) -> None:
    _want(labels, "labels", torch.int32)
    _want(shift_labels, "shift_labels", torch.int32, tuple(labels.shape))
    _on_device(labels=labels, shift_labels=shift_labels)
    st = load_library().alst_shift_labels(_ptr(labels), _ptr(shift_labels), labels.numel(),
                                          ignore_index, _stream())
    _check(st, "alst_shift_labels")


def alst_tiled_ce_token_losses(workspace, N: int, H: int, V: int, tile: int, token_loss_out,
                               flags: int = 0) -> None:
    _want(workspace, "workspace", torch.uint8)
    _want(token_loss_out, "token_loss_out", torch.float32, (N,))
    _on_device(workspace=workspace, token_loss_out=token_loss_out)
    st = load_library().alst_tiled_ce_token_losses(_ptr(workspace), workspace.numel(), N, H, V, tile,
                                                   flags, _ptr(token_loss_out), _stream())
    _check(st, "alst_tiled_ce_token_losses")


def alst_tiled_mlp_workspace_bytes(N: int, H: int, I: int, tile: int, backward: bool, flags: int = 0) -> int:
    return int(load_library().alst_tiled_mlp_workspace_bytes(N, H, I, tile, 1 if backward else 0, flags))


def alloc_mlp_workspace(N: int, H: int, I: int, tile: int, backward: bool, flags: int = 0,
                        device="cuda") -> torch.Tensor:
    nbytes = alst_tiled_mlp_workspace_bytes(N, H, I, tile, backward, flags)
    if nbytes == 0:
        raise AlstError(ALST_ERR_SHAPE, "alst_tiled_mlp_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _want_mlp_inputs(x, Wg, Wu, Wd):
    _want(x, "x", torch.bfloat16)
    if x.dim() != 2 or Wg.dim() != 2:
        raise TypeError("x must be [N,H] and Wg [I,H]")
    N, H = x.shape
    I = Wg.shape[0]
    _want(Wg, "Wg", torch.bfloat16, (I, H))
    _want(Wu, "Wu", torch.bfloat16, (I, H))
    _want(Wd, "Wd", torch.bfloat16, (H, I))
    return N, H, I


def alst_tiled_mlp_forward(x, Wg, Wu, Wd, tile: int, *, y, workspace, flags: int = 0) -> None:
    """x [N,H], Wg/Wu [I,H], Wd [H,I] bf16 device tensors; y [N,H] bf16 is overwritten."""
    N, H, I = _want_mlp_inputs(x, Wg, Wu, Wd)
    _want(y, "y", torch.bfloat16, (N, H))
    _want(workspace, "workspace", torch.uint8)
    _on_device(x=x, Wg=Wg, Wu=Wu, Wd=Wd, y=y, workspace=workspace)
    st = load_library().alst_tiled_mlp_forward(_ptr(x), _ptr(Wg), _ptr(Wu), _ptr(Wd), N, H, I, tile,
                                               _ptr(y), _ptr(workspace), workspace.numel(), flags,
                                               _stream())
    _check(st, "alst_tiled_mlp_forward")


def alst_tiled_mlp_backward(x, Wg, Wu, Wd, dy, tile: int, *, dx, dWg, dWu, dWd, workspace,
                            flags: int = 0) -> None:
    N, H, I = _want_mlp_inputs(x, Wg, Wu, Wd)
    _want(dy, "dy", torch.bfloat16, (N, H))
    _want(dx, "dx", torch.bfloat16, (N, H))
    _want_dw(dWg, I, H, flags, "dWg")
    _want_dw(dWu, I, H, flags, "dWu")
    _want_dw(dWd, H, I, flags, "dWd")
    _want(workspace, "workspace", torch.uint8)
    _on_device(x=x, Wg=Wg, Wu=Wu, Wd=Wd, dy=dy, dx=dx, dWg=dWg, dWu=dWu, dWd=dWd, workspace=workspace)
    st = load_library().alst_tiled_mlp_backward(_ptr(x), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(dy), N, H,
                                                I, tile, _ptr(dx), _ptr(dWg), _ptr(dWu), _ptr(dWd),
                                                _ptr(workspace), workspace.numel(), flags, _stream())
    _check(st, "alst_tiled_mlp_backward")


def alst_tiled_linear_workspace_bytes(N: int, K: int, M: int, tile: int, backward: bool, flags: int = 0) -> int:
    return int(load_library().alst_tiled_linear_workspace_bytes(N, K, M, tile, 1 if backward else 0, flags))


def alst_tiled_linear_forward(x, W, tile: int, *, y) -> None:
    """y [N,M] = x [N,K] W[M,K]^T (bf16 device tensors)."""
    _want(x, "x", torch.bfloat16)
    N, K = x.shape
    M = W.shape[0]
    _want(W, "W", torch.bfloat16, (M, K))
    _want(y, "y", torch.bfloat16, (N, M))
    _on_device(x=x, W=W, y=y)
    st = load_library().alst_tiled_linear_forward(_ptr(x), _ptr(W), N, K, M, tile, _ptr(y), None, 0, 0,
                                                  _stream())
    _check(st, "alst_tiled_linear_forward")


def alst_tiled_linear_backward(x, W, dy, tile: int, *, dx, dW, workspace, flags: int = 0) -> None:
    _want(x, "x", torch.bfloat16)
    N, K = x.shape
    M = W.shape[0]
    _want(W, "W", torch.bfloat16, (M, K))
    _want(dy, "dy", torch.bfloat16, (N, M))
    _want(dx, "dx", torch.bfloat16, (N, K))
    _want_dw(dW, M, K, flags)
    _want(workspace, "workspace", torch.uint8, optional=True)
    _on_device(x=x, W=W, dy=dy, dx=dx, dW=dW, workspace=workspace)
    st = load_library().alst_tiled_linear_backward(_ptr(x), _ptr(W), _ptr(dy), N, K, M, tile, _ptr(dx),
                                                   _ptr(dW), _ptr(workspace),
                                                   0 if workspace is None else workspace.numel(),
                                                   flags, _stream())
    _check(st, "alst_tiled_linear_backward")


PROFILE_KINDS = ("logits_gemm", "dhidden_gemm", "dw_gemm", "tile_small_kernels",
                 "mlp_linear_gemm", "mlp_wgrad_gemm", "mlp_small_kernels", "unused")


def alst_profile_enable(on: bool) -> None:
    _check(load_library().alst_profile_enable(1 if on else 0), "alst_profile_enable")


def alst_profile_read() -> dict:
    """{kind: (total_ms, spans)} for the spans recorded since the last read."""
    ms = (ctypes.c_double * 8)()
    n = (ctypes.c_int64 * 8)()
    _check(load_library().alst_profile_read(ms, n), "alst_profile_read")
    return {k: (ms[i], int(n[i])) for i, k in enumerate(PROFILE_KINDS)}


def alst_debug_block_tile(tiles_r: int, tiles_c: int, parts: int, bid: int):
    """(workgroups of the launch, part, tr, tc) for workgroup `bid`; part = -1 for a padding one."""
    part, tr, tc = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    n = load_library().alst_debug_block_tile(tiles_r, tiles_c, parts, bid, ctypes.byref(part),
                                             ctypes.byref(tr), ctypes.byref(tc))
    if n < 0:
        raise AlstError(-n, "alst_debug_block_tile")
    return n, part.value, tr.value, tc.value


def alst_debug_mfma_rate(data: int, iters: int = 100000) -> float:
    """Sustained TFLOP/s of a bf16 matrix instruction on the current device (no memory traffic).
    data bit 0: small-integer (0) or random (1) operands; bit 1: 32x32x16 (0) or 16x16x32 (1) form."""
    scratch = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    out = ctypes.c_double()
    _check(load_library().alst_debug_mfma_rate(data, iters, _ptr(scratch), ctypes.byref(out), _stream()),
           "alst_debug_mfma_rate")
    return out.value

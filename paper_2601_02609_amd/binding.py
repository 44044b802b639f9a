"""ctypes binding of the libcce C ABI (include/cce.h).  Argument marshalling only.

PyTorch is used for device memory and the current HIP stream; every step of the
computation runs in the library's kernels.  There is no fallback: if the shared
library has not been built the import of the library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

from . import build as _build

CCE_OK = 0
CCE_ERR_INVALID = -1
CCE_ERR_UNSUPPORTED = -2
CCE_ERR_HIP = -3
CCE_ERR_TOO_LARGE = -4
STATIC_SCRATCH_BYTES = 16 << 20
CCE_STATUS_BAD_LABEL = 1

EXPORTED_SYMBOLS = [
    "cce_version", "cce_strerror", "cce_last_hip_error", "cce_workspace_bytes",
    "cce_materialised_logit_bytes", "cce_forward", "cce_backward", "cce_read_status",
    "cce_forward_ex", "cce_backward_ex", "cce_forward_static",
    "cce_profile_begin", "cce_profile_end", "cce_set_backward_tiling",
    "cce_get_backward_tiling", "cce_get_backward_gemm_tile", "cce_set_backward_gemm_tile",
    "cce_set_backward_accumulator", "cce_get_backward_accumulator",
    # include/cce_aux.h
    "cce_rmsnorm_workspace_bytes", "cce_rmsnorm_forward", "cce_rmsnorm_backward",
    "cce_rmsnorm_residual_forward", "cce_rmsnorm_residual_backward",
    "cce_sumsq_workspace_bytes", "cce_grad_sumsq", "cce_clip_coef", "cce_adamw_step",
    "cce_mfma_probe", "cce_mfma_probe_data", "cce_device_info",
    # include/cce_shard.h
    "cce_shard_forward", "cce_shard_merge", "cce_shard_backward",
    # include/cce_compact.h
    "cce_compact_workspace_bytes", "cce_forward_compact", "cce_backward_compact",
    "cce_forward_compact_ex", "cce_backward_compact_ex",
    "cce_get_row_skipping", "cce_set_row_skipping", "cce_get_compact_tiling",
    # include/cce_fp8.h
    "cce_fp8_scale_bytes", "cce_quantize_e4m3", "cce_fp8_forward", "cce_fp8_backward",
]
KERNEL_FAMILIES = ["lse_partial_kernel", "grad_tile_kernel", "grad_gemm_kernel"]

_lib = None


class CCEError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().cce_strerror(code).decode()
        hip = lib().cce_last_hip_error()
        super().__init__(f"{where}: {msg} (code {code}, hip error {hip})")


def lib() -> ctypes.CDLL:
    """Load libcce.so (built in-tree by paper_2601_02609_amd.build); raise if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB_PATH
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build it first (python -m paper_2601_02609_amd.build). "
            "There is no CPU or PyTorch fallback for this library.")
    L = ctypes.CDLL(path)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    L.cce_version.restype = ctypes.c_char_p
    L.cce_version.argtypes = []
    L.cce_strerror.restype = ctypes.c_char_p
    L.cce_strerror.argtypes = [ctypes.c_int]
    L.cce_last_hip_error.restype = ctypes.c_int
    L.cce_last_hip_error.argtypes = []
    L.cce_workspace_bytes.restype = sz
    L.cce_workspace_bytes.argtypes = [i64, i64, i64]
    L.cce_materialised_logit_bytes.restype = sz
    L.cce_materialised_logit_bytes.argtypes = [i64, i64]
    L.cce_forward.restype = ctypes.c_int
    L.cce_forward.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]
    L.cce_backward.restype = ctypes.c_int
    L.cce_backward.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, ctypes.c_int, vp, sz, vp]
    f32 = ctypes.c_float
    L.cce_forward_ex.restype = ctypes.c_int
    L.cce_forward_ex.argtypes = [vp, vp, vp, i64, i64, i64, i32, f32, f32, vp, vp, vp, vp, sz, vp]
    L.cce_backward_ex.restype = ctypes.c_int
    L.cce_backward_ex.argtypes = [vp, vp, vp, vp, vp, f32, i64, i64, i64, i32, f32, f32, vp, vp, ctypes.c_int, vp, sz, vp]
    L.cce_forward_static.restype = ctypes.c_int
    L.cce_forward_static.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, vp]
    L.cce_read_status.restype = ctypes.c_int
    L.cce_read_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32)]
    L.cce_profile_begin.restype = ctypes.c_int
    L.cce_profile_begin.argtypes = []
    L.cce_profile_end.restype = ctypes.c_int
    L.cce_profile_end.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    L.cce_set_backward_tiling.restype = ctypes.c_int
    L.cce_set_backward_tiling.argtypes = [ctypes.c_int, ctypes.c_int]
    L.cce_get_backward_tiling.restype = ctypes.c_int
    L.cce_get_backward_tiling.argtypes = [i64, i64, i64] + [ctypes.POINTER(ctypes.c_int)] * 2
    L.cce_set_backward_accumulator.restype = ctypes.c_int
    L.cce_set_backward_accumulator.argtypes = [ctypes.c_int]
    L.cce_get_backward_accumulator.restype = ctypes.c_int
    L.cce_get_backward_accumulator.argtypes = [i64, i64, i64, ctypes.POINTER(ctypes.c_int)]
    L.cce_set_backward_gemm_tile.restype = ctypes.c_int
    L.cce_set_backward_gemm_tile.argtypes = [ctypes.c_int]
    L.cce_get_backward_gemm_tile.restype = ctypes.c_int
    L.cce_get_backward_gemm_tile.argtypes = [i64, i64, i64] + [ctypes.POINTER(ctypes.c_int)] * 2
    L.cce_rmsnorm_workspace_bytes.restype = sz
    L.cce_rmsnorm_workspace_bytes.argtypes = [i64, i64]
    L.cce_rmsnorm_forward.restype = ctypes.c_int
    L.cce_rmsnorm_forward.argtypes = [vp, vp, i64, i64, f32, vp, vp, vp]
    L.cce_rmsnorm_backward.restype = ctypes.c_int
    L.cce_rmsnorm_backward.argtypes = [vp, vp, vp, vp, i64, i64, vp, vp, ctypes.c_int, vp, sz, vp]
    L.cce_rmsnorm_residual_forward.restype = ctypes.c_int
    L.cce_rmsnorm_residual_forward.argtypes = [vp, vp, vp, i64, i64, f32, vp, vp, vp]
    L.cce_rmsnorm_residual_backward.restype = ctypes.c_int
    L.cce_rmsnorm_residual_backward.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, ctypes.c_int, vp, sz, vp]
    L.cce_sumsq_workspace_bytes.restype = sz
    L.cce_sumsq_workspace_bytes.argtypes = []
    L.cce_grad_sumsq.restype = ctypes.c_int
    L.cce_grad_sumsq.argtypes = [vp, i64, vp, ctypes.c_int, vp, sz, vp]
    L.cce_clip_coef.restype = ctypes.c_int
    L.cce_clip_coef.argtypes = [vp, f32, f32, vp, vp]
    L.cce_adamw_step.restype = ctypes.c_int
    L.cce_adamw_step.argtypes = [vp, vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i64, vp, vp]
    L.cce_device_info.restype = ctypes.c_int
    L.cce_device_info.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    L.cce_mfma_probe.restype = ctypes.c_int
    L.cce_mfma_probe.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp]
    L.cce_mfma_probe_data.restype = ctypes.c_int
    L.cce_mfma_probe_data.argtypes = [ctypes.c_int, ctypes.c_int, vp, vp, vp]
    L.cce_shard_forward.restype = ctypes.c_int
    L.cce_shard_forward.argtypes = [vp, vp, vp, i64, i64, i64, i64, ctypes.c_int, vp, vp, sz, vp]
    L.cce_shard_merge.restype = ctypes.c_int
    L.cce_shard_merge.argtypes = [vp, ctypes.c_int, vp, i64, i64, i32, f32, f32, vp, vp, vp, vp, vp]
    L.cce_shard_backward.restype = ctypes.c_int
    L.cce_shard_backward.argtypes = [vp, vp, vp, vp, vp, f32, i64, i64, i64, i64, i64, i32, f32, f32,
                                     vp, vp, ctypes.c_int, vp, sz, vp]
    L.cce_get_row_skipping.restype = ctypes.c_int
    L.cce_get_row_skipping.argtypes = [i64, i64, i64, i64, ctypes.POINTER(ctypes.c_int)]
    L.cce_get_compact_tiling.restype = ctypes.c_int
    L.cce_get_compact_tiling.argtypes = [i64, i64, i64, i64] + [ctypes.POINTER(ctypes.c_int)] * 2
    L.cce_set_row_skipping.restype = ctypes.c_int
    L.cce_set_row_skipping.argtypes = [ctypes.c_int]
    L.cce_compact_workspace_bytes.restype = sz
    L.cce_compact_workspace_bytes.argtypes = [i64, i64, i64, i64]
    L.cce_forward_compact.restype = ctypes.c_int
    L.cce_forward_compact.argtypes = [vp, vp, vp, i64, i64, i64, i32, i64, vp, vp, vp, sz, vp]
    L.cce_backward_compact.restype = ctypes.c_int
    L.cce_backward_compact.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i64, vp, vp, ctypes.c_int, vp, sz, vp]
    L.cce_forward_compact_ex.restype = ctypes.c_int
    L.cce_forward_compact_ex.argtypes = [vp, vp, vp, i64, i64, i64, i32, i64, ctypes.c_float, ctypes.c_float,
                                         vp, vp, vp, vp, sz, vp]
    L.cce_backward_compact_ex.restype = ctypes.c_int
    L.cce_backward_compact_ex.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, i64, i64, i64, i32, i64,
                                          ctypes.c_float, ctypes.c_float, vp, vp, ctypes.c_int, vp, sz, vp]
    L.cce_fp8_scale_bytes.restype = sz
    L.cce_fp8_scale_bytes.argtypes = [i64, i64]
    L.cce_quantize_e4m3.restype = ctypes.c_int
    L.cce_quantize_e4m3.argtypes = [vp, i64, i64, vp, vp, vp]
    L.cce_fp8_forward.restype = ctypes.c_int
    L.cce_fp8_forward.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]
    L.cce_fp8_backward.restype = ctypes.c_int
    L.cce_fp8_backward.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, vp, vp, ctypes.c_int, vp, sz, vp]
    _lib = L
    return L


def version() -> str:
    return lib().cce_version().decode()


def workspace_bytes(N: int, D: int, V: int) -> int:
    return int(lib().cce_workspace_bytes(N, D, V))


def materialised_logit_bytes(N: int, V: int) -> int:
    return int(lib().cce_materialised_logit_bytes(N, V))


def alloc_workspace(N: int, D: int, V: int, device="cuda") -> torch.Tensor:
    n = workspace_bytes(N, D, V)
    if n == 0:
        raise CCEError(CCE_ERR_UNSUPPORTED, "cce_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _check(t: torch.Tensor, dtype, shape, name):
    if t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name}: expected contiguous cuda {dtype} {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)} contiguous={t.is_contiguous()} cuda={t.is_cuda}")


def cce_forward(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor,
                ignore_index: int = -100, *, workspace: Optional[torch.Tensor] = None,
                loss: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per-token loss and log-sum-exp (fp32 [N] each) of bf16 hidden [N, D] x weight [V, D]."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    if workspace is None:
        workspace = alloc_workspace(N, D, V, hidden.device)
    if loss is None:
        loss = torch.empty(N, dtype=torch.float32, device=hidden.device)
    if lse is None:
        lse = torch.empty(N, dtype=torch.float32, device=hidden.device)
    _check(loss, torch.float32, (N,), "loss")
    _check(lse, torch.float32, (N,), "lse")
    rc = lib().cce_forward(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), N, D, V,
                           ignore_index, loss.data_ptr(), lse.data_ptr(),
                           workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_forward")
    return loss, lse


def cce_forward_static(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor,
                       ignore_index: int, loss: torch.Tensor, lse: torch.Tensor,
                       status: Optional[torch.Tensor] = None,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
    """cce_forward with the library's static scratch: no workspace, and nothing is allocated here
    either -- every output is the caller's (loss, lse fp32 [N]; status int32 [1] or None)."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    _check(loss, torch.float32, (N,), "loss")
    _check(lse, torch.float32, (N,), "lse")
    if status is not None:
        _check(status, torch.int32, (1,), "status")
    rc = lib().cce_forward_static(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), N, D, V,
                                  ignore_index, loss.data_ptr(), lse.data_ptr(),
                                  status.data_ptr() if status is not None else None, _stream_ptr(stream))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_forward_static")


def cce_backward(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor,
                 lse: torch.Tensor, dloss: torch.Tensor, ignore_index: int = -100, *,
                 workspace: Optional[torch.Tensor] = None,
                 d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                 accumulate_dw: bool = False,
                 stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """dHidden (bf16 [N, D]) and dW (fp32 [V, D]) for upstream per-token gradient dloss [N]."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    _check(lse, torch.float32, (N,), "lse")
    _check(dloss, torch.float32, (N,), "dloss")
    if workspace is None:
        workspace = alloc_workspace(N, D, V, hidden.device)
    if d_hidden is None:
        d_hidden = torch.empty(N, D, dtype=torch.bfloat16, device=hidden.device)
    if d_weight is None:
        if accumulate_dw:
            raise ValueError("accumulate_dw needs an existing d_weight")
        d_weight = torch.empty(V, D, dtype=torch.float32, device=hidden.device)
    _check(d_hidden, torch.bfloat16, (N, D), "d_hidden")
    _check(d_weight, torch.float32, (V, D), "d_weight")
    rc = lib().cce_backward(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(),
                            lse.data_ptr(), dloss.data_ptr(), N, D, V, ignore_index,
                            d_hidden.data_ptr(), d_weight.data_ptr(), 1 if accumulate_dw else 0,
                            workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_backward")
    return d_hidden, d_weight


def cce_forward_ex(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor,
                   ignore_index: int = -100, *, label_smoothing: float = 0.0, z_loss: float = 0.0,
                   want_mean: bool = False, workspace: Optional[torch.Tensor] = None,
                   loss: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None):
    """Loss variants of the forward: (loss [N], lse [N], mean_loss [1] or None)."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    if workspace is None:
        workspace = alloc_workspace(N, D, V, hidden.device)
    if loss is None:
        loss = torch.empty(N, dtype=torch.float32, device=hidden.device)
    if lse is None:
        lse = torch.empty(N, dtype=torch.float32, device=hidden.device)
    _check(loss, torch.float32, (N,), "loss")
    _check(lse, torch.float32, (N,), "lse")
    mean = torch.empty(1, dtype=torch.float32, device=hidden.device) if want_mean else None
    rc = lib().cce_forward_ex(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), N, D, V,
                              ignore_index, label_smoothing, z_loss, loss.data_ptr(), lse.data_ptr(),
                              mean.data_ptr() if mean is not None else None,
                              workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_forward_ex")
    return loss, lse, mean


def cce_backward_ex(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor,
                    lse: torch.Tensor, dloss: Optional[torch.Tensor], ignore_index: int = -100, *,
                    grad_scale: float = 1.0, label_smoothing: float = 0.0, z_loss: float = 0.0,
                    workspace: Optional[torch.Tensor] = None,
                    d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                    accumulate_dw: bool = False,
                    stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Loss variants of the backward; dloss=None selects mean reduction (grad_scale / n_valid)."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    _check(lse, torch.float32, (N,), "lse")
    if dloss is not None:
        _check(dloss, torch.float32, (N,), "dloss")
    if workspace is None:
        workspace = alloc_workspace(N, D, V, hidden.device)
    if d_hidden is None:
        d_hidden = torch.empty(N, D, dtype=torch.bfloat16, device=hidden.device)
    if d_weight is None:
        if accumulate_dw:
            raise ValueError("accumulate_dw needs an existing d_weight")
        d_weight = torch.empty(V, D, dtype=torch.float32, device=hidden.device)
    _check(d_hidden, torch.bfloat16, (N, D), "d_hidden")
    _check(d_weight, torch.float32, (V, D), "d_weight")
    rc = lib().cce_backward_ex(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(),
                               lse.data_ptr(), dloss.data_ptr() if dloss is not None else None, grad_scale,
                               N, D, V, ignore_index, label_smoothing, z_loss,
                               d_hidden.data_ptr(), d_weight.data_ptr(), 1 if accumulate_dw else 0,
                               workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_backward_ex")
    return d_hidden, d_weight


def read_status(workspace: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> int:
    out = ctypes.c_int32(0)
    rc = lib().cce_read_status(workspace.data_ptr(), _stream_ptr(stream), ctypes.byref(out))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_read_status")
    return int(out.value)


def set_backward_tiling(row_tiles: int = 0, vocab_tiles: int = 0) -> None:
    """Force the backward tiling (in 256-wide tiles); (0, 0) restores the automatic choice."""
    rc = lib().cce_set_backward_tiling(row_tiles, vocab_tiles)
    if rc != CCE_OK:
        raise CCEError(rc, "cce_set_backward_tiling")


def get_backward_tiling(N: int, D: int, V: int) -> Tuple[int, int]:
    """(row_tiles, vocab_tiles) of the backward for this shape, in 256-wide tiles."""
    a, b = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().cce_get_backward_tiling(N, D, V, ctypes.byref(a), ctypes.byref(b))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_get_backward_tiling")
    return int(a.value), int(b.value)


def set_backward_accumulator(mode: int = 0) -> None:
    """dHidden running sum: 1 = fp32 in the workspace, 2 = split 16-bit planes, 0 = automatic."""
    rc = lib().cce_set_backward_accumulator(mode)
    if rc != CCE_OK:
        raise CCEError(rc, "cce_set_backward_accumulator")


def get_backward_accumulator(N: int, D: int, V: int) -> int:
    m = ctypes.c_int(0)
    rc = lib().cce_get_backward_accumulator(N, D, V, ctypes.byref(m))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_get_backward_accumulator")
    return int(m.value)


def set_backward_gemm_tile(tile_cols: int = 0) -> None:
    """Force the contraction output tile to 256 x tile_cols (128 or 256); 0 = automatic."""
    rc = lib().cce_set_backward_gemm_tile(tile_cols)
    if rc != CCE_OK:
        raise CCEError(rc, "cce_set_backward_gemm_tile")


def get_backward_gemm_tile(N: int, D: int, V: int) -> Tuple[int, int]:
    """(rows, columns) of the contraction output tile chosen for this shape."""
    a, b = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().cce_get_backward_gemm_tile(N, D, V, ctypes.byref(a), ctypes.byref(b))
    if rc != CCE_OK:
        raise CCEError(rc, "cce_get_backward_gemm_tile")
    return int(a.value), int(b.value)


def profile_begin() -> None:
    rc = lib().cce_profile_begin()
    if rc != CCE_OK:
        raise CCEError(rc, "cce_profile_begin")


def profile_end() -> dict:
    """{family name: (milliseconds, launches)} accumulated since profile_begin()."""
    n = len(KERNEL_FAMILIES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    rc = lib().cce_profile_end(ms, cnt)
    if rc != CCE_OK:
        raise CCEError(rc, "cce_profile_end")
    return {KERNEL_FAMILIES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}


# ---------------------------------------------------------------- include/cce_aux.h

def _rc(rc: int, where: str) -> None:
    if rc != CCE_OK:
        raise CCEError(rc, where)


def cce_rmsnorm_forward(x: torch.Tensor, gamma: torch.Tensor, eps: float, *,
                        y: Optional[torch.Tensor] = None, rstd: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(y bf16 [N, D], rstd fp32 [N]) of bf16 x [N, D] and gamma [D]."""
    N, D = x.shape
    _check(x, torch.bfloat16, (N, D), "x")
    _check(gamma, torch.bfloat16, (D,), "gamma")
    if y is None:
        y = torch.empty_like(x)
    if rstd is None:
        rstd = torch.empty(N, dtype=torch.float32, device=x.device)
    _check(y, torch.bfloat16, (N, D), "y")
    _check(rstd, torch.float32, (N,), "rstd")
    _rc(lib().cce_rmsnorm_forward(x.data_ptr(), gamma.data_ptr(), N, D, eps, y.data_ptr(), rstd.data_ptr(),
                                  _stream_ptr(stream)), "cce_rmsnorm_forward")
    return y, rstd


def cce_rmsnorm_backward(x: torch.Tensor, gamma: torch.Tensor, rstd: torch.Tensor, dy: torch.Tensor, *,
                         dx: Optional[torch.Tensor] = None, dgamma: Optional[torch.Tensor] = None,
                         accumulate_dgamma: bool = False, workspace: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(dx bf16 [N, D], dgamma fp32 [D]) for the upstream gradient dy bf16 [N, D]."""
    N, D = x.shape
    _check(x, torch.bfloat16, (N, D), "x")
    _check(gamma, torch.bfloat16, (D,), "gamma")
    _check(rstd, torch.float32, (N,), "rstd")
    _check(dy, torch.bfloat16, (N, D), "dy")
    n = int(lib().cce_rmsnorm_workspace_bytes(N, D))
    if n == 0:
        raise CCEError(CCE_ERR_UNSUPPORTED, "cce_rmsnorm_workspace_bytes")
    ws = workspace if workspace is not None else torch.empty(n, dtype=torch.uint8, device=x.device)
    if dx is None:
        dx = torch.empty_like(x)
    _check(dx, torch.bfloat16, (N, D), "dx")
    if dgamma is None:
        if accumulate_dgamma:
            raise ValueError("accumulate_dgamma needs an existing dgamma")
        dgamma = torch.empty(D, dtype=torch.float32, device=x.device)
    _check(dgamma, torch.float32, (D,), "dgamma")
    _rc(lib().cce_rmsnorm_backward(x.data_ptr(), gamma.data_ptr(), rstd.data_ptr(), dy.data_ptr(), N, D,
                                   dx.data_ptr(), dgamma.data_ptr(), 1 if accumulate_dgamma else 0,
                                   ws.data_ptr(), ws.numel(), _stream_ptr(stream)), "cce_rmsnorm_backward")
    return dx, dgamma


def cce_rmsnorm_residual_forward(x: torch.Tensor, residual: torch.Tensor, gamma: torch.Tensor, eps: float, *,
                                 y: Optional[torch.Tensor] = None, rstd: Optional[torch.Tensor] = None,
                                 stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """residual <- x + residual (in place), then (y, rstd) of the norm of that sum."""
    N, D = x.shape
    _check(x, torch.bfloat16, (N, D), "x")
    _check(residual, torch.bfloat16, (N, D), "residual")
    _check(gamma, torch.bfloat16, (D,), "gamma")
    if y is None:
        y = torch.empty_like(x)
    if rstd is None:
        rstd = torch.empty(N, dtype=torch.float32, device=x.device)
    _check(y, torch.bfloat16, (N, D), "y")
    _check(rstd, torch.float32, (N,), "rstd")
    _rc(lib().cce_rmsnorm_residual_forward(x.data_ptr(), residual.data_ptr(), gamma.data_ptr(), N, D, eps,
                                           y.data_ptr(), rstd.data_ptr(), _stream_ptr(stream)),
        "cce_rmsnorm_residual_forward")
    return y, rstd


def cce_rmsnorm_residual_backward(h: torch.Tensor, gamma: torch.Tensor, rstd: torch.Tensor, dy: torch.Tensor,
                                  d_residual: Optional[torch.Tensor] = None, *,
                                  dh: Optional[torch.Tensor] = None, dgamma: Optional[torch.Tensor] = None,
                                  accumulate_dgamma: bool = False, workspace: Optional[torch.Tensor] = None,
                                  stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(dh bf16 [N, D], dgamma fp32 [D]): gradient of h = x + residual, d_residual added if given."""
    N, D = h.shape
    _check(h, torch.bfloat16, (N, D), "h")
    _check(gamma, torch.bfloat16, (D,), "gamma")
    _check(rstd, torch.float32, (N,), "rstd")
    _check(dy, torch.bfloat16, (N, D), "dy")
    if d_residual is not None:
        _check(d_residual, torch.bfloat16, (N, D), "d_residual")
    n = int(lib().cce_rmsnorm_workspace_bytes(N, D))
    if n == 0:
        raise CCEError(CCE_ERR_UNSUPPORTED, "cce_rmsnorm_workspace_bytes")
    ws = workspace if workspace is not None else torch.empty(n, dtype=torch.uint8, device=h.device)
    if dh is None:
        dh = torch.empty_like(h)
    _check(dh, torch.bfloat16, (N, D), "dh")
    if dgamma is None:
        if accumulate_dgamma:
            raise ValueError("accumulate_dgamma needs an existing dgamma")
        dgamma = torch.empty(D, dtype=torch.float32, device=h.device)
    _check(dgamma, torch.float32, (D,), "dgamma")
    _rc(lib().cce_rmsnorm_residual_backward(h.data_ptr(), gamma.data_ptr(), rstd.data_ptr(), dy.data_ptr(),
                                            d_residual.data_ptr() if d_residual is not None else None, N, D,
                                            dh.data_ptr(), dgamma.data_ptr(), 1 if accumulate_dgamma else 0,
                                            ws.data_ptr(), ws.numel(), _stream_ptr(stream)),
        "cce_rmsnorm_residual_backward")
    return dh, dgamma


def cce_grad_sumsq(grad: torch.Tensor, sumsq: Optional[torch.Tensor] = None, accumulate: bool = False, *,
                   workspace: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Device fp64 [1] holding sum g^2 (added to `sumsq` when accumulate)."""
    if grad.dtype != torch.float32 or not grad.is_contiguous() or not grad.is_cuda:
        raise ValueError("grad: expected a contiguous cuda float32 tensor")
    if sumsq is None:
        if accumulate:
            raise ValueError("accumulate needs an existing sumsq")
        sumsq = torch.empty(1, dtype=torch.float64, device=grad.device)
    _check(sumsq, torch.float64, (1,), "sumsq")
    ws = workspace if workspace is not None else torch.empty(int(lib().cce_sumsq_workspace_bytes()),
                                                             dtype=torch.uint8, device=grad.device)
    _rc(lib().cce_grad_sumsq(grad.data_ptr(), grad.numel(), sumsq.data_ptr(), 1 if accumulate else 0,
                             ws.data_ptr(), ws.numel(), _stream_ptr(stream)), "cce_grad_sumsq")
    return sumsq


def cce_clip_coef(sumsq: torch.Tensor, max_norm: float, eps_norm: float = 1e-6, *,
                  stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Device fp32 [1]: min(1, max_norm / (sqrt(sumsq) + eps_norm))."""
    _check(sumsq, torch.float64, (1,), "sumsq")
    coef = torch.empty(1, dtype=torch.float32, device=sumsq.device)
    _rc(lib().cce_clip_coef(sumsq.data_ptr(), max_norm, eps_norm, coef.data_ptr(), _stream_ptr(stream)),
        "cce_clip_coef")
    return coef


def cce_adamw_step(param: torch.Tensor, grad: torch.Tensor, m: torch.Tensor, v: torch.Tensor, step: int, *,
                   lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
                   weight_decay: float = 0.0, param_bf16: Optional[torch.Tensor] = None,
                   clip_coef: Optional[torch.Tensor] = None,
                   stream: Optional[torch.cuda.Stream] = None) -> None:
    """In-place fused AdamW step on fp32 param / m / v; optionally also writes the bf16 copy."""
    n = param.numel()
    for name, t in (("param", param), ("grad", grad), ("m", m), ("v", v)):
        if t.dtype != torch.float32 or t.numel() != n or not t.is_contiguous() or not t.is_cuda:
            raise ValueError(f"{name}: expected a contiguous cuda float32 tensor of {n} elements")
    if param_bf16 is not None and (param_bf16.dtype != torch.bfloat16 or param_bf16.numel() != n
                                   or not param_bf16.is_contiguous()):
        raise ValueError("param_bf16: expected a contiguous bfloat16 tensor of the same size")
    _rc(lib().cce_adamw_step(param.data_ptr(), param_bf16.data_ptr() if param_bf16 is not None else None,
                             grad.data_ptr(), m.data_ptr(), v.data_ptr(), n, lr, beta1, beta2, eps, weight_decay,
                             step, clip_coef.data_ptr() if clip_coef is not None else None,
                             _stream_ptr(stream)), "cce_adamw_step")


def mfma_probe_tflops(workgroups: int = 2048, iters: int = 4000) -> float:
    """TFLOP/s of a register-only bf16 MFMA loop on the current device (measurement aid)."""
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    s = _stream_ptr(None)
    _rc(lib().cce_mfma_probe(workgroups, 10, sink.data_ptr(), s), "cce_mfma_probe")
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    _rc(lib().cce_mfma_probe(workgroups, iters, sink.data_ptr(), s), "cce_mfma_probe")
    b.record()
    torch.cuda.synchronize()
    flops = float(workgroups) * 8 * iters * 8 * 32768
    return flops / (a.elapsed_time(b) * 1e-3) / 1e12


def mfma_probe_data_tflops(operands: torch.Tensor, workgroups: int = 2048, iters: int = 4000) -> float:
    """TFLOP/s of the register-only bf16 MFMA loop whose operand fragments are loaded once from
    `operands` (bf16, at least 512 * 48 values) before the loop (measurement aid)."""
    if operands.dtype != torch.bfloat16 or not operands.is_contiguous() or operands.numel() < 512 * 48:
        raise ValueError("operands: expected a contiguous bfloat16 tensor of at least 24576 values")
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    s = _stream_ptr(None)
    _rc(lib().cce_mfma_probe_data(workgroups, 10, operands.data_ptr(), sink.data_ptr(), s), "cce_mfma_probe_data")
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    _rc(lib().cce_mfma_probe_data(workgroups, iters, operands.data_ptr(), sink.data_ptr(), s), "cce_mfma_probe_data")
    b.record()
    torch.cuda.synchronize()
    flops = float(workgroups) * 8 * iters * 8 * 32768
    return flops / (a.elapsed_time(b) * 1e-3) / 1e12


def device_info() -> Tuple[int, int]:
    """(compute units, peak shader clock in kHz) of the current device."""
    cu, khz = ctypes.c_int(0), ctypes.c_int(0)
    _rc(lib().cce_device_info(ctypes.byref(cu), ctypes.byref(khz)), "cce_device_info")
    return int(cu.value), int(khz.value)


# ---------------------------------------------------------------- include/cce_shard.h

def cce_shard_forward(hidden: torch.Tensor, weight_shard: torch.Tensor, labels: torch.Tensor,
                      vocab_offset: int, *, want_sumz: bool = False,
                      stats: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Per-token (max, sum-exp, label logit, logit sum) of one vocabulary shard, fp32 [N, 4]."""
    N, D = hidden.shape
    Vs = weight_shard.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight_shard, torch.bfloat16, (Vs, D), "weight_shard")
    _check(labels, torch.int32, (N,), "labels")
    if workspace is None:
        workspace = alloc_workspace(N, D, Vs, hidden.device)
    if stats is None:
        stats = torch.empty(N, 4, dtype=torch.float32, device=hidden.device)
    _check(stats, torch.float32, (N, 4), "stats")
    _rc(lib().cce_shard_forward(hidden.data_ptr(), weight_shard.data_ptr(), labels.data_ptr(), N, D, Vs,
                                vocab_offset, 1 if want_sumz else 0, stats.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_shard_forward")
    return stats


def cce_shard_merge(stats: torch.Tensor, labels: torch.Tensor, V_total: int, ignore_index: int = -100, *,
                    label_smoothing: float = 0.0, z_loss: float = 0.0, want_mean: bool = False,
                    status: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None):
    """(loss [N], lse [N], mean_loss [1] or None) from the stacked shard statistics [P, N, 4]."""
    P, N, _ = stats.shape
    _check(stats, torch.float32, (P, N, 4), "stats")
    _check(labels, torch.int32, (N,), "labels")
    if status is not None:
        _check(status, torch.int32, (1,), "status")
    loss = torch.empty(N, dtype=torch.float32, device=stats.device)
    lse = torch.empty(N, dtype=torch.float32, device=stats.device)
    mean = torch.empty(1, dtype=torch.float32, device=stats.device) if want_mean else None
    _rc(lib().cce_shard_merge(stats.data_ptr(), P, labels.data_ptr(), N, V_total, ignore_index,
                              label_smoothing, z_loss, loss.data_ptr(), lse.data_ptr(),
                              mean.data_ptr() if mean is not None else None,
                              status.data_ptr() if status is not None else None,
                              _stream_ptr(stream)), "cce_shard_merge")
    return loss, lse, mean


def cce_shard_backward(hidden: torch.Tensor, weight_shard: torch.Tensor, labels: torch.Tensor,
                       lse: torch.Tensor, dloss: Optional[torch.Tensor], vocab_offset: int, V_total: int,
                       ignore_index: int = -100, *, grad_scale: float = 1.0,
                       label_smoothing: float = 0.0, z_loss: float = 0.0,
                       workspace: Optional[torch.Tensor] = None,
                       d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                       accumulate_dw: bool = False,
                       stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(partial dHidden bf16 [N, D], dW of the shard fp32 [Vs, D]) from the global lse."""
    N, D = hidden.shape
    Vs = weight_shard.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight_shard, torch.bfloat16, (Vs, D), "weight_shard")
    _check(labels, torch.int32, (N,), "labels")
    _check(lse, torch.float32, (N,), "lse")
    if dloss is not None:
        _check(dloss, torch.float32, (N,), "dloss")
    if workspace is None:
        workspace = alloc_workspace(N, D, Vs, hidden.device)
    if d_hidden is None:
        d_hidden = torch.empty(N, D, dtype=torch.bfloat16, device=hidden.device)
    if d_weight is None:
        if accumulate_dw:
            raise ValueError("accumulate_dw needs an existing d_weight")
        d_weight = torch.empty(Vs, D, dtype=torch.float32, device=hidden.device)
    _check(d_hidden, torch.bfloat16, (N, D), "d_hidden")
    _check(d_weight, torch.float32, (Vs, D), "d_weight")
    _rc(lib().cce_shard_backward(hidden.data_ptr(), weight_shard.data_ptr(), labels.data_ptr(), lse.data_ptr(),
                                 dloss.data_ptr() if dloss is not None else None, grad_scale,
                                 N, D, Vs, vocab_offset, V_total, ignore_index, label_smoothing, z_loss,
                                 d_hidden.data_ptr(), d_weight.data_ptr(), 1 if accumulate_dw else 0,
                                 workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_shard_backward")
    return d_hidden, d_weight


# ---------------------------------------------------------------- include/cce_fp8.h

def fp8_scale_bytes(rows: int, D: int) -> int:
    return int(lib().cce_fp8_scale_bytes(rows, D))


def cce_quantize_e4m3(x: torch.Tensor, *, q: Optional[torch.Tensor] = None, scales: Optional[torch.Tensor] = None,
                      stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """(E4M3 codes uint8 [rows, D], block-scale exponent bytes uint8 [fp8_scale_bytes]) of bf16 x."""
    rows, D = x.shape
    _check(x, torch.bfloat16, (rows, D), "x")
    n = fp8_scale_bytes(rows, D)
    if n == 0:
        raise CCEError(CCE_ERR_UNSUPPORTED, "cce_fp8_scale_bytes")
    if q is None:
        q = torch.empty(rows, D, dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(n, dtype=torch.uint8, device=x.device)
    _check(q, torch.uint8, (rows, D), "q")
    _check(scales, torch.uint8, (n,), "scales")
    _rc(lib().cce_quantize_e4m3(x.data_ptr(), rows, D, q.data_ptr(), scales.data_ptr(), _stream_ptr(stream)),
        "cce_quantize_e4m3")
    return q, scales


def cce_fp8_forward(hidden_q: torch.Tensor, hidden_scales: torch.Tensor, weight_q: torch.Tensor,
                    weight_scales: torch.Tensor, labels: torch.Tensor, ignore_index: int = -100, *,
                    workspace: Optional[torch.Tensor] = None, loss: Optional[torch.Tensor] = None,
                    lse: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Per-token loss and log-sum-exp from the E4M3 operands."""
    N, D = hidden_q.shape
    V = weight_q.shape[0]
    _check(hidden_q, torch.uint8, (N, D), "hidden_q")
    _check(weight_q, torch.uint8, (V, D), "weight_q")
    _check(hidden_scales, torch.uint8, (fp8_scale_bytes(N, D),), "hidden_scales")
    _check(weight_scales, torch.uint8, (fp8_scale_bytes(V, D),), "weight_scales")
    _check(labels, torch.int32, (N,), "labels")
    if workspace is None:
        workspace = alloc_workspace(N, D, V, hidden_q.device)
    if loss is None:
        loss = torch.empty(N, dtype=torch.float32, device=hidden_q.device)
    if lse is None:
        lse = torch.empty(N, dtype=torch.float32, device=hidden_q.device)
    _check(loss, torch.float32, (N,), "loss")
    _check(lse, torch.float32, (N,), "lse")
    _rc(lib().cce_fp8_forward(hidden_q.data_ptr(), hidden_scales.data_ptr(), weight_q.data_ptr(),
                              weight_scales.data_ptr(), labels.data_ptr(), N, D, V, ignore_index,
                              loss.data_ptr(), lse.data_ptr(), workspace.data_ptr(), workspace.numel(),
                              _stream_ptr(stream)), "cce_fp8_forward")
    return loss, lse


def cce_fp8_backward(hidden_q: torch.Tensor, hidden_scales: torch.Tensor, weight_q: torch.Tensor,
                     weight_scales: torch.Tensor, hidden: torch.Tensor, weight: torch.Tensor,
                     labels: torch.Tensor, lse: torch.Tensor, dloss: torch.Tensor, ignore_index: int = -100, *,
                     workspace: Optional[torch.Tensor] = None,
                     d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                     accumulate_dw: bool = False,
                     stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """dHidden (bf16) and dW (fp32): gradient tiles from the E4M3 logits, contracted with the bf16 operands."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden_q, torch.uint8, (N, D), "hidden_q")
    _check(weight_q, torch.uint8, (V, D), "weight_q")
    _check(hidden_scales, torch.uint8, (fp8_scale_bytes(N, D),), "hidden_scales")
    _check(weight_scales, torch.uint8, (fp8_scale_bytes(V, D),), "weight_scales")
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    _check(lse, torch.float32, (N,), "lse")
    _check(dloss, torch.float32, (N,), "dloss")
    if workspace is None:
        workspace = alloc_workspace(N, D, V, hidden.device)
    if d_hidden is None:
        d_hidden = torch.empty(N, D, dtype=torch.bfloat16, device=hidden.device)
    if d_weight is None:
        if accumulate_dw:
            raise ValueError("accumulate_dw needs an existing d_weight")
        d_weight = torch.empty(V, D, dtype=torch.float32, device=hidden.device)
    _check(d_hidden, torch.bfloat16, (N, D), "d_hidden")
    _check(d_weight, torch.float32, (V, D), "d_weight")
    _rc(lib().cce_fp8_backward(hidden_q.data_ptr(), hidden_scales.data_ptr(), weight_q.data_ptr(),
                               weight_scales.data_ptr(), hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(),
                               lse.data_ptr(), dloss.data_ptr(), N, D, V, ignore_index,
                               d_hidden.data_ptr(), d_weight.data_ptr(), 1 if accumulate_dw else 0,
                               workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_fp8_backward")
    return d_hidden, d_weight


# ---------------------------------------------------------------- include/cce_compact.h

def compact_workspace_bytes(N: int, D: int, V: int, max_valid_rows: int) -> int:
    return int(lib().cce_compact_workspace_bytes(N, D, V, max_valid_rows))


def set_row_skipping(mode: int = 0) -> None:
    """1 = never skip rows, 2 = skip whenever the bound is below N, 0 = automatic."""
    _rc(lib().cce_set_row_skipping(mode), "cce_set_row_skipping")


def get_row_skipping(N: int, D: int, V: int, max_valid_rows: int) -> bool:
    m = ctypes.c_int(0)
    _rc(lib().cce_get_row_skipping(N, D, V, max_valid_rows, ctypes.byref(m)), "cce_get_row_skipping")
    return bool(m.value)


def get_compact_tiling(N: int, D: int, V: int, max_valid_rows: int) -> Tuple[int, int]:
    a, b = ctypes.c_int(0), ctypes.c_int(0)
    _rc(lib().cce_get_compact_tiling(N, D, V, max_valid_rows, ctypes.byref(a), ctypes.byref(b)), "cce_get_compact_tiling")
    return a.value, b.value


def alloc_compact_workspace(N: int, D: int, V: int, max_valid_rows: int, device="cuda") -> torch.Tensor:
    n = compact_workspace_bytes(N, D, V, max_valid_rows)
    if n == 0:
        raise CCEError(CCE_ERR_UNSUPPORTED, "cce_compact_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def cce_forward_compact(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor, max_valid_rows: int,
                        ignore_index: int = -100, *, workspace: Optional[torch.Tensor] = None,
                        loss: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                        stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """cce_forward over the valid rows only (max_valid_rows: host upper bound on their number)."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    if workspace is None:
        workspace = alloc_compact_workspace(N, D, V, max_valid_rows, hidden.device)
    if loss is None:
        loss = torch.empty(N, dtype=torch.float32, device=hidden.device)
    if lse is None:
        lse = torch.empty(N, dtype=torch.float32, device=hidden.device)
    _check(loss, torch.float32, (N,), "loss")
    _check(lse, torch.float32, (N,), "lse")
    _rc(lib().cce_forward_compact(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), N, D, V, ignore_index,
                                  max_valid_rows, loss.data_ptr(), lse.data_ptr(),
                                  workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_forward_compact")
    return loss, lse


def cce_backward_compact(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor, lse: torch.Tensor,
                         dloss: torch.Tensor, max_valid_rows: int, ignore_index: int = -100, *,
                         workspace: Optional[torch.Tensor] = None,
                         d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                         accumulate_dw: bool = False,
                         stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """cce_backward over the valid rows only."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    _check(lse, torch.float32, (N,), "lse")
    _check(dloss, torch.float32, (N,), "dloss")
    if workspace is None:
        workspace = alloc_compact_workspace(N, D, V, max_valid_rows, hidden.device)
    if d_hidden is None:
        d_hidden = torch.empty(N, D, dtype=torch.bfloat16, device=hidden.device)
    if d_weight is None:
        if accumulate_dw:
            raise ValueError("accumulate_dw needs an existing d_weight")
        d_weight = torch.empty(V, D, dtype=torch.float32, device=hidden.device)
    _check(d_hidden, torch.bfloat16, (N, D), "d_hidden")
    _check(d_weight, torch.float32, (V, D), "d_weight")
    _rc(lib().cce_backward_compact(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), lse.data_ptr(),
                                   dloss.data_ptr(), N, D, V, ignore_index, max_valid_rows,
                                   d_hidden.data_ptr(), d_weight.data_ptr(), 1 if accumulate_dw else 0,
                                   workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_backward_compact")
    return d_hidden, d_weight


def cce_forward_compact_ex(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor, max_valid_rows: int,
                           ignore_index: int = -100, *, label_smoothing: float = 0.0, z_loss: float = 0.0,
                           want_mean: bool = False, workspace: Optional[torch.Tensor] = None,
                           loss: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                           stream: Optional[torch.cuda.Stream] = None):
    """Loss variants of the forward over the valid rows only: (loss [N], lse [N], mean_loss [1] or None)."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    if workspace is None:
        workspace = alloc_compact_workspace(N, D, V, max_valid_rows, hidden.device)
    if loss is None:
        loss = torch.empty(N, dtype=torch.float32, device=hidden.device)
    if lse is None:
        lse = torch.empty(N, dtype=torch.float32, device=hidden.device)
    _check(loss, torch.float32, (N,), "loss")
    _check(lse, torch.float32, (N,), "lse")
    mean = torch.empty(1, dtype=torch.float32, device=hidden.device) if want_mean else None
    _rc(lib().cce_forward_compact_ex(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), N, D, V, ignore_index,
                                     max_valid_rows, label_smoothing, z_loss, loss.data_ptr(), lse.data_ptr(),
                                     mean.data_ptr() if mean is not None else None,
                                     workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_forward_compact_ex")
    return loss, lse, mean


def cce_backward_compact_ex(hidden: torch.Tensor, weight: torch.Tensor, labels: torch.Tensor, lse: torch.Tensor,
                            dloss: Optional[torch.Tensor], max_valid_rows: int, ignore_index: int = -100, *,
                            grad_scale: float = 1.0, label_smoothing: float = 0.0, z_loss: float = 0.0,
                            workspace: Optional[torch.Tensor] = None,
                            d_hidden: Optional[torch.Tensor] = None, d_weight: Optional[torch.Tensor] = None,
                            accumulate_dw: bool = False,
                            stream: Optional[torch.cuda.Stream] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Loss variants of the backward over the valid rows only; dloss=None selects mean reduction."""
    N, D = hidden.shape
    V = weight.shape[0]
    _check(hidden, torch.bfloat16, (N, D), "hidden")
    _check(weight, torch.bfloat16, (V, D), "weight")
    _check(labels, torch.int32, (N,), "labels")
    _check(lse, torch.float32, (N,), "lse")
    if dloss is not None:
        _check(dloss, torch.float32, (N,), "dloss")
    if workspace is None:
        workspace = alloc_compact_workspace(N, D, V, max_valid_rows, hidden.device)
    if d_hidden is None:
        d_hidden = torch.empty(N, D, dtype=torch.bfloat16, device=hidden.device)
    if d_weight is None:
        if accumulate_dw:
            raise ValueError("accumulate_dw needs an existing d_weight")
        d_weight = torch.empty(V, D, dtype=torch.float32, device=hidden.device)
    _check(d_hidden, torch.bfloat16, (N, D), "d_hidden")
    _check(d_weight, torch.float32, (V, D), "d_weight")
    _rc(lib().cce_backward_compact_ex(hidden.data_ptr(), weight.data_ptr(), labels.data_ptr(), lse.data_ptr(),
                                      dloss.data_ptr() if dloss is not None else None, grad_scale,
                                      N, D, V, ignore_index, max_valid_rows, label_smoothing, z_loss,
                                      d_hidden.data_ptr(), d_weight.data_ptr(), 1 if accumulate_dw else 0,
                                      workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "cce_backward_compact_ex")
    return d_hidden, d_weight

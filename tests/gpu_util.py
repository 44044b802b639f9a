"""Helpers shared by the GPU parity tests: host<->device marshalling and error measures."""
from __future__ import annotations

import numpy as np
import torch

from paper_2601_02609_amd import inputs as I

LOSS_ATOL = 2e-3       # per-token loss and lse, absolute
GRAD_RTOL = 1e-2       # dHidden and dW, relative Frobenius error


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_host(t: torch.Tensor) -> np.ndarray:
    """bf16 device tensor -> float64 numpy (exact)."""
    bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return I.bf16_bits_to_f32(bits).astype(np.float64)


def dev_inputs(w):
    H = bf16_dev(w.hidden)
    W = bf16_dev(w.weight)
    y = torch.from_numpy(w.labels).cuda()
    return H, W, y


def rel_fro(x: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((x - ref).ravel())
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)

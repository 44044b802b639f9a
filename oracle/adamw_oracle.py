"""fp64 CPU oracle for the fused AdamW step and the gradient-clipping coefficient, the step
behind the LM head (it consumes the fp32 weight gradient).

TEST INFRASTRUCTURE ONLY: the slow, plain definition the HIP kernels are checked against.
It shares no code with the GPU path, imports nothing from the package and is never called
from the product path.

Steps, in the order of the paper's fused AdamW kernel (supplementary section on the fused
AdamW kernel) and of its GPU-resident clipping algorithm (gradient-clipping strategies):

    clip_coef = min(1, max_norm / (||g||_2 + eps_norm))
    g   <- g * clip_coef
    p   <- p * (1 - lr * weight_decay)            decoupled decay, before the update
    m   <- beta1 m + (1 - beta1) g
    v   <- beta2 v + (1 - beta2) g^2
    p   <- p - lr * (m / bc1) / (sqrt(v / bc2) + eps),   bc_k = 1 - beta_k^step

Everything is float64 here; the kernels compute in fp32 (the paper keeps optimizer arithmetic
and state in FP32).  Pinned by tests/test_next_oracle_pins.py against torch.optim.AdamW and
torch.nn.utils.clip_grad_norm_ (float64, CPU) and closed forms.
"""
from __future__ import annotations

import math

import numpy as np

__all__ = ["clip_coef", "adamw_step"]


def clip_coef(grads, max_norm: float, eps_norm: float = 1e-6) -> float:
    """min(1, max_norm / (global L2 norm of all gradient arrays + eps_norm))."""
    total = 0.0
    for g in grads:
        g = np.asarray(g, dtype=np.float64)
        total += float((g * g).sum())
    return min(1.0, max_norm / (math.sqrt(total) + eps_norm))


def adamw_step(p, g, m, v, step: int, lr: float, beta1: float, beta2: float, eps: float,
               weight_decay: float, clip: float = 1.0):
    """One step; returns new (p, m, v) as float64 arrays.  `step` counts from 1."""
    p = np.asarray(p, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) * clip
    m = np.asarray(m, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if step < 1:
        raise ValueError("step counts from 1")
    bc1 = 1.0 - beta1 ** step
    bc2 = 1.0 - beta2 ** step
    p = p * (1.0 - lr * weight_decay)
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    p = p - lr * (m / bc1) / (np.sqrt(v / bc2) + eps)
    return p, m, v

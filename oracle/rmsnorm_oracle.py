"""fp64 CPU oracle for RMSNorm, the step in front of the LM head.

TEST INFRASTRUCTURE ONLY: the slow, plain definition the HIP kernels are checked against.
It shares no code with the GPU path, imports nothing from the package and is never called
from the product path.

What it computes, and where the paper defines it:

* forward   y_i = x_i / r * gamma_i,  r = sqrt(mean_j x_j^2 + eps)   (RMSNorm definition in the
            mathematical-foundations section; the fused forward kernel also stores
            rstd = 1 / r per row for the backward)
* backward  the derivative of that definition for an upstream gradient g = dL/dy:
              dx_i = rstd * (gamma_i g_i - xhat_i * c),   xhat = x * rstd,
              c    = mean_j (g_j gamma_j xhat_j)
              dgamma_i = sum over rows of g_i xhat_i
            Reading taken: the paper's backward proposition and its kernel listing both
            print the second term of dx with a stray factor gamma_i (and the proposition
            drops the 1/d of the mean); neither is the derivative of the printed forward
            unless gamma = 1.  The oracle is the derivative itself, which the pins
            (torch autograd, central finite differences) confirm; dgamma is as printed.

* residual form  the fused RMSNorm-with-residual kernel of the paper first forms
            h = x + residual, stores h as the new residual stream, and normalises h.  The
            tensors are bf16, so the stored h is the sum rounded once to bf16 (nearest even) and
            it is that stored value which is normalised (reading: the listing computes the
            variance from the very value it has just stored).  Backward: x and residual both
            receive dh = d(norm)/dh + whatever arrives through the residual stream.

Inputs are bf16 bit patterns (uint16), widened exactly to float64; everything after that is
float64.  Pinned by tests/test_next_oracle_pins.py.
"""
from __future__ import annotations

import numpy as np

__all__ = ["widen_bf16", "round_bf16", "forward", "backward", "forward_residual", "backward_residual"]


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    bits = np.asarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns")
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def forward(x_bits: np.ndarray, gamma_bits: np.ndarray, eps: float):
    """(y [N, D], rstd [N]) in float64."""
    x = widen_bf16(x_bits)
    gamma = widen_bf16(gamma_bits)
    if x.ndim != 2 or gamma.shape != (x.shape[1],):
        raise ValueError("x is [N, D], gamma is [D]")
    rstd = 1.0 / np.sqrt((x * x).mean(axis=1) + eps)
    return x * rstd[:, None] * gamma[None, :], rstd


def backward(x_bits: np.ndarray, gamma_bits: np.ndarray, dy_bits: np.ndarray, eps: float):
    """(dx [N, D], dgamma [D]) in float64 for the upstream gradient dy (bf16 bits)."""
    x = widen_bf16(x_bits)
    gamma = widen_bf16(gamma_bits)
    g = widen_bf16(dy_bits)
    if g.shape != x.shape:
        raise ValueError("dy has the shape of x")
    rstd = 1.0 / np.sqrt((x * x).mean(axis=1) + eps)
    xhat = x * rstd[:, None]
    c = (g * gamma[None, :] * xhat).mean(axis=1)
    dx = rstd[:, None] * (gamma[None, :] * g - xhat * c[:, None])
    dgamma = (g * xhat).sum(axis=0)
    return dx, dgamma


def round_bf16(v: np.ndarray) -> np.ndarray:
    """float64 -> bf16 bit patterns, round to nearest, ties to even (finite values).  The two
    candidates are the bf16 number obtained by dropping the low 16 bits of the float32 nearest to
    v (its magnitude is at most one bf16 step away from |v|) and the next larger magnitude; the
    distances are compared in float64, so v is rounded once."""
    v = np.asarray(v, dtype=np.float64)
    f_bits = v.astype(np.float32).view(np.uint32)
    lo_bits = f_bits >> np.uint32(16)
    cand = np.stack([lo_bits - np.uint32(1), lo_bits, lo_bits + np.uint32(1)])      # neighbouring magnitudes
    cand = np.where((lo_bits & np.uint32(0x7FFF)) == 0, np.stack([lo_bits, lo_bits, lo_bits + np.uint32(1)]), cand)
    vals = (cand << np.uint32(16)).astype(np.uint32).view(np.float32).astype(np.float64)
    dist = np.abs(vals - v[None])
    # nearest; on a tie the candidate with an even last bit
    best = np.zeros(v.shape, dtype=np.int64)
    for k in (1, 2):
        better = (dist[k] < np.take_along_axis(dist, best[None], 0)[0]) | \
                 ((dist[k] == np.take_along_axis(dist, best[None], 0)[0]) & ((cand[k] & np.uint32(1)) == 0))
        best = np.where(better, k, best)
    return np.take_along_axis(cand, best[None], 0)[0].astype(np.uint16)


def forward_residual(x_bits: np.ndarray, residual_bits: np.ndarray, gamma_bits: np.ndarray, eps: float):
    """(h bits uint16 [N, D], y [N, D], rstd [N]): h = bf16(x + residual), y = RMSNorm(h)."""
    h_bits = round_bf16(widen_bf16(x_bits) + widen_bf16(residual_bits))
    y, rstd = forward(h_bits, gamma_bits, eps)
    return h_bits, y, rstd


def backward_residual(h_bits: np.ndarray, gamma_bits: np.ndarray, dy_bits: np.ndarray, eps: float,
                      d_residual_bits: np.ndarray | None = None):
    """(dh [N, D], dgamma [D]): gradient of h (= of x and of the incoming residual)."""
    dh, dgamma = backward(h_bits, gamma_bits, dy_bits, eps)
    if d_residual_bits is not None:
        dh = dh + widen_bf16(d_residual_bits)
    return dh, dgamma

"""fp64 CPU oracle for the vocabulary-parallel share of the fused LM-head + cross-entropy path.

TEST INFRASTRUCTURE ONLY (same rules as cce_oracle.py: no code shared with the GPU path,
nothing imported from the package, never called from the product path).

A device that holds the rows [v_off, v_off + Vs) of the LM-head matrix reduces them, per
token, to the online-softmax state of that vocabulary range plus the two sums the loss
needs; the states of disjoint ranges combine into the state of their union (online-softmax
definition and correctness theorem: the running maximum m and the denominator
d = sum exp(z - m) of a prefix can be corrected for a later maximum, and by the same identity
exp(z - m1) = exp(z - m2) exp(m2 - m1) two disjoint ranges combine).  Everything here is the
plain definition on fully materialised shard logits, in float64:

* shard_stats   m = max_v z_v,  d = sum_v exp(z_v - m),  z_y if the label lies in the shard
                else 0,  sum_v z_v                       (v over the shard's rows)
* merge         M = max_p m_p,  lse = M + ln sum_p d_p exp(m_p - M);  z_y and sum z add up;
                loss as in the cross-entropy / smoothed cross-entropy / z-loss definitions
* shard_backward  G_iv = dloss_i ((1 + 2 lambda lse_i) exp(z_iv - lse_i) - (1 - eps) [v = y_i]
                - eps / V_total) for the shard's v (cross-entropy gradient proposition, CCE
                backward theorem, z-loss gradient proposition, with the GLOBAL lse);
                dH_partial = G W_shard,  dW_shard = G^T H

Pinned by tests/test_shard_oracle_pins.py against torch.logsumexp, torch cross_entropy with
autograd on the undivided matrix (float64), invariance to the partition and to the shard
order, and labels on shard boundaries.
"""
from __future__ import annotations

import numpy as np

__all__ = ["shard_stats", "merge", "shard_backward"]


def _widen(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def shard_stats(hidden_bits, weight_shard_bits, labels, vocab_offset):
    """[N, 4] float64: (m, d, z_y or 0, sum z) over the shard's rows, for every token."""
    H = _widen(hidden_bits)
    Ws = _widen(weight_shard_bits)
    labels = np.asarray(labels, dtype=np.int64)
    N, Vs = H.shape[0], Ws.shape[0]
    Z = H @ Ws.T
    out = np.zeros((N, 4), dtype=np.float64)
    out[:, 0] = Z.max(axis=1)
    out[:, 1] = np.exp(Z - out[:, 0:1]).sum(axis=1)
    local = labels - int(vocab_offset)
    mine = (local >= 0) & (local < Vs)
    rows = np.nonzero(mine)[0]
    out[rows, 2] = Z[rows, local[rows]]
    out[:, 3] = Z.sum(axis=1)
    return out


def merge(stats, labels, V_total, ignore_index=-100, label_smoothing=0.0, z_loss=0.0):
    """(loss [N], lse [N]) from the list / array of per-shard statistics [P, N, 4]."""
    stats = np.asarray(stats, dtype=np.float64)
    labels = np.asarray(labels, dtype=np.int64)
    if stats.ndim != 3 or stats.shape[2] != 4:
        raise ValueError("stats must be [P, N, 4]")
    if np.any((labels != ignore_index) & ((labels < 0) | (labels >= V_total))):
        raise ValueError("label outside [0, V_total)")
    valid = labels != ignore_index
    m, d = stats[:, :, 0], stats[:, :, 1]
    M = m.max(axis=0)
    lse_all = M + np.log((d * np.exp(m - M[None, :])).sum(axis=0))
    zy = stats[:, :, 2].sum(axis=0)
    sumz = stats[:, :, 3].sum(axis=0)
    ce = lse_all - zy
    uniform = lse_all - sumz / float(V_total)
    loss_all = (1.0 - label_smoothing) * ce + label_smoothing * uniform + z_loss * lse_all ** 2
    return np.where(valid, loss_all, 0.0), np.where(valid, lse_all, 0.0)


def shard_backward(hidden_bits, weight_shard_bits, labels, lse, dloss, vocab_offset, V_total,
                   ignore_index=-100, label_smoothing=0.0, z_loss=0.0):
    """(dH_partial [N, D], dW_shard [Vs, D]) in float64 from the global log-sum-exp."""
    H = _widen(hidden_bits)
    Ws = _widen(weight_shard_bits)
    labels = np.asarray(labels, dtype=np.int64)
    lse = np.asarray(lse, dtype=np.float64)
    Vs = Ws.shape[0]
    valid = labels != ignore_index
    Z = H @ Ws.T
    P = np.exp(Z - lse[:, None])
    G = (1.0 + 2.0 * z_loss * lse)[:, None] * P - label_smoothing / float(V_total)
    local = labels - int(vocab_offset)
    rows = np.nonzero(valid & (local >= 0) & (local < Vs))[0]
    G[rows, local[rows]] -= (1.0 - label_smoothing)
    g = np.where(valid, np.asarray(dloss, dtype=np.float64), 0.0)
    G = G * g[:, None]
    G[~valid] = 0.0
    return G @ Ws, G.T @ H

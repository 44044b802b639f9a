"""fp64 CPU oracle for the fused LM-head + cross-entropy path.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
library is checked against.  It shares no code with the GPU path, imports
nothing from the package, and must never be called from the product path; only
tests, the smoke check and the benchmark's ``cpu_baseline`` leg use it.

What it computes, and where the paper defines it:

* logits           Z = H W^T (language-model head without bias; chunked-forward
                   algorithm of the Cut Cross-Entropy section, the step that forms
                   the partial logits of a vocabulary chunk)
* log-sum-exp      lse_i = m_i + ln sum_v exp(Z_iv - m_i), m_i = max_v Z_iv
                   (stable log-sum-exp, numerical-stability appendix; the online
                   softmax correctness theorem states that the streamed recurrence
                   reaches exactly this value, so the oracle is the plain formula)
* per-token loss   L_i = lse_i - Z_{i,y_i}        (cross-entropy definition in the
                   mathematical-foundations section; restated in the CCE section)
* logit gradient   dL_i/dZ_iv = softmax(Z_i)_v - 1[v = y_i]   (cross-entropy
                   gradient proposition; CCE backward theorem)
* input gradients  dH = G W,  dW = G^T H  with  G_iv = dloss_i * dL_i/dZ_iv
                   (chunk-level backward algorithm of the CCE section, summed
                   over all chunks)

Loss variants (same section of the paper as the cross-entropy definition):
* label smoothing  L_smooth = (1 - eps) L + eps L_uniform,  L_uniform = -(1/V) sum_v z_v + lse
                   (smoothed cross-entropy definition); its logit gradient is
                   softmax - (1 - eps) onehot - eps / V
* z-loss           L_total = L + lambda_z lse^2 (z-loss definition), gradient contribution
                   2 lambda_z lse softmax (z-loss gradient proposition)
* mean reduction   sum of the per-token losses over the number of non-ignored rows (the
                   materialising cross-entropy kernel of the paper divides by n_non_ignore)
Both variants are per token and combine as (1 - eps) L + eps L_uniform + lambda_z lse^2.

Readings taken where the paper is silent (each is listed in the design notes):
rows whose label equals ``ignore_index`` give loss 0, lse 0 and contribute
exactly nothing to either gradient whatever their ``dloss`` holds (the forward
kernel listing stores 0 and returns for such rows); the upstream gradient is
a per-token factor; labels outside [0, V) other than ``ignore_index`` are an
error.  No bias, no label shift, no logit scaling or soft-capping.

Inputs are bf16 bit patterns (``uint16``); they are widened exactly to float64
and every operation after that is float64.  Row blocking only bounds memory:
each block still materialises its full [rows x V] logits.

All functions are pinned by tests/test_oracle_pins.py against closed forms,
invariants, a brute-force loop, central finite differences and
``torch.nn.functional.cross_entropy`` (float64, CPU, with autograd).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "widen_bf16", "logits", "forward", "grad_logits", "backward", "dweight_rows", "mean_loss",
    "logit_memory_bytes", "chunk_reduction_factor",
]


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly."""
    bits = np.asarray(bits)
    if bits.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns")
    as_f32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return as_f32.astype(np.float64)


def _check(hidden_bits, weight_bits, labels, ignore_index):
    if hidden_bits.ndim != 2 or weight_bits.ndim != 2:
        raise ValueError("hidden is [N, D], weight is [V, D]")
    N, D = hidden_bits.shape
    V, D2 = weight_bits.shape
    if D != D2:
        raise ValueError("hidden and weight disagree on D")
    labels = np.asarray(labels)
    if labels.shape != (N,):
        raise ValueError("labels is [N]")
    valid = labels != ignore_index
    lab = labels[valid]
    if lab.size and (lab.min() < 0 or lab.max() >= V):
        raise ValueError("label outside [0, V) that is not ignore_index")
    return N, D, V, valid


def logits(hidden_bits: np.ndarray, weight_bits: np.ndarray) -> np.ndarray:
    """Z[i, v] = sum_k H[i, k] W[v, k] in float64, fully materialised."""
    return widen_bf16(hidden_bits) @ widen_bf16(weight_bits).T


def _lse_rows(Z: np.ndarray) -> np.ndarray:
    m = Z.max(axis=1)
    return m + np.log(np.exp(Z - m[:, None]).sum(axis=1))


def forward(hidden_bits, weight_bits, labels, ignore_index=-100, row_block=1024,
            label_smoothing=0.0, z_loss=0.0):
    """Per-token loss and log-sum-exp, float64 [N] each.

    loss_i = (1 - eps) (lse_i - z_iy) + eps (lse_i - mean_v z_iv) + lambda_z lse_i^2.
    Ignored rows: loss = lse = 0 exactly.
    """
    N, D, V, valid = _check(hidden_bits, weight_bits, labels, ignore_index)
    W = widen_bf16(weight_bits)
    loss = np.zeros(N, dtype=np.float64)
    lse = np.zeros(N, dtype=np.float64)
    for r0 in range(0, N, row_block):
        r1 = min(N, r0 + row_block)
        Z = widen_bf16(hidden_bits[r0:r1]) @ W.T
        l = _lse_rows(Z)
        vb = valid[r0:r1]
        idx = np.nonzero(vb)[0]
        zy = Z[idx, labels[r0:r1][idx]]
        lse[r0 + idx] = l[idx]
        ce = l[idx] - zy
        uniform = l[idx] - Z[idx].mean(axis=1)
        loss[r0 + idx] = (1.0 - label_smoothing) * ce + label_smoothing * uniform + z_loss * l[idx] ** 2
    return loss, lse


def grad_logits(hidden_bits, weight_bits, labels, dloss, ignore_index=-100,
                label_smoothing=0.0, z_loss=0.0):
    """G[i, v] = dloss_i * dloss_i/dz_iv; zero rows where ignored.

    d loss_i / d z_iv = softmax_v - (1 - eps) 1[v = y_i] - eps / V + 2 lambda_z lse_i softmax_v.
    Materialises [N x V]: for small inputs or row subsets.
    """
    N, D, V, valid = _check(hidden_bits, weight_bits, labels, ignore_index)
    Z = logits(hidden_bits, weight_bits)
    l = _lse_rows(Z)
    P = np.exp(Z - l[:, None])
    idx = np.nonzero(valid)[0]
    if z_loss != 0.0:
        P = P + (2.0 * z_loss) * l[:, None] * P
    if label_smoothing != 0.0:
        P = P - label_smoothing / V
    P[idx, np.asarray(labels)[idx]] -= (1.0 - label_smoothing)
    g = np.where(valid, np.asarray(dloss, dtype=np.float64), 0.0)   # select, not multiply
    G = P * g[:, None]
    G[~valid] = 0.0
    return G


def backward(hidden_bits, weight_bits, labels, dloss, ignore_index=-100, row_block=1024,
             label_smoothing=0.0, z_loss=0.0):
    """dH [N, D] and dW [V, D] in float64 for upstream per-token gradient dloss [N]."""
    N, D, V, valid = _check(hidden_bits, weight_bits, labels, ignore_index)
    W = widen_bf16(weight_bits)
    dH = np.zeros((N, D), dtype=np.float64)
    dW = np.zeros((V, D), dtype=np.float64)
    for r0 in range(0, N, row_block):
        r1 = min(N, r0 + row_block)
        Hb = widen_bf16(hidden_bits[r0:r1])
        G = grad_logits(hidden_bits[r0:r1], weight_bits, np.asarray(labels)[r0:r1],
                        np.asarray(dloss)[r0:r1], ignore_index, label_smoothing, z_loss)
        dH[r0:r1] = G @ W
        dW += G.T @ Hb
    return dH, dW


def dweight_rows(hidden_bits, weight_bits, labels, dloss, vocab_rows, ignore_index=-100, row_block=1024,
                 label_smoothing=0.0, z_loss=0.0):
    """Rows `vocab_rows` of dW:  dW[v, :] = sum_i G[i, v] H[i, :]  (same definition as
    backward(), restricted to a few vocabulary rows so that it stays affordable at the
    benchmark's full sizes).  Every token row still sees its full-vocabulary softmax."""
    N, D, V, valid = _check(hidden_bits, weight_bits, labels, ignore_index)
    vocab_rows = np.asarray(vocab_rows, dtype=np.int64)
    out = np.zeros((vocab_rows.size, D), dtype=np.float64)
    for r0 in range(0, N, row_block):
        r1 = min(N, r0 + row_block)
        G = grad_logits(hidden_bits[r0:r1], weight_bits, np.asarray(labels)[r0:r1],
                        np.asarray(dloss)[r0:r1], ignore_index, label_smoothing, z_loss)
        out += G[:, vocab_rows].T @ widen_bf16(hidden_bits[r0:r1])
    return out


def mean_loss(loss, labels, ignore_index=-100):
    """(mean of the per-token losses over non-ignored rows, their count); mean = 0 if none."""
    valid = np.asarray(labels) != ignore_index
    n = int(valid.sum())
    return (float(np.asarray(loss, dtype=np.float64)[valid].sum() / n) if n else 0.0), n


def logit_memory_bytes(B: int, N: int, V: int, bytes_per_logit: int = 4) -> int:
    """Size of the materialised logit tensor: B x N x V x 4 bytes (memory-bottleneck
    definition at the start of the CCE section)."""
    return B * N * V * bytes_per_logit


def chunk_reduction_factor(V: int, C: int) -> float:
    """Memory reduction of chunking the vocabulary into pieces of C: V / C
    (CCE memory-reduction theorem)."""
    return V / C

"""Seeded synthetic workloads for the fused LM-head + cross-entropy path.

This module only *draws inputs*.  It contains none of the method's arithmetic
(no logits, no softmax, no gradients) so that both the CPU oracle's tests and
the GPU path can be fed from it without sharing any computation.

The paper measures on Qwen2.5-0.5B fine-tuned on an instruction dataset
(experimental-setup paragraph of the evaluation section); neither the weights
nor the data are available here, so these draws stand in for them.  They keep
the real shapes (vocabulary 151 936, hidden 896 / 2048 / 3584, batch x sequence
token counts from the paper's memory examples in the introduction and in the
Cut Cross-Entropy section), a unit-RMS hidden state as produced by a final
RMSNorm, a logit scale of about 2.5-3, Zipf-distributed labels and the padding
fractions the paper discusses for padded versus packed batches.

All tensors are returned as NumPy arrays; bf16 tensors are ``uint16`` arrays of
bit patterns (NumPy has no bfloat16 dtype).

Draw order for one workload (one ``numpy.random.default_rng(seed)`` stream):
hidden, weight, labels, ignore mask, dloss-variant noise.
"""
from __future__ import annotations

from dataclasses import dataclass, field
import numpy as np

IGNORE_INDEX = -100


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    N: int                      # tokens (batch x sequence)
    D: int                      # hidden size
    V: int                      # vocabulary size
    hidden: str = "rms"         # "iid": N(0,1) per element; "rms": rows scaled to RMS 1
    w_scale: float = 2.5        # weight std = w_scale / sqrt(D)
    labels: str = "zipf"        # "uniform" or "zipf"
    zipf_s: float = 1.1
    ignore_frac: float = 0.0
    seed: int = 0
    ignore_index: int = IGNORE_INDEX


# The five benchmark configurations (shape, distributions, padding fraction).
CONFIGS = {
    "tiny":    WorkloadSpec("tiny", 256, 64, 1000, hidden="iid", w_scale=2.5,
                            labels="uniform", ignore_frac=0.10),
    "qwen05b": WorkloadSpec("qwen05b", 8192, 896, 151936, w_scale=2.5,
                            zipf_s=1.1, ignore_frac=0.15),
    "1b":      WorkloadSpec("1b", 16384, 2048, 151936, w_scale=2.5,
                            zipf_s=1.1, ignore_frac=0.0),
    "7b":      WorkloadSpec("7b", 32768, 3584, 151936, w_scale=2.5,
                            zipf_s=1.1, ignore_frac=0.05),
    "smallv":  WorkloadSpec("smallv", 16384, 4096, 32000, w_scale=3.0,
                            zipf_s=1.3, ignore_frac=0.25),
}
CONFIG_ORDER = ["tiny", "qwen05b", "1b", "7b", "smallv"]


@dataclass
class Workload:
    spec: WorkloadSpec
    hidden: np.ndarray          # uint16 [N, D]  bf16 bit patterns
    weight: np.ndarray          # uint16 [V, D]  bf16 bit patterns
    labels: np.ndarray          # int32  [N]     ignore_index marks padding
    dloss_mean: np.ndarray      # float32 [N]    1 / N_valid everywhere
    dloss_var: np.ndarray       # float32 [N]    u_i / N_valid, NaN at ignored rows
    n_valid: int = field(default=0)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return uint16 bits.

    Inputs here are finite, so NaN quieting is not needed.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _zipf_labels(rng: np.random.Generator, n: int, V: int, s: float) -> np.ndarray:
    # p(r) ~ r^-s for rank r = 1..V; label = r - 1 (id 0 is the most frequent).
    ranks = np.arange(1, V + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** (-s))
    cdf /= cdf[-1]
    u = rng.random(n)
    lab = np.searchsorted(cdf, u, side="left")
    return np.minimum(lab, V - 1).astype(np.int32)


def make_workload(spec: WorkloadSpec) -> Workload:
    rng = np.random.default_rng(spec.seed)
    N, D, V = spec.N, spec.D, spec.V

    X = rng.standard_normal((N, D), dtype=np.float32)
    if spec.hidden == "rms":
        rms = np.sqrt(np.mean(X.astype(np.float64) ** 2, axis=1, keepdims=True))
        X = (X / rms.astype(np.float32)).astype(np.float32)
    elif spec.hidden != "iid":
        raise ValueError(f"unknown hidden recipe {spec.hidden!r}")
    hidden = f32_to_bf16_bits(X)
    del X

    # Draw W in row blocks to bound the fp32 temporary (same stream, same values
    # as one big draw because standard_normal fills in C order).
    weight = np.empty((V, D), dtype=np.uint16)
    scale = np.float32(spec.w_scale / np.sqrt(D))
    blk = max(1, (1 << 26) // max(D, 1))
    for r0 in range(0, V, blk):
        r1 = min(V, r0 + blk)
        weight[r0:r1] = f32_to_bf16_bits(rng.standard_normal((r1 - r0, D), dtype=np.float32) * scale)

    if spec.labels == "uniform":
        labels = rng.integers(0, V, size=N, dtype=np.int64).astype(np.int32)
    elif spec.labels == "zipf":
        labels = _zipf_labels(rng, N, V, spec.zipf_s)
    else:
        raise ValueError(f"unknown label recipe {spec.labels!r}")

    k = int(round(spec.ignore_frac * N))
    perm = rng.permutation(N)
    labels[perm[:k]] = spec.ignore_index
    n_valid = N - k

    inv = np.float32(1.0 / max(n_valid, 1))
    dloss_mean = np.full(N, inv, dtype=np.float32)
    u = rng.uniform(0.5, 1.5, size=N).astype(np.float32)
    dloss_var = (u * inv).astype(np.float32)
    dloss_var[labels == spec.ignore_index] = np.float32("nan")

    return Workload(spec, hidden, weight, labels, dloss_mean, dloss_var, n_valid)


def make_config(name: str) -> Workload:
    return make_workload(CONFIGS[name])


def custom_spec(N: int, D: int, V: int, *, seed: int = 0, hidden: str = "rms",
                w_scale: float = 2.5, labels: str = "zipf", zipf_s: float = 1.1,
                ignore_frac: float = 0.1, name: str | None = None) -> WorkloadSpec:
    """A workload of arbitrary shape with the same recipes (for ragged / edge tests)."""
    return WorkloadSpec(name or f"custom_{N}x{D}x{V}", N, D, V, hidden=hidden,
                        w_scale=w_scale, labels=labels, zipf_s=zipf_s,
                        ignore_frac=ignore_frac, seed=seed)

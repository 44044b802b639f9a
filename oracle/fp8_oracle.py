"""fp64 CPU oracle for the FP8 (E4M3) variant of the fused LM-head + cross-entropy path.

TEST INFRASTRUCTURE ONLY (same rules as cce_oracle.py: no code shared with the GPU path,
nothing imported from the package, never called from the product path).

What it computes, and where the paper defines it:

* E4M3 format      1 sign, 4 exponent, 3 mantissa bits, bias 7, largest finite value 448,
                   smallest subnormal 2^-9 (FP8 E4M3 format definition).  No infinities; the
                   code with all exponent and mantissa bits set is NaN.
* block quantiser  blocks of 128 consecutive elements, each with its own scale; scaled values are
                   clamped to [-448, 448] and rounded to E4M3 (block-wise E4M3 quantisation
                   algorithm).  Reading taken here: the scale is the paper's amax / 448 rounded
                   UP to a power of two, 2^e with e = ceil(log2(amax / 448)), stored as the
                   biased exponent byte e + 127 (an all-zero block gets e = 0); rounding is to
                   nearest, ties to even.  A power-of-two scale is applied exactly by the
                   block-scaled matrix instruction of the target GPU, where the paper's
                   arbitrary scale would need a rescaling of all partial sums every 128
                   elements (its FP32-promotion definition); values, clamp and block size are the
                   paper's.
* logits           Z = H^ W^T with H^, W^ the dequantised operands (code value x 2^e), exact
                   products, float64 sums (the paper's FP32-accumulation passage asks for
                   accumulation wider than the operands).
* loss, lse        as in the bf16 path, from Z.
* gradients        G = dloss (softmax(Z) - onehot) from the FP8 logits; dH = G W and dW = G^T H
                   with the bf16 master operands (reading: the paper gives no FP8 backward for
                   this product; the straight-through gradient with respect to the unquantised
                   operands is taken, so the two gradient contractions are those of the bf16
                   path).

* printed quantiser  ``quantize_blocks_printed`` is the block-wise E4M3 quantisation algorithm exactly as
                   the paper prints it -- scale = amax / 448 as a real number (float64 here), block / scale clamped to +-448 and rounded to
                   E4M3 -- with no power-of-two rounding of the scale.  The GPU path does not
                   compute it (its matrix instruction takes exponent-only scales); it exists so that
                   the distance between the reading above and the paper's own quantiser is a tested
                   number: tests bound the logit and loss differences between the two.  Readings:
                   round to nearest even (the paper does not say); an all-zero block gets scale 0 and
                   codes 0 (the printed division would be 0 / 0).

Pinned by tests/test_fp8_oracle_pins.py: the format constants the paper states, all 256 codes
round-tripping, torch's float8_e4m3fn conversion on the CPU (round to nearest even), the
quantiser's invariants and error bound, and agreement of the FP8 forward with the bf16 oracle
and torch cross_entropy on inputs that quantise without loss.
"""
from __future__ import annotations

import numpy as np

__all__ = ["BLOCK", "E4M3_MAX", "e4m3_decode", "e4m3_encode", "quantize_blocks", "dequantize",
           "logits", "forward", "backward", "quantize_blocks_printed", "dequantize_printed", "forward_from_logits"]

BLOCK = 128
E4M3_MAX = 448.0


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    """E4M3 bit patterns (uint8) -> float64 (NaN for 0x7f / 0xff)."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = (c & 7).astype(np.float64)
    sub = m * 2.0 ** -9                                   # exponent field 0: m / 8 * 2^(1 - 7)
    nor = (1.0 + m / 8.0) * np.exp2((e - 7).astype(np.float64))
    v = np.where(e == 0, sub, nor)
    v = np.where((e == 15) & ((c & 7) == 7), np.nan, v)
    return sign * v


def e4m3_encode(x: np.ndarray) -> np.ndarray:
    """float64 -> E4M3 bit patterns, round to nearest (ties to even mantissa), saturating at
    +-448.  Written from the format definition: the representable magnitudes are listed and the
    nearest one is picked."""
    x = np.asarray(x, dtype=np.float64)
    mags = e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))          # 0 .. 448, increasing
    a = np.minimum(np.abs(x), E4M3_MAX)
    hi = np.searchsorted(mags, a, side="left")                       # first magnitude >= a
    hi = np.minimum(hi, len(mags) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - mags[lo], mags[hi] - a
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))      # tie: even code = even mantissa
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    return np.where(np.signbit(x), code | 0x80, code).astype(np.uint8)


def _widen_bf16(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def quantize_blocks(x_bits: np.ndarray):
    """bf16 bit patterns [rows, D] (D a multiple of 128) -> (codes uint8 [rows, D],
    scale exponents int32 [rows, D / 128]); value = decode(code) * 2^exponent."""
    x = _widen_bf16(x_bits)
    rows, D = x.shape
    if D % BLOCK:
        raise ValueError("D must be a multiple of 128")
    xb = x.reshape(rows, D // BLOCK, BLOCK)
    amax = np.abs(xb).max(axis=2)
    with np.errstate(divide="ignore"):
        e = np.ceil(np.log2(amax / E4M3_MAX))
    e = np.where(amax == 0.0, 0.0, e)
    e = np.clip(e, -127, 127).astype(np.int32)
    scaled = np.clip(xb / np.exp2(e.astype(np.float64))[:, :, None], -E4M3_MAX, E4M3_MAX)
    return e4m3_encode(scaled).reshape(rows, D), e


def dequantize(codes: np.ndarray, exps: np.ndarray) -> np.ndarray:
    rows, D = codes.shape
    v = e4m3_decode(codes).reshape(rows, D // BLOCK, BLOCK)
    return (v * np.exp2(np.asarray(exps, dtype=np.float64))[:, :, None]).reshape(rows, D)


def logits(hq, hs, wq, ws) -> np.ndarray:
    return dequantize(hq, hs) @ dequantize(wq, ws).T


def quantize_blocks_printed(x_bits: np.ndarray):
    """The paper's block-wise E4M3 quantisation algorithm as printed: per block of 128,
    scale = amax / 448, codes = E4M3(clamp(block / scale, -448, 448)).  bf16 bit patterns
    [rows, D] -> (codes uint8 [rows, D], scales float64 [rows, D / 128]); value = decode(code) * scale.

    block / scale is formed as block * 448 / amax: the product is exact in float64 (bf16 values have
    8 significant bits), so one correctly rounded division stands for the real-number quotient and
    exact ties (e.g. block = 3/8 amax -> 168, midway between 160 and 176) stay ties."""
    x = _widen_bf16(x_bits)
    rows, D = x.shape
    if D % BLOCK:
        raise ValueError("D must be a multiple of 128")
    xb = x.reshape(rows, D // BLOCK, BLOCK)
    amax = np.abs(xb).max(axis=2)
    scale = amax / E4M3_MAX
    with np.errstate(divide="ignore", invalid="ignore"):
        scaled = np.where(amax[:, :, None] > 0.0, xb * E4M3_MAX / amax[:, :, None], 0.0)
    scaled = np.clip(scaled, -E4M3_MAX, E4M3_MAX)
    return e4m3_encode(scaled).reshape(rows, D), scale


def dequantize_printed(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    rows, D = codes.shape
    v = e4m3_decode(codes).reshape(rows, D // BLOCK, BLOCK)
    return (v * np.asarray(scales, dtype=np.float64)[:, :, None]).reshape(rows, D)


def forward_from_logits(Z, labels, ignore_index=-100):
    """loss = lse - z_label and lse (float64) of materialised logits; ignored rows give 0, 0."""
    labels = np.asarray(labels, dtype=np.int64)
    valid = labels != ignore_index
    m = Z.max(axis=1)
    lse_all = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
    idx = np.nonzero(valid)[0]
    loss = np.zeros(len(labels))
    lse = np.zeros(len(labels))
    lse[idx] = lse_all[idx]
    loss[idx] = lse_all[idx] - Z[idx, labels[idx]]
    return loss, lse


def forward(hq, hs, wq, ws, labels, ignore_index=-100):
    """Per-token loss and log-sum-exp (float64) from the FP8 logits; ignored rows give 0, 0."""
    labels = np.asarray(labels, dtype=np.int64)
    Z = logits(hq, hs, wq, ws)
    V = Z.shape[1]
    if np.any((labels != ignore_index) & ((labels < 0) | (labels >= V))):
        raise ValueError("label outside [0, V)")
    valid = labels != ignore_index
    m = Z.max(axis=1)
    lse_all = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
    idx = np.nonzero(valid)[0]
    loss = np.zeros(len(labels))
    lse = np.zeros(len(labels))
    lse[idx] = lse_all[idx]
    loss[idx] = lse_all[idx] - Z[idx, labels[idx]]
    return loss, lse


def backward(hq, hs, wq, ws, hidden_bits, weight_bits, labels, dloss, ignore_index=-100):
    """(dH [N, D], dW [V, D]) in float64: gradient tiles from the FP8 logits, contracted with
    the bf16 master operands."""
    labels = np.asarray(labels, dtype=np.int64)
    Z = logits(hq, hs, wq, ws)
    valid = labels != ignore_index
    m = Z.max(axis=1)
    lse = m + np.log(np.exp(Z - m[:, None]).sum(axis=1))
    G = np.exp(Z - lse[:, None])
    idx = np.nonzero(valid)[0]
    G[idx, labels[idx]] -= 1.0
    g = np.where(valid, np.asarray(dloss, dtype=np.float64), 0.0)
    G = G * g[:, None]
    G[~valid] = 0.0
    return G @ _widen_bf16(weight_bits), G.T @ _widen_bf16(hidden_bits)

"""Pins of oracle/fp8_oracle.py (CPU)."""
import numpy as np
import pytest
import torch

from oracle import cce_oracle as O
from oracle import fp8_oracle as F
from paper_2601_02609_amd import inputs as I


def test_format_constants_the_paper_states():
    """FP8 E4M3 format definition: 1-4-3 bits, bias 7, range +-448, smallest subnormal 2^-9."""
    allc = np.arange(256, dtype=np.uint8)
    v = F.e4m3_decode(allc)
    finite = v[np.isfinite(v)]
    assert finite.max() == 448.0 and finite.min() == -448.0
    assert np.min(np.abs(finite[finite != 0])) == 2.0 ** -9
    assert F.e4m3_decode(np.array([0x38], dtype=np.uint8))[0] == 1.0          # exponent field 7 = bias
    assert F.e4m3_decode(np.array([0x7E], dtype=np.uint8))[0] == 448.0
    assert np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.isfinite(v).sum() == 254
    assert 448.0 / 2 ** 3 == 56.0 and F.e4m3_decode(np.array([0x08], dtype=np.uint8))[0] == 2.0 ** -6   # smallest normal


def test_every_finite_code_round_trips():
    allc = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    back = F.e4m3_encode(F.e4m3_decode(allc))
    assert np.array_equal(back & 0x7F, allc & 0x7F)
    nz = (allc & 0x7F) != 0
    assert np.array_equal(back[nz], allc[nz])


def test_encode_matches_torch_float8_cast_in_range():
    """torch's CPU cast to float8_e4m3fn rounds to nearest even; compared on random values, on
    every midpoint between neighbouring codes, and just beside them."""
    rng = np.random.default_rng(0)
    mags = F.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
    mids = (mags[:-1] + mags[1:]) / 2
    x = np.concatenate([rng.uniform(-448, 448, 20000), rng.standard_normal(20000) * 0.01,
                        mids, -mids, np.nextafter(mids, 0), np.nextafter(mids, 1e9), mags, [0.0]])
    x = x.astype(np.float32).astype(np.float64)                     # torch casts from fp32
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = F.e4m3_encode(x)
    zero = x == 0
    assert np.array_equal(got[~zero], ref[~zero])
    assert np.all((got[zero] & 0x7F) == 0)


def test_encode_saturates():
    assert np.array_equal(F.e4m3_encode(np.array([1e9, -1e9, 449.0, 464.0])), np.array([0x7E, 0xFE, 0x7E, 0x7E], dtype=np.uint8))


def test_quantiser_invariants_and_error_bound():
    w = I.make_workload(I.custom_spec(50, 384, 70, seed=3))
    for bits in (w.hidden, w.weight):
        codes, e = F.quantize_blocks(bits)
        x = F._widen_bf16(bits)
        xb = x.reshape(x.shape[0], -1, 128)
        amax = np.abs(xb).max(axis=2)
        scale = np.exp2(e.astype(np.float64))
        # the scale is the smallest power of two that keeps the block within +-448
        assert np.all(amax / scale <= 448.0) and np.all(amax / scale > 224.0)
        assert not np.any((codes & 0x7F) == 0x7F)
        err = np.abs(F.dequantize(codes, e) - x).reshape(xb.shape)
        # half a unit in the last place: 2^-4 relative for normal results, 2^-10 scale for subnormal ones
        bound = np.maximum(np.abs(xb) * 2.0 ** -4, scale[:, :, None] * 2.0 ** -10)
        assert np.all(err <= bound)
        # power-of-two scale: at most twice the error of the paper's amax / 448 scale (its
        # error proposition is stated for that scale)
        assert np.all(err <= 2 * np.maximum(np.abs(xb) * 2.0 ** -4, (amax / 448.0)[:, :, None] * 2.0 ** -10) + 1e-300)


def test_zero_block_and_exact_powers():
    bits = np.zeros((2, 256), dtype=np.uint16)
    bits[1, 128:] = 0x3F80                     # 1.0 in bf16: amax / 448 = 2^-8.8 -> e = -8, code for 256 = 0x78
    codes, e = F.quantize_blocks(bits)
    assert np.all(codes[0] == 0) and np.all(e[0] == 0) and e[1, 0] == 0 and e[1, 1] == -8
    assert np.all(codes[1, 128:] == 0x78) and np.all(F.dequantize(codes, e)[1, 128:] == 1.0)
    bits[1, 128] = I.f32_to_bf16_bits(np.array([448.0], dtype=np.float32))[0]     # amax = 448 exactly: e = 0
    codes, e = F.quantize_blocks(bits)
    assert e[1, 1] == 0 and codes[1, 128] == 0x7E and codes[1, 129] == 0x38


def _lossless_workload(seed, N=40, D=256, V=90):
    """bf16 inputs that the block quantiser represents exactly: E4M3 values times a power of
    two per block, with one element of magnitude 448 x 2^e in every block."""
    rng = np.random.default_rng(seed)
    def make(rows, spread):
        codes = rng.integers(0, 0x7F, size=(rows, D), dtype=np.int64).astype(np.uint8)
        codes = np.where((codes & 0x78) < 0x28, codes | 0x28, codes)         # keep 3+ exponent steps above subnormals
        codes |= (rng.integers(0, 2, size=codes.shape, dtype=np.int64).astype(np.uint8) << 7)
        e = rng.integers(-12, -12 + spread, size=(rows, D // 128))
        codes.reshape(rows, -1, 128)[:, :, 0] = 0x7E
        v = F.e4m3_decode(codes).reshape(rows, -1, 128) * np.exp2(e.astype(np.float64))[:, :, None]
        bits = I.f32_to_bf16_bits(v.reshape(rows, D).astype(np.float32))
        assert np.array_equal(F._widen_bf16(bits), v.reshape(rows, D))      # 4 significant bits fit bf16
        return bits
    H, W = make(N, 3), make(V, 3)
    labels = rng.integers(0, V, size=N).astype(np.int32)
    labels[::7] = -100
    return H, W, labels


def test_fp8_path_equals_bf16_oracle_and_torch_on_lossless_inputs():
    H, W, labels = _lossless_workload(4)
    hq, hs = F.quantize_blocks(H)
    wq, ws = F.quantize_blocks(W)
    assert np.array_equal(F.dequantize(hq, hs), F._widen_bf16(H))
    loss, lse = F.forward(hq, hs, wq, ws, labels)
    o_loss, o_lse = O.forward(H, W, labels)
    np.testing.assert_allclose(loss, o_loss, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(lse, o_lse, rtol=1e-12, atol=1e-12)
    Z = torch.from_numpy(F._widen_bf16(H)) @ torch.from_numpy(F._widen_bf16(W)).T
    ref = torch.nn.functional.cross_entropy(Z, torch.from_numpy(labels.astype(np.int64)), ignore_index=-100, reduction="none")
    np.testing.assert_allclose(loss, ref.numpy(), rtol=1e-12, atol=1e-12)
    dloss = np.random.default_rng(1).standard_normal(len(labels))
    dH, dW = F.backward(hq, hs, wq, ws, H, W, labels, dloss)
    o_dH, o_dW = O.backward(H, W, labels, dloss)
    np.testing.assert_allclose(dH, o_dH, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(dW, o_dW, rtol=1e-10, atol=1e-14)


def test_fp8_logits_stay_close_to_bf16_logits_on_the_workload_recipe():
    """On the synthetic recipe the FP8 logits differ from the bf16 ones by quantisation noise of
    the expected size (relative step 2^-4 per element, averaged over D terms), not more."""
    w = I.make_workload(I.custom_spec(64, 896, 300, seed=6))
    hq, hs = F.quantize_blocks(w.hidden)
    wq, ws = F.quantize_blocks(w.weight)
    Zq = F.logits(hq, hs, wq, ws)
    Z = O.logits(w.hidden, w.weight)
    rel = np.linalg.norm(Zq - Z) / np.linalg.norm(Z)
    assert 1e-3 < rel < 6e-2


# ---------------------------------------------------------------------------------------------
# The paper's quantiser as printed (scale = amax / 448), and how far the power-of-two-scale
# reading that the GPU path implements lies from it.
# ---------------------------------------------------------------------------------------------
def test_printed_quantiser_invariants():
    """Block-wise E4M3 quantisation algorithm: with scale = amax / 448 the largest element of every
    block maps to the code of +-448 exactly, all codes are finite, an all-zero block stays zero, and
    the reconstruction error is at most half a unit in the last place of the scaled value."""
    w = I.make_workload(I.custom_spec(50, 384, 70, seed=3))
    for bits in (w.hidden, w.weight):
        codes, scale = F.quantize_blocks_printed(bits)
        assert scale.dtype == np.float64 and codes.dtype == np.uint8
        x = F._widen_bf16(bits)
        xb = x.reshape(x.shape[0], -1, 128)
        amax = np.abs(xb).max(axis=2)
        assert np.array_equal(scale, amax / 448.0)
        cb = codes.reshape(xb.shape)
        at_max = np.abs(xb) == amax[:, :, None]
        assert np.all((cb[at_max] & 0x7F) == 0x7E)                   # +-448
        assert not np.any((codes & 0x7F) == 0x7F)
        err = np.abs(F.dequantize_printed(codes, scale) - x).reshape(xb.shape)
        s = scale.astype(np.float64)[:, :, None]
        # 2^-4 relative for normal results, half of 2^-9 scaled units for subnormal ones (plus the
        # float64 rounding of the quotient and of the product with the scale)
        assert np.all(err <= np.maximum(np.abs(xb) * (2.0 ** -4 + 2.0 ** -50), s * 2.0 ** -10))
    zero = np.zeros((1, 128), dtype=np.uint16)
    c0, s0 = F.quantize_blocks_printed(zero)
    assert np.all(c0 == 0) and s0[0, 0] == 0.0 and np.all(F.dequantize_printed(c0, s0) == 0.0)


def test_printed_quantiser_matches_torch_float8_cast():
    """The same algorithm with library pieces: block * 448 / amax, clamp, cast to
    torch.float8_e4m3fn (round to nearest even; torch casts from fp32, and the quotients of bf16
    values by a bf16 amax that lie on or near a rounding boundary survive the fp32 step unchanged on
    these inputs)."""
    w = I.make_workload(I.custom_spec(64, 512, 90, seed=11))
    for bits in (w.hidden, w.weight):
        codes, scale = F.quantize_blocks_printed(bits)
        x = torch.from_numpy(F._widen_bf16(bits)).reshape(bits.shape[0], -1, 128)
        amax = x.abs().amax(dim=2, keepdim=True)
        ref = (x * 448.0 / amax).clamp(-448.0, 448.0).to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        got = codes.reshape(ref.shape)
        nz = (got & 0x7F) != 0                                         # signed zero aside
        assert np.array_equal(got[nz], ref[nz]) and np.all((ref[~nz] & 0x7F) == 0)
        # the exact ties the recipe produces (block = 3/8, 3/16, ... of amax) go to the even code
        q = (x * 448.0 / amax).numpy()
        mags = F.e4m3_decode(np.arange(0, 0x7F, dtype=np.uint8))
        mids = (mags[:-1] + mags[1:]) / 2
        tie = np.isin(np.abs(q), mids)
        assert tie.sum() > 0 and np.all((got[tie] & 1) == 0)


def test_printed_scale_on_lossless_inputs_equals_power_of_two_scale():
    """Where every block's amax is 448 x 2^e both rules give the same scale, hence the same codes
    and the same logits."""
    H, W, labels = _lossless_workload(5)
    cp, sp = F.quantize_blocks_printed(H)
    c2, e2 = F.quantize_blocks(H)
    assert np.array_equal(cp, c2) and np.array_equal(sp.astype(np.float64), np.exp2(e2.astype(np.float64)))


@pytest.mark.parametrize("spec", [(192, 896, 4096, 6), (128, 2048, 3000, 7), (96, 4096, 2000, 8)])
def test_distance_between_power_of_two_and_printed_quantiser(spec):
    """What the power-of-two scale costs against the paper's amax / 448, on the workload recipe.

    Expected from the format: an E4M3 value carries a relative rounding error of about 2.7 % rms
    (step 2^-3 relative, uniform error, averaged over the mantissa); a product of two about 3.8 %; a
    logit -- D such products with independent errors -- the same 3.8 % of the logit scale, whichever
    scale rule is used.  The power-of-two rule leaves the block maximum in (224, 448] instead of at
    448, which pushes a few more elements into the next-coarser binade: a few percent more error, not
    a factor.  Two quantisations with independent errors then differ by about sqrt(2) x 3.8 % = 5.3 %
    of the logit norm, and a per-token loss by a few tenths at most (logit scale 2.5-3)."""
    N, D, V, seed = spec
    w = I.make_workload(I.custom_spec(N, D, V, seed=seed, ignore_frac=0.15))
    Zp2 = F.logits(*F.quantize_blocks(w.hidden), *F.quantize_blocks(w.weight))
    Zpr = F.dequantize_printed(*F.quantize_blocks_printed(w.hidden)) @ F.dequantize_printed(*F.quantize_blocks_printed(w.weight)).T
    Z = O.logits(w.hidden, w.weight)
    rel = lambda a, b: float(np.linalg.norm(a - b) / np.linalg.norm(b))
    d_pair, e_p2, e_pr = rel(Zp2, Zpr), rel(Zp2, Z), rel(Zpr, Z)
    print(f"[fp8 distance] D={D}: relF(pow2 - printed)={d_pair:.4f}  relF(pow2 - bf16)={e_p2:.4f}  relF(printed - bf16)={e_pr:.4f}")
    assert 0.03 < d_pair < 0.07
    assert e_pr < 0.05 and e_p2 < 0.05 and e_p2 < 1.10 * e_pr          # the reading costs < 10 % more error
    l2, s2 = F.forward_from_logits(Zp2, w.labels)
    lp, sp = F.forward_from_logits(Zpr, w.labels)
    valid = w.labels != -100
    d = np.abs(l2 - lp)[valid]
    print(f"[fp8 distance] per-token loss |pow2 - printed|: mean {d.mean():.3f} max {d.max():.3f}; "
          f"mean loss {l2[valid].mean():.4f} vs {lp[valid].mean():.4f}; max |lse diff| {np.abs(s2 - sp).max():.3f}")
    assert d.mean() < 0.16 and d.max() < 0.8 and np.abs(s2 - sp).max() < 0.4
    assert abs(l2[valid].mean() - lp[valid].mean()) < 0.05
    assert np.all(l2[~valid] == 0) and np.all(lp[~valid] == 0)

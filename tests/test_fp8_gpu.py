"""GPU parity of the FP8 (E4M3, block-128 power-of-two scales) variant against oracle/fp8_oracle.py.

Quantisation is byte work: codes and scale bytes must be identical to the oracle's.  The
forward / backward then start from the SAME codes on both sides, so what is compared is the
arithmetic after the quantiser: exact E4M3 products (fp64 sums in the oracle; in the MFMA, fp32
accumulation of 64-term groups whose internal sum keeps about 13 bits below its largest product
-- measured with random codes) -- to the tolerances of the bf16 path: loss / lse 2e-3 absolute,
gradients 1e-2 relative Frobenius.
"""
import numpy as np
import pytest
import torch

from oracle import fp8_oracle as F
from paper_2601_02609_amd import inputs as I
from tests.gpu_util import LOSS_ATOL, GRAD_RTOL, bf16_dev, bf16_host, dev_inputs, rel_fro

pytestmark = pytest.mark.gpu
IGN = -100


@pytest.fixture(scope="module")
def B():
    from paper_2601_02609_amd import binding
    binding.lib()
    return binding


def scales_to_rows(scales: np.ndarray, rows: int, D: int) -> np.ndarray:
    """Grouped device layout [D/128][groups][32][4] -> exponent bytes [rows, D/128]."""
    kb, groups = D // 128, (rows + 127) // 128
    s = scales.reshape(kb, groups, 32, 4)
    r = np.arange(rows)
    return s[:, r >> 7, r & 31, (r >> 5) & 3].T.copy()


def quantize_dev(B, bits):
    x = bf16_dev(bits)
    q, sc = B.cce_quantize_e4m3(x)
    torch.cuda.synchronize()
    return x, q, sc


@pytest.mark.parametrize("rows,D", [(1, 128), (130, 256), (300, 896), (257, 1024)])
def test_quantiser_is_bit_exact(B, rows, D):
    w = I.make_workload(I.custom_spec(rows, D, 8, seed=41))
    bits = w.hidden.copy()
    # exercise zeros, an all-zero block, exact powers and a wide range of block magnitudes
    bits[0, :5] = 0
    if rows > 2:
        bits[1, :128] = 0
        f = I.bf16_bits_to_f32(bits[2])
        bits[2] = I.f32_to_bf16_bits((f * np.exp2(np.repeat(np.arange(D // 128) * 5 - 12, 128))).astype(np.float32))
    bits[0, 7] = I.f32_to_bf16_bits(np.array([448.0], dtype=np.float32))[0]
    _, q, sc = quantize_dev(B, bits)
    o_codes, o_exp = F.quantize_blocks(bits)
    g_codes = q.cpu().numpy()
    g_all = sc.cpu().numpy()
    g_exp = scales_to_rows(g_all, rows, D).astype(np.int32) - 127
    assert np.array_equal(g_exp, o_exp)
    # -0 and +0 are the same value; everything else must be the same byte
    same = (g_codes == o_codes) | (((g_codes | o_codes) & 0x7F) == 0)
    assert np.all(same), f"{(~same).sum()} codes differ"
    # rows past the matrix in the last group hold 127
    groups = (rows + 127) // 128
    full = g_all.reshape(D // 128, groups, 32, 4)
    r = np.arange(rows, groups * 128)
    assert np.all(full[:, r >> 7, r & 31, (r >> 5) & 3] == 127)


def run_fp8(B, w):
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    hq, hs = B.cce_quantize_e4m3(H)
    wq, wsc = B.cce_quantize_e4m3(W)
    ws = B.alloc_workspace(N, D, V)
    loss, lse = B.cce_fp8_forward(hq, hs, wq, wsc, y, IGN, workspace=ws)
    dl = torch.from_numpy(np.nan_to_num(w.dloss_var, nan=0.0)).cuda()
    dH, dW = B.cce_fp8_backward(hq, hs, wq, wsc, H, W, y, lse, dl, IGN, workspace=ws)
    torch.cuda.synchronize()
    assert B.read_status(ws) == 0
    return (loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
            bf16_host(dH), dW.cpu().numpy().astype(np.float64))


@pytest.mark.parametrize("shape", [(300, 128, 700), (700, 896, 3000), (513, 1024, 1100), (256, 256, 256)])
def test_fp8_forward_backward_match_oracle(B, shape):
    N, D, V = shape
    w = I.make_workload(I.custom_spec(N, D, V, seed=42, ignore_frac=0.15))
    print(f"[fp8] N={N} D={D} V={V}", flush=True)
    loss, lse, dH, dW = run_fp8(B, w)
    hq, hs = F.quantize_blocks(w.hidden)
    wq, wsx = F.quantize_blocks(w.weight)
    o_loss, o_lse = F.forward(hq, hs, wq, wsx, w.labels, IGN)
    dl = np.nan_to_num(w.dloss_var, nan=0.0)
    o_dH, o_dW = F.backward(hq, hs, wq, wsx, w.hidden, w.weight, w.labels, dl, IGN)
    ign = w.labels == IGN
    assert np.all(loss[ign] == 0.0) and np.all(lse[ign] == 0.0) and np.all(dH[ign] == 0.0)
    e = (np.abs(loss - o_loss).max(), np.abs(lse - o_lse).max(), rel_fro(dH, o_dH), rel_fro(dW, o_dW))
    print(f"[fp8] max|dloss|={e[0]:.2e} max|dlse|={e[1]:.2e} relF(dH)={e[2]:.2e} relF(dW)={e[3]:.2e}", flush=True)
    assert e[0] <= LOSS_ATOL and e[1] <= LOSS_ATOL and e[2] <= GRAD_RTOL and e[3] <= GRAD_RTOL


# Distance of the GPU variant from the paper's OWN quantiser (scale = amax / 448, printed in its
# block-wise E4M3 quantisation algorithm), which the GPU does not compute (its matrix instruction
# takes power-of-two scales).  Expected from the format (derivation in
# tests/test_fp8_oracle_pins.py::test_distance_between_power_of_two_and_printed_quantiser): both
# quantisers put about 3.8 % rms noise on a logit, independently, so per-token loss and lse differ
# by a few tenths at most and by ~0.11 on average at logit scale 2.5; the means over tokens agree
# to a few hundredths.
PRINTED_LOSS_MAX, PRINTED_LOSS_MEAN, PRINTED_LSE_MAX, PRINTED_MEAN_LOSS = 0.8, 0.16, 0.4, 0.05


@pytest.mark.parametrize("shape", [(700, 896, 3000), (384, 2048, 2500)])
def test_fp8_gpu_against_the_printed_scale_quantiser(B, shape):
    N, D, V = shape
    w = I.make_workload(I.custom_spec(N, D, V, seed=44, ignore_frac=0.15))
    loss, lse, dH, dW = run_fp8(B, w)
    Zpr = F.dequantize_printed(*F.quantize_blocks_printed(w.hidden)) @ F.dequantize_printed(*F.quantize_blocks_printed(w.weight)).T
    p_loss, p_lse = F.forward_from_logits(Zpr, w.labels, IGN)
    hq, hs = F.quantize_blocks(w.hidden)
    wq, wsx = F.quantize_blocks(w.weight)
    o_loss, o_lse = F.forward(hq, hs, wq, wsx, w.labels, IGN)
    valid = w.labels != IGN
    d = np.abs(loss - p_loss)[valid]
    d_lse = np.abs(lse - p_lse)[valid]
    d_mean = abs(loss[valid].mean() - p_loss[valid].mean())
    print(f"[fp8] N={N} D={D} V={V}: GPU vs power-of-two-scale oracle max|dloss|={np.abs(loss - o_loss).max():.2e}; "
          f"GPU vs printed-scale oracle |dloss| mean {d.mean():.3f} max {d.max():.3f}, max|dlse| {d_lse.max():.3f}, "
          f"mean loss {loss[valid].mean():.4f} vs {p_loss[valid].mean():.4f}", flush=True)
    assert np.abs(loss - o_loss).max() <= LOSS_ATOL and np.abs(lse - o_lse).max() <= LOSS_ATOL
    assert d.max() <= PRINTED_LOSS_MAX and d.mean() <= PRINTED_LOSS_MEAN
    assert d_lse.max() <= PRINTED_LSE_MAX and d_mean <= PRINTED_MEAN_LOSS
    assert np.all(loss[~valid] == 0.0) and np.all(p_loss[~valid] == 0.0)


def test_fp8_uses_the_block_scales(B):
    """Blocks of very different magnitude along K and along the rows: a result that ignored or
    misplaced a scale byte would be off by powers of two."""
    N, D, V = 260, 512, 390
    w = I.make_workload(I.custom_spec(N, D, V, seed=43, ignore_frac=0.0))
    rng = np.random.default_rng(3)
    def rescale(bits, lo, hi):
        f = I.bf16_bits_to_f32(bits)
        e = rng.integers(lo, hi, size=(bits.shape[0], D // 128))
        return I.f32_to_bf16_bits((f * np.exp2(np.repeat(e, 128, axis=1)).astype(np.float32)).astype(np.float32))
    w.hidden[:] = rescale(w.hidden, -3, 4)
    w.weight[:] = rescale(w.weight, -3, 4)
    loss, lse, dH, dW = run_fp8(B, w)
    hq, hs = F.quantize_blocks(w.hidden)
    wq, wsx = F.quantize_blocks(w.weight)
    assert len(np.unique(hs)) >= 5 and len(np.unique(wsx)) >= 5
    o_loss, o_lse = F.forward(hq, hs, wq, wsx, w.labels, IGN)
    assert np.abs(lse - o_lse).max() <= LOSS_ATOL * max(1.0, np.abs(o_lse).max() / 10)
    assert np.abs(loss - o_loss).max() <= LOSS_ATOL * max(1.0, np.abs(o_lse).max() / 10)


def test_fp8_argument_errors(B):
    w = I.make_workload(I.custom_spec(64, 192, 100, seed=9))
    H, W, y = dev_inputs(w)
    with pytest.raises(B.CCEError):
        B.cce_quantize_e4m3(H)                      # D not a multiple of 128
    assert B.fp8_scale_bytes(64, 192) == 0 and B.fp8_scale_bytes(300, 896) == 7 * 3 * 128


def test_fp8_at_the_headline_shape_sampled(B):
    """N=8192, D=896, V=151936: quantised codes of sampled rows bit-exact; loss / lse / dHidden on a
    seeded sample of rows and dW on sampled vocabulary rows against the oracle."""
    w = I.make_config("qwen05b")
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    H, W, y = dev_inputs(w)
    hq, hs = B.cce_quantize_e4m3(H)
    wq, wsc = B.cce_quantize_e4m3(W)
    ws = B.alloc_workspace(N, D, V)
    loss, lse = B.cce_fp8_forward(hq, hs, wq, wsc, y, IGN, workspace=ws)
    rng = np.random.default_rng(13)
    rows = np.unique(np.concatenate([[0, N - 1, 255, 256], rng.choice(N, 20, replace=False)])).astype(np.int64)
    dl_np = np.zeros(N, dtype=np.float32)
    dl_np[rows] = 1.0 / w.n_valid
    dH, dW = B.cce_fp8_backward(hq, hs, wq, wsc, H, W, y, lse, torch.from_numpy(dl_np).cuda(), IGN, workspace=ws)
    torch.cuda.synchronize()
    assert B.read_status(ws) == 0
    print(f"[fp8] headline shape: oracle on {rows.size} rows", flush=True)
    o_wq, o_ws = F.quantize_blocks(w.weight)
    assert np.array_equal(scales_to_rows(wsc.cpu().numpy(), V, D).astype(np.int32) - 127, o_ws)
    g_wq = wq.cpu().numpy()
    assert np.all((g_wq == o_wq) | (((g_wq | o_wq) & 0x7F) == 0))
    o_hq, o_hs = F.quantize_blocks(w.hidden[rows])
    o_loss, o_lse = F.forward(o_hq, o_hs, o_wq, o_ws, w.labels[rows], IGN)
    g_loss, g_lse = loss.cpu().numpy().astype(np.float64)[rows], lse.cpu().numpy().astype(np.float64)[rows]
    assert np.abs(g_loss - o_loss).max() <= LOSS_ATOL and np.abs(g_lse - o_lse).max() <= LOSS_ATOL
    o_dH, o_dW = F.backward(o_hq, o_hs, o_wq, o_ws, w.hidden[rows], w.weight, w.labels[rows], dl_np[rows], IGN)
    assert rel_fro(bf16_host(dH[torch.from_numpy(rows).cuda()]), o_dH) <= GRAD_RTOL
    vrows = np.unique(np.concatenate([w.labels[rows][w.labels[rows] >= 0], rng.choice(V, 200, replace=False)]))
    g_dW = dW[torch.from_numpy(vrows).cuda()].cpu().numpy().astype(np.float64)
    assert rel_fro(g_dW, o_dW[vrows]) <= GRAD_RTOL

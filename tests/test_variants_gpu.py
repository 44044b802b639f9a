"""GPU parity of the loss variants (label smoothing, z-loss, mean reduction) against the oracle.

Same tolerances as the plain path: per-token loss and lse within 2e-3 absolute, dHidden and dW
within 1e-2 relative Frobenius error, ignored rows exactly 0.
"""
import numpy as np
import pytest
import torch

from oracle import cce_oracle as O
from paper_2601_02609_amd import inputs as I
from tests.gpu_util import LOSS_ATOL, GRAD_RTOL, bf16_host, dev_inputs, rel_fro

pytestmark = pytest.mark.gpu
IGN = -100


@pytest.fixture(scope="module")
def B():
    from paper_2601_02609_amd import binding
    binding.lib()
    return binding


def run_variant(B, w, dloss_np, eps, lam, want_mean=False, grad_scale=1.0):
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    ws = B.alloc_workspace(N, D, V)
    loss, lse, mean = B.cce_forward_ex(H, W, y, IGN, label_smoothing=eps, z_loss=lam, want_mean=want_mean, workspace=ws)
    dl = torch.from_numpy(dloss_np).cuda() if dloss_np is not None else None
    dH, dW = B.cce_backward_ex(H, W, y, lse, dl, IGN, grad_scale=grad_scale, label_smoothing=eps, z_loss=lam, workspace=ws)
    torch.cuda.synchronize()
    assert B.read_status(ws) == 0
    return (loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
            bf16_host(dH), dW.cpu().numpy().astype(np.float64), None if mean is None else float(mean.item()))


@pytest.mark.parametrize("eps,lam", [(0.1, 0.0), (0.0, 1e-3), (0.2, 1e-4)])
@pytest.mark.parametrize("shape", [(700, 128, 3000), (513, 896, 1100)])
def test_variants_match_oracle(B, shape, eps, lam):
    N, D, V = shape
    w = I.make_workload(I.custom_spec(N, D, V, seed=21, ignore_frac=0.2))
    print(f"[variants] N={N} D={D} V={V} eps={eps} lambda={lam}", flush=True)
    loss, lse, dH, dW, _ = run_variant(B, w, w.dloss_var, eps, lam)
    o_loss, o_lse = O.forward(w.hidden, w.weight, w.labels, IGN, label_smoothing=eps, z_loss=lam)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, w.dloss_var, IGN, label_smoothing=eps, z_loss=lam)
    ign = w.labels == IGN
    assert np.all(loss[ign] == 0.0) and np.all(lse[ign] == 0.0) and np.all(dH[ign] == 0.0)
    e = (np.abs(loss - o_loss).max(), np.abs(lse - o_lse).max(), rel_fro(dH, o_dH), rel_fro(dW, o_dW))
    print(f"[variants] max|dloss|={e[0]:.2e} max|dlse|={e[1]:.2e} relF(dH)={e[2]:.2e} relF(dW)={e[3]:.2e}", flush=True)
    assert e[0] <= LOSS_ATOL and e[1] <= LOSS_ATOL and e[2] <= GRAD_RTOL and e[3] <= GRAD_RTOL
    # the variants change the loss, so the comparison above is not vacuous
    p_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN)
    assert np.abs(o_loss - p_loss).max() > 10 * LOSS_ATOL


def test_mean_reduction(B):
    """dloss = NULL: every valid row gets grad_scale / n_valid; mean_loss is the oracle's mean."""
    w = I.make_workload(I.custom_spec(700, 128, 3000, seed=22, ignore_frac=0.3))
    loss, lse, dH, dW, mean = run_variant(B, w, None, 0.0, 0.0, want_mean=True, grad_scale=2.0)
    o_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN)
    o_mean, n = O.mean_loss(o_loss, w.labels, IGN)
    assert n == w.n_valid and abs(mean - o_mean) <= LOSS_ATOL
    dl = np.full(700, 2.0 / n, dtype=np.float32)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, dl, IGN)
    assert rel_fro(dH, o_dH) <= GRAD_RTOL and rel_fro(dW, o_dW) <= GRAD_RTOL
    # identical (bit for bit) to passing that dloss explicitly
    _, _, dH2, dW2, _ = run_variant(B, w, dl, 0.0, 0.0)
    assert np.array_equal(dH, dH2) and np.array_equal(dW, dW2)


def test_mean_reduction_with_no_valid_rows(B):
    w = I.make_workload(I.custom_spec(300, 64, 500, seed=23, ignore_frac=1.0))
    loss, lse, dH, dW, mean = run_variant(B, w, None, 0.1, 1e-3, want_mean=True)
    assert mean == 0.0 and np.all(loss == 0) and np.all(dH == 0) and np.all(dW == 0)


def test_zero_weight_closed_form(B):
    """W = 0: loss = ln V + lambda ln^2 V for any eps (closed form of the variant definitions)."""
    import math
    w = I.make_workload(I.custom_spec(130, 64, 1000, seed=24, ignore_frac=0.1))
    w.weight[:] = 0
    loss, lse, dH, dW, _ = run_variant(B, w, w.dloss_mean, 0.25, 0.05)
    valid = w.labels != IGN
    lnV = math.log(1000)
    assert np.abs(loss[valid] - (lnV + 0.05 * lnV * lnV)).max() <= 1e-3
    assert np.all(dH == 0.0)


def test_variant_argument_errors(B):
    w = I.make_workload(I.custom_spec(64, 64, 100, seed=9))
    H, W, y = dev_inputs(w)
    for eps, lam in [(-0.1, 0.0), (1.0, 0.0), (0.0, -1.0), (0.0, float("nan"))]:
        with pytest.raises(B.CCEError):
            B.cce_forward_ex(H, W, y, IGN, label_smoothing=eps, z_loss=lam)


def test_variants_at_the_headline_shape_sampled(B):
    """Label smoothing + z-loss + mean reduction at N=8192, D=896, V=151936: loss / lse / dHidden on a
    seeded sample of rows (each needs only its own row and the full vocabulary), the mean over all
    rows from the oracle's closed relation to the plain loss on that sample, and the row-sum
    property of the smoothed gradient on all of dW."""
    w = I.make_config("qwen05b")
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    eps, lam = 0.1, 1e-4
    H, W, y = dev_inputs(w)
    ws = B.alloc_workspace(N, D, V)
    loss, lse, mean = B.cce_forward_ex(H, W, y, IGN, label_smoothing=eps, z_loss=lam, want_mean=True, workspace=ws)
    dH, dW = B.cce_backward_ex(H, W, y, lse, None, IGN, grad_scale=1.0, label_smoothing=eps, z_loss=lam, workspace=ws)
    torch.cuda.synchronize()
    g_loss, g_lse = loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, N - 1, 255, 256], rng.choice(N, 28, replace=False)])).astype(np.int64)
    print(f"[variants] headline shape: oracle on {rows.size} rows", flush=True)
    o_loss, o_lse = O.forward(w.hidden[rows], w.weight, w.labels[rows], IGN, label_smoothing=eps, z_loss=lam)
    dl = np.full(rows.size, 1.0 / w.n_valid, dtype=np.float32)
    o_dH, _ = O.backward(w.hidden[rows], w.weight, w.labels[rows], dl, IGN, label_smoothing=eps, z_loss=lam)
    assert np.abs(g_loss[rows] - o_loss).max() <= LOSS_ATOL and np.abs(g_lse[rows] - o_lse).max() <= LOSS_ATOL
    assert rel_fro(bf16_host(dH[torch.from_numpy(rows).cuda()]), o_dH) <= GRAD_RTOL
    # the in-library mean is the mean of the per-token losses it returned
    assert abs(float(mean.item()) - g_loss.sum() / w.n_valid) <= 1e-4
    # rows of the smoothed gradient sum to 2 lambda lse_i dloss_i (zero without the z-loss), hence
    # sum_v dW[v, :] = sum_i 2 lambda lse_i / n_valid * h_i
    Hf = I.bf16_bits_to_f32(w.hidden).astype(np.float64)
    want = (2 * lam * g_lse[:, None] / w.n_valid * Hf).sum(axis=0)
    got = dW.double().sum(dim=0).cpu().numpy()
    scale = dW.double().abs().sum(dim=0).max().item()
    assert np.abs(got - want).max() <= 2e-3 * scale

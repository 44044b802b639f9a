"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

Configuration 2 (the headline shape) is compared against the full fp64 oracle, every
element.  Configurations 3-5 are too large for a full fp64 pass within a test, so they are
checked on outputs the oracle can compute one by one:
  * loss / lse and dHidden rows of a seeded sample of token rows (each row's oracle value
    needs only that row and the full vocabulary, so it is exact);
  * rows of dW on a seeded sample of vocabulary ids, from a second backward whose upstream
    gradient is non-zero only on a seeded subset of token rows (all N rows still flow
    through the kernels; the oracle then needs only that subset);
and on properties that hold at any size: ignored rows give exact zeros, the columns of dW
sum to zero (each row of softmax - onehot sums to zero), everything is finite.
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


def test_config2_full_oracle(B):
    w = I.make_config("qwen05b")
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    print(f"[full] qwen05b N={N} D={D} V={V}: GPU", flush=True)
    H, W, y = dev_inputs(w)
    ws = B.alloc_workspace(N, D, V)
    assert ws.numel() <= 0.01 * B.materialised_logit_bytes(N, V)
    loss, lse = B.cce_forward(H, W, y, IGN, workspace=ws)
    dl = torch.from_numpy(w.dloss_mean).cuda()
    dH, dW = B.cce_backward(H, W, y, lse, dl, IGN, workspace=ws)
    torch.cuda.synchronize()
    assert B.read_status(ws) == 0
    g_loss, g_lse = loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    g_dH = bf16_host(dH)
    print("[full] qwen05b: oracle forward", flush=True)
    o_loss, o_lse = O.forward(w.hidden, w.weight, w.labels, IGN)
    e_loss, e_lse = np.abs(g_loss - o_loss).max(), np.abs(g_lse - o_lse).max()
    print(f"[full] qwen05b: max|dloss|={e_loss:.2e} max|dlse|={e_lse:.2e}; oracle backward", flush=True)
    assert e_loss <= LOSS_ATOL and e_lse <= LOSS_ATOL
    ign = w.labels == IGN
    assert np.all(g_loss[ign] == 0) and np.all(g_lse[ign] == 0) and np.all(g_dH[ign] == 0)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, w.dloss_mean, IGN)
    e_dH = rel_fro(g_dH, o_dH)
    del o_dH
    # compare dW in slabs to bound host memory
    num = den = 0.0
    for r0 in range(0, V, 16384):
        g = dW[r0:r0 + 16384].cpu().numpy().astype(np.float64)
        num += float(((g - o_dW[r0:r0 + 16384]) ** 2).sum())
        den += float((o_dW[r0:r0 + 16384] ** 2).sum())
    e_dW = (num / den) ** 0.5
    print(f"[full] qwen05b: relF(dH)={e_dH:.2e} relF(dW)={e_dW:.2e}", flush=True)
    assert e_dH <= GRAD_RTOL and e_dW <= GRAD_RTOL


@pytest.mark.parametrize("name", ["1b", "7b", "smallv"])
def test_large_configs_sampled(B, name):
    w = I.make_config(name)
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    print(f"[full] {name} N={N} D={D} V={V}: GPU", flush=True)
    H, W, y = dev_inputs(w)
    ws = B.alloc_workspace(N, D, V)
    loss, lse = B.cce_forward(H, W, y, IGN, workspace=ws)
    dl = torch.from_numpy(w.dloss_mean).cuda()
    dH, dW = B.cce_backward(H, W, y, lse, dl, IGN, workspace=ws)
    torch.cuda.synchronize()
    assert B.read_status(ws) == 0

    g_loss, g_lse = loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    ign = w.labels == IGN
    assert np.all(np.isfinite(g_loss)) and np.all(g_loss[ign] == 0) and np.all(g_lse[ign] == 0)
    assert bool(torch.isfinite(dW).all()) and bool(torch.isfinite(dH.float()).all())
    if ign.any():
        ign_idx = torch.from_numpy(np.nonzero(ign)[0]).cuda()
        assert bool((dH[ign_idx] == 0).all())
    # columns of dW sum to zero (up to fp32/bf16 rounding of ~N terms per entry)
    colsum = dW.double().sum(dim=0).abs().max().item()
    scale = dW.double().abs().sum(dim=0).max().item()
    print(f"[full] {name}: max|colsum dW|={colsum:.3e} vs sum|dW|={scale:.3e}", flush=True)
    assert colsum <= 2e-3 * scale

    rng = np.random.default_rng(123)
    rows = np.unique(np.concatenate([[0, N - 1, 255, 256], rng.choice(N, 44, replace=False),
                                     np.nonzero(ign)[0][:4]])).astype(np.int64)
    print(f"[full] {name}: oracle on {rows.size} sampled rows", flush=True)
    o_loss, o_lse = O.forward(w.hidden[rows], w.weight, w.labels[rows], IGN)
    o_dH, _ = O.backward(w.hidden[rows], w.weight, w.labels[rows], w.dloss_mean[rows], IGN)
    e_loss, e_lse = np.abs(g_loss[rows] - o_loss).max(), np.abs(g_lse[rows] - o_lse).max()
    g_dH = bf16_host(dH[torch.from_numpy(rows).cuda()])
    e_dH = rel_fro(g_dH, o_dH)
    print(f"[full] {name}: max|dloss|={e_loss:.2e} max|dlse|={e_lse:.2e} relF(dH rows)={e_dH:.2e}", flush=True)
    assert e_loss <= LOSS_ATOL and e_lse <= LOSS_ATOL and e_dH <= GRAD_RTOL
    del dH

    # dW: upstream gradient only on a subset of rows; the oracle then needs only those rows
    sub = np.sort(rng.choice(np.nonzero(~ign)[0], 384, replace=False))
    dl2 = np.zeros(N, dtype=np.float32)
    dl2[sub] = w.dloss_var[sub]
    dH2, dW2 = B.cce_backward(H, W, y, lse, torch.from_numpy(dl2).cuda(), IGN, workspace=ws, d_weight=dW)
    torch.cuda.synchronize()
    vrows = np.unique(np.concatenate([[0, 1, 255, 256, V - 1, V - 2], w.labels[sub][:200],
                                      rng.choice(V, 600, replace=False)])).astype(np.int64)
    print(f"[full] {name}: oracle dW on {vrows.size} vocabulary rows from {sub.size} token rows", flush=True)
    o_dWr = O.dweight_rows(w.hidden[sub], w.weight, w.labels[sub], dl2[sub], vrows, IGN, row_block=128)
    g_dWr = dW2[torch.from_numpy(vrows).cuda()].cpu().numpy().astype(np.float64)
    e_dW = rel_fro(g_dWr, o_dWr)
    print(f"[full] {name}: relF(dW rows)={e_dW:.2e}", flush=True)
    assert e_dW <= GRAD_RTOL
    # rows of dH2 outside the subset have dloss = 0: exactly zero gradient
    mask = np.ones(N, bool)
    mask[sub] = False
    assert bool((dH2[torch.from_numpy(np.nonzero(mask)[0][:4096]).cuda()] == 0).all())

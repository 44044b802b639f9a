"""GPU parity of the loss variants over the valid rows only (cce_forward_compact_ex /
cce_backward_compact_ex, include/cce_compact.h) against the oracle.

The oracle is the undivided definition with the variant's loss (oracle/cce_oracle.py: smoothed
cross-entropy, z-loss, mean over the non-ignored rows): leaving ignored rows out changes which rows
the kernels see, not what is computed.  Tolerances are those of the plain path: per-token loss and
lse within 2e-3 absolute, dHidden and dW within 1e-2 relative Frobenius error, ignored rows exactly 0.
"""
import numpy as np
import pytest
import torch

from oracle import cce_oracle as O
from paper_2601_02609_amd import inputs as I
from tests.gpu_util import LOSS_ATOL, GRAD_RTOL, bf16_host, dev_inputs, rel_fro

pytestmark = pytest.mark.gpu
IGN = -100
ROW_BOUND = 2


@pytest.fixture(scope="module")
def B():
    from paper_2601_02609_amd import binding
    binding.lib()
    return binding


@pytest.fixture(autouse=True)
def always_skip(B):
    """Small shapes would not pay for row skipping: force it, so that the compact row space is tested."""
    B.set_row_skipping(2)
    yield
    B.set_row_skipping(0)


def run(B, w, dloss_np, bound, eps, lam, want_mean=False, grad_scale=1.0):
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    ws = B.alloc_compact_workspace(N, D, V, bound)
    loss = torch.full((N,), 7.0, device="cuda")
    lse = torch.full((N,), 7.0, device="cuda")
    _, _, mean = B.cce_forward_compact_ex(H, W, y, bound, IGN, label_smoothing=eps, z_loss=lam, want_mean=want_mean,
                                          workspace=ws, loss=loss, lse=lse)
    st_f = B.read_status(ws)
    dl = torch.from_numpy(dloss_np).cuda() if dloss_np is not None else None
    dH = torch.full((N, D), 3.0, dtype=torch.bfloat16, device="cuda")
    dW = torch.full((V, D), 3.0, dtype=torch.float32, device="cuda")
    B.cce_backward_compact_ex(H, W, y, lse, dl, bound, IGN, grad_scale=grad_scale, label_smoothing=eps, z_loss=lam,
                              workspace=ws, d_hidden=dH, d_weight=dW)
    torch.cuda.synchronize()
    st_b = B.read_status(ws)
    return (loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
            bf16_host(dH), dW.cpu().numpy().astype(np.float64), None if mean is None else float(mean.item()), st_f, st_b)


@pytest.mark.parametrize("eps,lam", [(0.1, 0.0), (0.0, 1e-3), (0.2, 1e-4)])
@pytest.mark.parametrize("shape,frac", [((700, 128, 3000), 0.2), ((1500, 896, 900), 0.35)])
def test_compact_variants_match_oracle(B, shape, frac, eps, lam):
    N, D, V = shape
    w = I.make_workload(I.custom_spec(N, D, V, seed=61, ignore_frac=frac))
    print(f"[compact variants] N={N} D={D} V={V} ignored={frac} eps={eps} lambda={lam}", flush=True)
    loss, lse, dH, dW, _, st_f, st_b = run(B, w, w.dloss_var, w.n_valid + 5, eps, lam)
    assert st_f == 0 and st_b == 0
    o_loss, o_lse = O.forward(w.hidden, w.weight, w.labels, IGN, label_smoothing=eps, z_loss=lam)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, w.dloss_var, IGN, label_smoothing=eps, z_loss=lam)
    ign = w.labels == IGN
    assert np.all(loss[ign] == 0.0) and np.all(lse[ign] == 0.0) and np.all(dH[ign] == 0.0)
    e = (np.abs(loss - o_loss).max(), np.abs(lse - o_lse).max(), rel_fro(dH, o_dH), rel_fro(dW, o_dW))
    print(f"[compact variants] max|dloss|={e[0]:.2e} max|dlse|={e[1]:.2e} relF(dH)={e[2]:.2e} relF(dW)={e[3]:.2e}", flush=True)
    assert e[0] <= LOSS_ATOL and e[1] <= LOSS_ATOL and e[2] <= GRAD_RTOL and e[3] <= GRAD_RTOL
    # the variants change the loss, so the comparison above is not vacuous
    p_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN)
    assert np.abs(o_loss - p_loss).max() > 10 * LOSS_ATOL


def test_compact_variant_rows_equal_the_all_rows_variant_bitwise(B):
    """A row's loss and lse do not depend on which other rows are computed."""
    w = I.make_workload(I.custom_spec(900, 256, 2500, seed=62, ignore_frac=0.4))
    loss, lse, *_ = run(B, w, w.dloss_var, w.n_valid, 0.15, 2e-4)
    H, W, y = dev_inputs(w)
    l2, s2, _ = B.cce_forward_ex(H, W, y, IGN, label_smoothing=0.15, z_loss=2e-4)
    assert np.array_equal(loss, l2.cpu().numpy().astype(np.float64))
    assert np.array_equal(lse, s2.cpu().numpy().astype(np.float64))


def test_compact_mean_reduction(B):
    """dloss = NULL: every valid row gets grad_scale / n_valid; mean_loss is the oracle's mean."""
    w = I.make_workload(I.custom_spec(700, 128, 3000, seed=63, ignore_frac=0.3))
    loss, lse, dH, dW, mean, st_f, st_b = run(B, w, None, w.n_valid, 0.1, 1e-4, want_mean=True, grad_scale=2.0)
    assert st_f == 0 and st_b == 0
    o_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN, label_smoothing=0.1, z_loss=1e-4)
    o_mean, n = O.mean_loss(o_loss, w.labels, IGN)
    assert n == w.n_valid and abs(mean - o_mean) <= LOSS_ATOL
    dl = np.full(700, 2.0 / n, dtype=np.float32)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, dl, IGN, label_smoothing=0.1, z_loss=1e-4)
    assert rel_fro(dH, o_dH) <= GRAD_RTOL and rel_fro(dW, o_dW) <= GRAD_RTOL
    # identical (bit for bit) to passing that dloss explicitly
    _, _, dH2, dW2, *_ = run(B, w, dl, w.n_valid, 0.1, 1e-4)
    assert np.array_equal(dH, dH2) and np.array_equal(dW, dW2)


def test_compact_mean_with_a_bound_that_drops_rows(B):
    """The mean is taken over the rows that took part: the first `bound` valid rows."""
    w = I.make_workload(I.custom_spec(640, 128, 1500, seed=64, ignore_frac=0.25))
    bound = w.n_valid - 100
    loss, lse, dH, dW, mean, st_f, st_b = run(B, w, None, bound, 0.0, 0.0, want_mean=True)
    assert (st_f & ROW_BOUND) and (st_b & ROW_BOUND)
    valid = np.nonzero(w.labels != IGN)[0]
    kept, dropped = valid[:bound], valid[bound:]
    labels_kept = w.labels.copy()
    labels_kept[dropped] = IGN
    o_loss, _ = O.forward(w.hidden, w.weight, labels_kept, IGN)
    o_mean, n = O.mean_loss(o_loss, labels_kept, IGN)
    assert n == bound and abs(mean - o_mean) <= LOSS_ATOL
    assert np.all(loss[dropped] == 0.0) and np.all(dH[dropped] == 0.0)
    dl = np.full(640, 1.0 / bound, dtype=np.float32)
    o_dH, o_dW = O.backward(w.hidden, w.weight, labels_kept, dl, IGN)
    assert rel_fro(dH, o_dH) <= GRAD_RTOL and rel_fro(dW, o_dW) <= GRAD_RTOL


def test_compact_mean_with_no_valid_rows(B):
    w = I.make_workload(I.custom_spec(300, 64, 500, seed=65, ignore_frac=1.0))
    loss, lse, dH, dW, mean, *_ = run(B, w, None, 10, 0.1, 1e-3, want_mean=True)
    assert mean == 0.0 and np.all(loss == 0) and np.all(dH == 0) and np.all(dW == 0)


def test_compact_variant_argument_errors(B):
    w = I.make_workload(I.custom_spec(300, 64, 500, seed=66, ignore_frac=0.5))
    H, W, y = dev_inputs(w)
    with pytest.raises(B.CCEError):
        B.cce_forward_compact_ex(H, W, y, w.n_valid, IGN, label_smoothing=1.0)
    with pytest.raises(B.CCEError):
        B.cce_forward_compact_ex(H, W, y, w.n_valid, IGN, z_loss=-1.0)
    lse = torch.zeros(300, device="cuda")
    with pytest.raises(B.CCEError):
        B.cce_backward_compact_ex(H, W, y, lse, None, w.n_valid, IGN, label_smoothing=-0.1)


def test_compact_variants_where_rows_are_not_skipped(B):
    """Automatic choice on a small shape: all rows are processed, the results are those of the _ex calls."""
    B.set_row_skipping(0)
    w = I.make_workload(I.custom_spec(700, 128, 3000, seed=67, ignore_frac=0.05))
    assert not B.get_row_skipping(700, 128, 3000, w.n_valid)
    loss, lse, dH, dW, mean, st_f, st_b = run(B, w, None, w.n_valid, 0.1, 1e-4, want_mean=True)
    H, W, y = dev_inputs(w)
    ws = B.alloc_workspace(700, 128, 3000)
    l2, s2, m2 = B.cce_forward_ex(H, W, y, IGN, label_smoothing=0.1, z_loss=1e-4, want_mean=True, workspace=ws)
    dH2, dW2 = B.cce_backward_ex(H, W, y, s2, None, IGN, label_smoothing=0.1, z_loss=1e-4, workspace=ws)
    assert np.array_equal(loss, l2.cpu().numpy().astype(np.float64)) and mean == float(m2.item())
    assert np.array_equal(dH, bf16_host(dH2)) and np.array_equal(dW, dW2.cpu().numpy().astype(np.float64))

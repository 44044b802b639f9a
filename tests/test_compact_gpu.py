"""GPU parity of the row-skipping entry points (include/cce_compact.h) against the oracle.

The oracle is the undivided definition (oracle/cce_oracle.py): skipping ignored rows changes
which rows the kernels see, not what is computed, so loss / lse / dHidden / dW must meet the same
tolerances, ignored rows must be exact zeros, and a bound that is too small must be flagged.
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
    """The small test shapes would not pay for row skipping (the library would quietly process all
    rows): force it, so that the compact row space is what is tested."""
    B.set_row_skipping(2)
    yield
    B.set_row_skipping(0)


def run_compact(B, w, dloss_np, bound):
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    ws = B.alloc_compact_workspace(N, D, V, bound)
    loss = torch.full((N,), 7.0, device="cuda")
    lse = torch.full((N,), 7.0, device="cuda")
    B.cce_forward_compact(H, W, y, bound, IGN, workspace=ws, loss=loss, lse=lse)
    st_f = B.read_status(ws)
    dl = torch.from_numpy(dloss_np).cuda()
    dH = torch.full((N, D), 3.0, dtype=torch.bfloat16, device="cuda")
    dW = torch.full((V, D), 3.0, dtype=torch.float32, device="cuda")
    B.cce_backward_compact(H, W, y, lse, dl, bound, IGN, workspace=ws, d_hidden=dH, d_weight=dW)
    torch.cuda.synchronize()
    st_b = B.read_status(ws)
    return (loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64),
            bf16_host(dH), dW.cpu().numpy().astype(np.float64), st_f, st_b)


@pytest.mark.parametrize("slack", [0, 37, 10 ** 9])
@pytest.mark.parametrize("shape,frac", [((700, 128, 3000), 0.2), ((333, 448, 1300), 0.6), ((600, 512, 2100), 0.0),
                                        ((1500, 896, 900), 0.35)])
def test_compact_matches_oracle(B, shape, frac, slack):
    N, D, V = shape
    w = I.make_workload(I.custom_spec(N, D, V, seed=51, ignore_frac=frac))
    bound = w.n_valid + slack
    print(f"[compact] N={N} D={D} V={V} valid={w.n_valid} bound={bound}", flush=True)
    loss, lse, dH, dW, st_f, st_b = run_compact(B, w, w.dloss_var, bound)
    assert st_f == 0 and st_b == 0
    o_loss, o_lse = O.forward(w.hidden, w.weight, w.labels, IGN)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, w.dloss_var, IGN)
    ign = w.labels == IGN
    assert np.all(loss[ign] == 0.0) and np.all(lse[ign] == 0.0) and np.all(dH[ign] == 0.0)
    e = (np.abs(loss - o_loss).max(), np.abs(lse - o_lse).max(), rel_fro(dH, o_dH), rel_fro(dW, o_dW))
    print(f"[compact] max|dloss|={e[0]:.2e} max|dlse|={e[1]:.2e} relF(dH)={e[2]:.2e} relF(dW)={e[3]:.2e}", flush=True)
    assert e[0] <= LOSS_ATOL and e[1] <= LOSS_ATOL and e[2] <= GRAD_RTOL and e[3] <= GRAD_RTOL


@pytest.mark.parametrize("acc", [1, 2])
@pytest.mark.parametrize("cols", [128, 256])
def test_compact_with_every_contraction_variant(B, cols, acc):
    """Row skipping with either contraction tile and either form of the dHidden running sum, over
    several row blocks and vocabulary chunks (forced tiling), a ragged last block included."""
    N, D, V = 1500, 512, 2100
    w = I.make_workload(I.custom_spec(N, D, V, seed=56, ignore_frac=0.3))
    try:
        B.set_backward_tiling(2, 3)
        B.set_backward_gemm_tile(cols)
        B.set_backward_accumulator(acc)
        loss, lse, dH, dW, st_f, st_b = run_compact(B, w, w.dloss_var, w.n_valid)
    finally:
        B.set_backward_tiling(0, 0)
        B.set_backward_gemm_tile(0)
        B.set_backward_accumulator(0)
    assert st_f == 0 and st_b == 0
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, w.dloss_var, IGN)
    ign = w.labels == IGN
    assert np.all(dH[ign] == 0.0)
    e = (rel_fro(dH, o_dH), rel_fro(dW, o_dW))
    print(f"[compact] tile 256x{cols} acc {acc}: relF(dH)={e[0]:.2e} relF(dW)={e[1]:.2e}", flush=True)
    assert e[0] <= GRAD_RTOL and e[1] <= GRAD_RTOL


def test_compact_forward_rows_equal_the_plain_forward_bitwise(B):
    """The forward of a row does not depend on which other rows are present: same bits as cce_forward."""
    w = I.make_workload(I.custom_spec(900, 256, 2500, seed=52, ignore_frac=0.3))
    H, W, y = dev_inputs(w)
    loss0, lse0 = B.cce_forward(H, W, y, IGN)
    loss1, lse1 = B.cce_forward_compact(H, W, y, w.n_valid, IGN)
    torch.cuda.synchronize()
    assert torch.equal(lse0, lse1) and torch.equal(loss0, loss1)


def test_bound_too_small_is_flagged(B):
    w = I.make_workload(I.custom_spec(700, 128, 3000, seed=53, ignore_frac=0.2))
    loss, lse, dH, dW, st_f, st_b = run_compact(B, w, w.dloss_mean, w.n_valid - 5)
    assert st_f & ROW_BOUND and st_b & ROW_BOUND
    # the rows that were kept are still right
    o_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN)
    valid = np.nonzero(w.labels != IGN)[0]
    kept = valid[: w.n_valid - 5]
    assert np.abs(loss[kept] - o_loss[kept]).max() <= LOSS_ATOL


def test_dropped_rows_give_zeros_not_stale_memory(B):
    """A bound that is too small drops the last valid rows: their loss, lse and dHidden rows are
    zero (the sentinels the outputs were prefilled with are gone) and the status bit is set."""
    w = I.make_workload(I.custom_spec(700, 128, 3000, seed=57, ignore_frac=0.2))
    drop = 9
    loss, lse, dH, dW, st_f, st_b = run_compact(B, w, w.dloss_mean, w.n_valid - drop)
    assert st_f & ROW_BOUND and st_b & ROW_BOUND
    valid = np.nonzero(w.labels != IGN)[0]
    dropped, kept = valid[-drop:], valid[:-drop]
    assert np.all(loss[dropped] == 0.0) and np.all(lse[dropped] == 0.0) and np.all(dH[dropped] == 0.0)
    assert np.all(loss[kept] != 7.0) and np.all(np.abs(dH[kept]).sum(axis=1) > 0)
    # what was computed is the gradient of the kept rows alone
    lab = w.labels.copy()
    lab[dropped] = IGN
    o_dH, o_dW = O.backward(w.hidden, w.weight, lab, w.dloss_mean, IGN)
    assert rel_fro(dH, o_dH) <= GRAD_RTOL and rel_fro(dW, o_dW) <= GRAD_RTOL


@pytest.mark.parametrize("slack", [0, 100])
def test_ignored_rows_are_inert_even_with_nan_hidden(B, slack):
    """The row-skipping path never loads the hidden row of an ignored token: NaN / Inf there (row 0
    included, and with a loose bound, where compact rows behind the last valid one exist) and NaN
    in dloss change no bit of any output."""
    spec = I.custom_spec(700, 128, 1500, seed=58, ignore_frac=0.3)
    w = I.make_workload(spec)
    w.labels[0] = IGN
    n_valid = int((w.labels != IGN).sum())
    assert n_valid + slack < spec.N                      # a bound >= N would switch row skipping off
    base = run_compact(B, w, w.dloss_mean, n_valid + slack)
    w2 = I.make_workload(spec)
    w2.labels[0] = IGN
    ign = w2.labels == IGN
    w2.hidden[ign] = 0x7FC0                              # bf16 NaN
    w2.hidden[np.nonzero(ign)[0][1]] = 0x7F80            # +Inf
    dl = w.dloss_mean.copy()
    dl[ign] = np.nan
    got = run_compact(B, w2, dl, n_valid + slack)
    for a, b in zip(base[:4], got[:4]):
        assert np.all(np.isfinite(b)) and np.array_equal(a, b)


def test_no_valid_rows_and_bad_labels(B):
    w = I.make_workload(I.custom_spec(300, 64, 500, seed=54, ignore_frac=1.0))
    loss, lse, dH, dW, st_f, st_b = run_compact(B, w, w.dloss_mean, 0)
    assert st_f == 0 and st_b == 0
    assert np.all(loss == 0) and np.all(lse == 0) and np.all(dH == 0) and np.all(dW == 0)
    w2 = I.make_workload(I.custom_spec(300, 64, 500, seed=55, ignore_frac=0.2))
    w2.labels[3] = 500                      # out of range: flagged, treated as not valid
    was_valid = 1 if w2.labels[3] != IGN else 0
    loss, lse, dH, dW, st_f, st_b = run_compact(B, w2, w2.dloss_mean, w2.n_valid)
    assert st_f & 1 and st_b & 1 and loss[3] == 0.0 and np.all(dH[3] == 0.0) and was_valid in (0, 1)


def test_automatic_choice(B):
    B.set_row_skipping(0)
    assert B.get_row_skipping(8192, 896, 151936, 6963)            # 15 % ignored: pays
    assert not B.get_row_skipping(32768, 3584, 151936, 31130)     # 5 % ignored: does not
    assert not B.get_row_skipping(8192, 896, 151936, 8192)
    B.set_row_skipping(1)
    assert not B.get_row_skipping(8192, 896, 151936, 6963)
    # without skipping a bound that is too small drops nothing and flags nothing
    w = I.make_workload(I.custom_spec(700, 128, 3000, seed=53, ignore_frac=0.2))
    loss, lse, dH, dW, st_f, st_b = run_compact(B, w, w.dloss_mean, w.n_valid - 5)
    o_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN)
    assert st_f == 0 and st_b == 0 and np.abs(loss - o_loss).max() <= LOSS_ATOL


def test_compact_argument_errors(B):
    w = I.make_workload(I.custom_spec(64, 64, 100, seed=9))
    H, W, y = dev_inputs(w)
    with pytest.raises(B.CCEError):
        B.cce_forward_compact(H, W, y, -1, IGN)
    assert B.compact_workspace_bytes(64, 60, 100, 10) == 0


def test_compact_at_the_headline_shape_sampled(B):
    """N=8192, D=896, V=151936 with the exact count of valid rows: loss / lse / dHidden on a seeded
    sample of rows and dW on sampled vocabulary rows against the oracle; workspace within 1 %."""
    w = I.make_config("qwen05b")
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    H, W, y = dev_inputs(w)
    ws = B.alloc_compact_workspace(N, D, V, w.n_valid)
    assert ws.numel() <= 0.01 * B.materialised_logit_bytes(N, V)
    loss, lse = B.cce_forward_compact(H, W, y, w.n_valid, IGN, workspace=ws)
    rng = np.random.default_rng(17)
    rows = np.unique(np.concatenate([[0, N - 1, 255, 256], rng.choice(N, 24, replace=False)])).astype(np.int64)
    dl_np = np.zeros(N, dtype=np.float32)
    dl_np[rows] = 1.0 / w.n_valid
    dH, dW = B.cce_backward_compact(H, W, y, lse, torch.from_numpy(dl_np).cuda(), w.n_valid, IGN, workspace=ws)
    torch.cuda.synchronize()
    assert B.read_status(ws) == 0
    print(f"[compact] headline shape: oracle on {rows.size} rows", flush=True)
    o_loss, o_lse = O.forward(w.hidden[rows], w.weight, w.labels[rows], IGN)
    g_loss, g_lse = loss.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    assert np.abs(g_loss[rows] - o_loss).max() <= LOSS_ATOL and np.abs(g_lse[rows] - o_lse).max() <= LOSS_ATOL
    ign = w.labels == IGN
    assert np.all(g_loss[ign] == 0) and np.all(g_lse[ign] == 0)
    o_dH, o_dW = O.backward(w.hidden[rows], w.weight, w.labels[rows], dl_np[rows], IGN)
    assert rel_fro(bf16_host(dH[torch.from_numpy(rows).cuda()]), o_dH) <= GRAD_RTOL
    other = np.setdiff1d(np.arange(N), rows)
    assert float(dH[torch.from_numpy(other).cuda()].float().abs().max().item()) == 0.0
    vrows = np.unique(np.concatenate([w.labels[rows][w.labels[rows] >= 0], rng.choice(V, 200, replace=False)]))
    assert rel_fro(dW[torch.from_numpy(vrows).cuda()].cpu().numpy().astype(np.float64), o_dW[vrows]) <= GRAD_RTOL

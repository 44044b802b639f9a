"""GPU parity of the vocabulary-parallel share (include/cce_shard.h) against the oracle.

One GPU plays every shard in turn: per-shard statistics against oracle/shard_oracle.py, the
merged loss / lse and the summed / concatenated gradients against the undivided oracle
(oracle/cce_oracle.py), to the same tolerances as the undivided path.  Summing P bf16 partial
dHidden adds P roundings of 2^-9 relative each, well inside the 1e-2 Frobenius bar.
"""
import numpy as np
import pytest
import torch

from oracle import cce_oracle as O
from oracle import shard_oracle as S
from paper_2601_02609_amd import inputs as I
from tests.gpu_util import LOSS_ATOL, GRAD_RTOL, bf16_dev, bf16_host, dev_inputs, rel_fro

pytestmark = pytest.mark.gpu
IGN = -100


@pytest.fixture(scope="module")
def B():
    from paper_2601_02609_amd import binding
    binding.lib()
    return binding


def parts_of(V, cuts):
    edges = [0] + list(cuts) + [V]
    return [(edges[i], edges[i + 1]) for i in range(len(edges) - 1)]


def run_sharded(B, w, parts, dloss_np, eps=0.0, lam=0.0, want_mean=False, grad_scale=1.0):
    """All shards on the one GPU; returns host arrays."""
    H, W, y = dev_inputs(w)
    N, D = w.hidden.shape
    V = w.weight.shape[0]
    stats = torch.empty(len(parts), N, 4, dtype=torch.float32, device="cuda")
    for p, (a, b) in enumerate(parts):
        B.cce_shard_forward(H, W[a:b], y, a, want_sumz=eps != 0.0, stats=stats[p])
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    loss, lse, mean = B.cce_shard_merge(stats, y, V, IGN, label_smoothing=eps, z_loss=lam,
                                        want_mean=want_mean, status=status)
    dl = torch.from_numpy(dloss_np).cuda() if dloss_np is not None else None
    dH_sum = np.zeros((N, D))
    dW = torch.empty(V, D, dtype=torch.float32, device="cuda")
    for a, b in parts:
        dh, _ = B.cce_shard_backward(H, W[a:b], y, lse, dl, a, V, IGN, grad_scale=grad_scale,
                                     label_smoothing=eps, z_loss=lam, d_weight=dW[a:b])
        dH_sum += bf16_host(dh)
    torch.cuda.synchronize()
    return (stats.cpu().numpy().astype(np.float64), loss.cpu().numpy().astype(np.float64),
            lse.cpu().numpy().astype(np.float64), dH_sum, dW.cpu().numpy().astype(np.float64),
            None if mean is None else float(mean.item()), int(status.item()))


@pytest.mark.parametrize("eps,lam", [(0.0, 0.0), (0.1, 1e-3)])
@pytest.mark.parametrize("shape,cuts", [((700, 128, 3000), [1000, 1300]), ((333, 448, 1300), [1]),
                                        ((600, 512, 2100), [256, 512, 1111, 2099])])
def test_shards_match_oracle(B, shape, cuts, eps, lam):
    N, D, V = shape
    w = I.make_workload(I.custom_spec(N, D, V, seed=31, ignore_frac=0.15))
    parts = parts_of(V, cuts)
    print(f"[shard] N={N} D={D} V={V} parts={parts} eps={eps} lambda={lam}", flush=True)
    stats, loss, lse, dH, dW, _, status = run_sharded(B, w, parts, w.dloss_var, eps, lam)
    assert status == 0
    # per-shard statistics against their definition
    for p, (a, b) in enumerate(parts):
        o = S.shard_stats(w.hidden, w.weight[a:b], w.labels, a)
        lse_p = stats[p, :, 0] + np.log(stats[p, :, 1])
        o_lse_p = o[:, 0] + np.log(o[:, 1])
        assert np.abs(stats[p, :, 0] - o[:, 0]).max() <= LOSS_ATOL          # max logit
        assert np.abs(lse_p - o_lse_p).max() <= LOSS_ATOL                   # (m, d) as a pair
        assert np.abs(stats[p, :, 2] - o[:, 2]).max() <= LOSS_ATOL          # label logit
        assert np.array_equal(stats[p, :, 2] != 0, o[:, 2] != 0)            # ... owned by the same shard
        if eps != 0.0:
            assert np.abs(stats[p, :, 3] - o[:, 3]).max() <= 1e-3 * max(1.0, np.abs(o[:, 3]).max())
        else:
            assert np.all(stats[p, :, 3] == 0.0)
    # merged result and gradients against the undivided definition
    o_loss, o_lse = O.forward(w.hidden, w.weight, w.labels, IGN, label_smoothing=eps, z_loss=lam)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, w.dloss_var, IGN, label_smoothing=eps, z_loss=lam)
    ign = w.labels == IGN
    assert np.all(loss[ign] == 0.0) and np.all(lse[ign] == 0.0) and np.all(dH[ign] == 0.0)
    e = (np.abs(loss - o_loss).max(), np.abs(lse - o_lse).max(), rel_fro(dH, o_dH), rel_fro(dW, o_dW))
    print(f"[shard] max|dloss|={e[0]:.2e} max|dlse|={e[1]:.2e} relF(dH)={e[2]:.2e} relF(dW)={e[3]:.2e}", flush=True)
    assert e[0] <= LOSS_ATOL and e[1] <= LOSS_ATOL and e[2] <= GRAD_RTOL and e[3] <= GRAD_RTOL


def test_one_shard_equals_the_undivided_path_bitwise(B):
    """P = 1 runs the same kernels on the same data: loss, lse and gradients are the same bits."""
    w = I.make_workload(I.custom_spec(520, 256, 1500, seed=32, ignore_frac=0.1))
    H, W, y = dev_inputs(w)
    V = 1500
    loss0, lse0 = B.cce_forward(H, W, y, IGN)
    dl = torch.from_numpy(w.dloss_mean).cuda()
    dH0, dW0 = B.cce_backward(H, W, y, lse0, dl, IGN)
    st = B.cce_shard_forward(H, W, y, 0)
    loss1, lse1, _ = B.cce_shard_merge(st.view(1, -1, 4), y, V, IGN)
    dH1, dW1 = B.cce_shard_backward(H, W, y, lse1, dl, 0, V, IGN)
    torch.cuda.synchronize()
    # the statistics cross the interface in natural units (one extra fp32 rounding each way)
    assert (lse1 - lse0).abs().max().item() <= 4e-6 and (loss1 - loss0).abs().max().item() <= 4e-6
    dH2, dW2 = B.cce_shard_backward(H, W, y, lse0, dl, 0, V, IGN)
    torch.cuda.synchronize()
    assert torch.equal(dH2, dH0) and torch.equal(dW2, dW0)
    assert rel_fro(bf16_host(dH1), bf16_host(dH0)) <= 1e-4


def test_sharded_mean_reduction_and_bad_label(B):
    w = I.make_workload(I.custom_spec(400, 128, 900, seed=33, ignore_frac=0.25))
    parts = parts_of(900, [300, 640])
    stats, loss, lse, dH, dW, mean, status = run_sharded(B, w, parts, None, want_mean=True, grad_scale=1.0)
    o_loss, _ = O.forward(w.hidden, w.weight, w.labels, IGN)
    o_mean, n = O.mean_loss(o_loss, w.labels, IGN)
    assert status == 0 and abs(mean - o_mean) <= LOSS_ATOL
    dl = np.full(400, 1.0 / n, dtype=np.float32)
    o_dH, o_dW = O.backward(w.hidden, w.weight, w.labels, dl, IGN)
    assert rel_fro(dH, o_dH) <= GRAD_RTOL and rel_fro(dW, o_dW) <= GRAD_RTOL
    # a label beyond the full vocabulary: flagged by the merge, inert in every shard's gradients
    bad = w.labels.copy()
    victim = int(np.nonzero(bad != IGN)[0][0])
    bad[victim] = 900
    w2 = I.Workload(w.spec, w.hidden, w.weight, bad, w.dloss_mean, w.dloss_var, w.n_valid - 1)
    _, loss2, lse2, dH2, _, _, status2 = run_sharded(B, w2, parts, w.dloss_mean)
    assert status2 != 0 and loss2[victim] == 0.0 and lse2[victim] == 0.0 and np.all(dH2[victim] == 0.0)


def test_shard_argument_errors(B):
    w = I.make_workload(I.custom_spec(64, 64, 100, seed=9))
    H, W, y = dev_inputs(w)
    lse = torch.zeros(64, device="cuda")
    dl = torch.zeros(64, device="cuda")
    with pytest.raises(B.CCEError):
        B.cce_shard_forward(H, W, y, -1)
    with pytest.raises(B.CCEError):
        B.cce_shard_backward(H, W, y, lse, dl, 50, 120, IGN)        # shard sticks out of the vocabulary
    st = torch.zeros(1, 64, 4, device="cuda")
    with pytest.raises(B.CCEError):
        B.cce_shard_merge(st, y, 100, IGN, label_smoothing=1.5)


def test_one_eighth_of_the_headline_vocabulary(B):
    """The share of one of 8 devices at the headline shape (N=8192, D=896, Vs=18992): statistics of
    shard 3 on sampled rows against their definition; merge of all 8 shards against the undivided
    GPU forward; shard 3's dW rows and partial dHidden on sampled rows against the oracle."""
    w = I.make_config("qwen05b")
    N, D, V = w.spec.N, w.spec.D, w.spec.V
    P = 8
    Vs = V // P
    assert Vs * P == V
    H, W, y = dev_inputs(w)
    ws = B.alloc_workspace(N, D, Vs)
    stats = torch.empty(P, N, 4, dtype=torch.float32, device="cuda")
    for p in range(P):
        B.cce_shard_forward(H, W[p * Vs:(p + 1) * Vs], y, p * Vs, stats=stats[p], workspace=ws)
    loss, lse, _ = B.cce_shard_merge(stats, y, V, IGN)
    loss0, lse0 = B.cce_forward(H, W, y, IGN)
    torch.cuda.synchronize()
    assert (lse - lse0).abs().max().item() <= 2e-5 and (loss - loss0).abs().max().item() <= 2e-5
    rng = np.random.default_rng(11)
    rows = np.unique(np.concatenate([[0, N - 1, 255, 256], rng.choice(N, 20, replace=False)])).astype(np.int64)
    p = 3
    a, b = p * Vs, (p + 1) * Vs
    print(f"[shard] headline share: oracle on {rows.size} rows of shard {p}", flush=True)
    o = S.shard_stats(w.hidden[rows], w.weight[a:b], w.labels[rows], a)
    g = stats[p].cpu().numpy().astype(np.float64)[rows]
    assert np.abs(g[:, 0] - o[:, 0]).max() <= LOSS_ATOL
    assert np.abs((g[:, 0] + np.log(g[:, 1])) - (o[:, 0] + np.log(o[:, 1]))).max() <= LOSS_ATOL
    assert np.abs(g[:, 2] - o[:, 2]).max() <= LOSS_ATOL
    # backward of the shard: upstream gradient on the sampled rows only, so that the oracle needs only them
    dl_np = np.zeros(N, dtype=np.float32)
    dl_np[rows] = 1.0 / w.n_valid
    dl = torch.from_numpy(dl_np).cuda()
    dH, dW = B.cce_shard_backward(H, W[a:b], y, lse, dl, a, V, IGN, workspace=ws)
    torch.cuda.synchronize()
    o_dH, o_dW = S.shard_backward(w.hidden[rows], w.weight[a:b], w.labels[rows], lse.cpu().numpy()[rows],
                                  dl_np[rows], a, V, IGN)
    assert rel_fro(bf16_host(dH[torch.from_numpy(rows).cuda()]), o_dH) <= GRAD_RTOL
    assert rel_fro(dW.cpu().numpy().astype(np.float64), o_dW) <= GRAD_RTOL
    other = np.setdiff1d(np.arange(N), rows)[:64]
    assert np.all(bf16_host(dH[torch.from_numpy(other).cuda()]) == 0.0)

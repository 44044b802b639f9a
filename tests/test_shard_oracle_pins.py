"""Pins of oracle/shard_oracle.py (CPU): the vocabulary-parallel share must reproduce the
undivided cross-entropy, whatever the partition.  Checked against torch (float64, autograd),
not against the other oracle files."""
import numpy as np
import pytest
import torch

from oracle import shard_oracle as S
from paper_2601_02609_amd import inputs as I


def _case(seed, N=37, D=64, V=203, ignore_frac=0.2):
    return I.make_workload(I.custom_spec(N, D, V, seed=seed, ignore_frac=ignore_frac))


def _f64(bits):
    return torch.from_numpy((np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64))


def _split(V, cuts):
    edges = [0] + list(cuts) + [V]
    return [(edges[i], edges[i + 1]) for i in range(len(edges) - 1)]


def _all_stats(w, parts):
    return np.stack([S.shard_stats(w.hidden, w.weight[a:b], w.labels, a) for a, b in parts])


@pytest.mark.parametrize("cuts", [[], [100], [1, 202], [64, 65, 150]])
def test_merged_lse_is_logsumexp_of_the_full_row(cuts):
    w = _case(1)
    parts = _split(w.weight.shape[0], cuts)
    _, lse = S.merge(_all_stats(w, parts), w.labels, w.weight.shape[0])
    Z = _f64(w.hidden) @ _f64(w.weight).T
    ref = torch.logsumexp(Z, dim=1).numpy()
    valid = w.labels != -100
    np.testing.assert_allclose(lse[valid], ref[valid], rtol=1e-13)
    assert np.all(lse[~valid] == 0.0)


@pytest.mark.parametrize("eps,lam", [(0.0, 0.0), (0.1, 0.0), (0.0, 1e-3), (0.2, 5e-4)])
def test_merged_loss_and_summed_gradients_match_torch_autograd(eps, lam):
    w = _case(2)
    V = w.weight.shape[0]
    parts = _split(V, [70, 140])
    loss, lse = S.merge(_all_stats(w, parts), w.labels, V, label_smoothing=eps, z_loss=lam)
    H = _f64(w.hidden).requires_grad_(True)
    W = _f64(w.weight).requires_grad_(True)
    Z = H @ W.T
    y = torch.from_numpy(w.labels.astype(np.int64))
    ce = torch.nn.functional.cross_entropy(Z, y, ignore_index=-100, reduction="none", label_smoothing=eps)
    ref = ce + lam * torch.logsumexp(Z, dim=1) ** 2 * (y != -100)
    np.testing.assert_allclose(loss, ref.detach().numpy(), rtol=1e-12, atol=1e-12)
    rng = np.random.default_rng(5)
    dloss = rng.standard_normal(len(loss))
    (ref * torch.from_numpy(dloss)).sum().backward()
    dH = np.zeros(tuple(H.shape))
    dW = np.zeros(tuple(W.shape))
    for a, b in parts:
        dh, dw = S.shard_backward(w.hidden, w.weight[a:b], w.labels, lse, dloss, a, V,
                                  label_smoothing=eps, z_loss=lam)
        dH += dh
        dW[a:b] = dw
    np.testing.assert_allclose(dH, H.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dW, W.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_shard_order_and_partition_do_not_matter():
    w = _case(3)
    V = w.weight.shape[0]
    a = _all_stats(w, _split(V, [50, 120]))
    b = _all_stats(w, _split(V, [17]))
    la, _ = S.merge(a, w.labels, V, label_smoothing=0.1)
    lb, _ = S.merge(b, w.labels, V, label_smoothing=0.1)
    lc, _ = S.merge(a[::-1], w.labels, V, label_smoothing=0.1)
    np.testing.assert_allclose(la, lb, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(la, lc, rtol=1e-12, atol=1e-13)


def test_label_logit_is_owned_by_exactly_one_shard():
    w = _case(4, ignore_frac=0.0)
    V = w.weight.shape[0]
    parts = _split(V, [60, 61, 150])
    labels = w.labels.copy()
    labels[:6] = [0, 59, 60, 61, 149, V - 1]          # first / last rows of shards
    st = np.stack([S.shard_stats(w.hidden, w.weight[a:b], labels, a) for a, b in parts])
    owners = (st[:, :, 2] != 0.0).sum(axis=0)
    assert np.all(owners <= 1)
    Z = (_f64(w.hidden) @ _f64(w.weight).T).numpy()
    np.testing.assert_allclose(st[:, :, 2].sum(axis=0), Z[np.arange(len(labels)), labels], rtol=1e-13)
    for p, (a, b) in enumerate(parts):
        inside = (labels >= a) & (labels < b)
        assert np.all(st[p, ~inside, 2] == 0.0)


def test_stats_of_a_shard_far_below_the_maximum_stay_finite():
    """A shard whose logits are all hugely negative relative to another contributes
    exp(m_p - M) = 0 to the merged sum without producing inf or nan."""
    stats = np.zeros((2, 1, 4))
    stats[0, 0] = [5.0, 2.0, 5.0, 7.0]
    stats[1, 0] = [-2000.0, 3.0, 0.0, -4000.0]
    loss, lse = S.merge(stats, np.array([0]), 10)
    assert np.isfinite(loss[0]) and abs(lse[0] - (5.0 + np.log(2.0))) < 1e-15
    assert abs(loss[0] - np.log(2.0)) < 1e-15

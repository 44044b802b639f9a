"""Pins for the fp64 oracle: what the paper and the mathematics fix, independent of the oracle.

Each test would fail for a plausible mistake in oracle/cce_oracle.py: a dropped
term, a wrong sign, a transposed operand, a missed ignore rule, a label off by one.
None of them retypes the oracle's own vectorised formulas: they use closed forms,
invariants, scalar brute-force loops, finite differences of the oracle's *forward*,
and torch's own cross-entropy + autograd (float64, CPU).
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import cce_oracle as O
from paper_2601_02609_amd import inputs as I

IGN = -100


def _bits(x):
    return I.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _small(N=12, D=8, V=16, seed=3, ignore=(2, 7)):
    rng = np.random.default_rng(seed)
    H = _bits(rng.standard_normal((N, D)))
    W = _bits(rng.standard_normal((V, D)) * 0.7)
    y = rng.integers(0, V, size=N).astype(np.int32)
    for i in ignore:
        y[i] = IGN
    dl = rng.uniform(0.5, 1.5, size=N).astype(np.float32)
    return H, W, y, dl


# ---------------------------------------------------------------- loss / lse

def test_bruteforce_scalar_loops():
    """Triple loop with math.exp/log on a tiny case (cross-entropy definition)."""
    H, W, y, dl = _small(N=6, D=5, V=9, ignore=(1,))
    Hf = I.bf16_bits_to_f32(H).astype(float)
    Wf = I.bf16_bits_to_f32(W).astype(float)
    loss, lse = O.forward(H, W, y, IGN)
    for i in range(6):
        z = [sum(Hf[i, k] * Wf[v, k] for k in range(5)) for v in range(9)]
        if y[i] == IGN:
            assert loss[i] == 0.0 and lse[i] == 0.0
            continue
        s = math.log(sum(math.exp(zz) for zz in z))
        assert abs(lse[i] - s) < 1e-12
        assert abs(loss[i] - (s - z[y[i]])) < 1e-12


def test_loss_is_lse_minus_label_logit():
    H, W, y, _ = _small()
    loss, lse = O.forward(H, W, y, IGN)
    Z = I.bf16_bits_to_f32(H).astype(np.float64) @ I.bf16_bits_to_f32(W).astype(np.float64).T
    for i in range(len(y)):
        if y[i] != IGN:
            assert abs(loss[i] - (lse[i] - Z[i, y[i]])) < 1e-12


@pytest.mark.parametrize("V", [1000, 151936, 32000])
def test_zero_weight_gives_ln_V(V):
    """W = 0: every logit is 0, so lse = loss = ln V (uniform prediction)."""
    N, D = 5, 4
    H = _bits(np.random.default_rng(0).standard_normal((N, D)))
    W = np.zeros((V, D), dtype=np.uint16)
    y = np.array([0, V - 1, V // 2, IGN, 3 % V], dtype=np.int32)
    loss, lse = O.forward(H, W, y, IGN)
    # ln 1000 = 3 ln 10, ln 151936 = 7 ln 2 + ln 1187, ln 32000 = 8 ln 2 + 3 ln 5
    ln2, ln5, ln10, ln1187 = 0.6931471805599453, 1.6094379124341003, 2.302585092994046, 7.079184394609668
    expect = {1000: 3 * ln10, 151936: 7 * ln2 + ln1187, 32000: 8 * ln2 + 3 * ln5}[V]
    assert abs(expect - {1000: 6.907755279, 151936: 11.931214659, 32000: 10.373491182}[V]) < 1e-8
    for i in range(N):
        if y[i] == IGN:
            assert loss[i] == 0.0 and lse[i] == 0.0
        else:
            assert abs(loss[i] - expect) < 1e-8 and abs(lse[i] - expect) < 1e-8


def test_zero_hidden_gives_ln_V():
    V = 37
    H = np.zeros((3, 6), dtype=np.uint16)
    W = _bits(np.random.default_rng(1).standard_normal((V, 6)))
    y = np.array([0, 36, 5], dtype=np.int32)
    loss, lse = O.forward(H, W, y, IGN)
    assert np.allclose(loss, math.log(V), atol=1e-13)
    assert np.allclose(lse, math.log(V), atol=1e-13)


def test_single_class_loss_zero():
    H, W, _, _ = _small(V=1)
    y = np.zeros(H.shape[0], dtype=np.int32)
    loss, lse = O.forward(H, W, y, IGN)
    assert np.all(np.abs(loss) < 1e-15)


def test_shift_invariance():
    """Adding one vector u to every row of W adds h_i.u to lse_i and leaves loss_i unchanged.
    (u is chosen so that W + u stays exactly representable in bf16.)"""
    rng = np.random.default_rng(5)
    N, D, V = 7, 4, 11
    Hq = np.round(rng.standard_normal((N, D)) * 4) / 4
    Wq = np.round(rng.standard_normal((V, D)) * 4) / 4
    u = np.array([0.5, -1.0, 0.25, 2.0])
    y = rng.integers(0, V, size=N).astype(np.int32)
    l0, s0 = O.forward(_bits(Hq), _bits(Wq), y, IGN)
    l1, s1 = O.forward(_bits(Hq), _bits(Wq + u), y, IGN)
    assert np.allclose(l0, l1, atol=1e-12)
    assert np.allclose(s1 - s0, Hq @ u, atol=1e-12)


def test_online_recurrence_reaches_oracle_lse():
    """The online (m, d) recurrence of the online-softmax definition, run element by
    element and also chunk by chunk, reaches the plain log-sum-exp (correctness theorem)."""
    H, W, y, _ = _small(N=4, D=8, V=50, ignore=())
    _, lse = O.forward(H, W, y, IGN)
    Z = O.logits(H, W)
    for i in range(4):
        m, d = -math.inf, 0.0
        for x in Z[i]:
            mn = max(m, x)
            d = d * math.exp(m - mn) + math.exp(x - mn)
            m = mn
        assert abs(math.log(d) + m - lse[i]) < 1e-12
        # chunked with a ragged tail (chunk 16 over V = 50)
        m, d = -math.inf, 0.0
        for c in range(0, 50, 16):
            zc = Z[i, c:c + 16]
            mn = max(m, zc.max())
            d = d * math.exp(m - mn) + float(np.exp(zc - mn).sum())
            m = mn
        assert abs(math.log(d) + m - lse[i]) < 1e-12


def test_large_logits_do_not_overflow():
    D = 4
    H = _bits(np.full((2, D), 16.0))
    W = _bits(np.array([[8.0] * D, [-8.0] * D, [7.5] * D]))
    y = np.array([0, 2], dtype=np.int32)
    loss, lse = O.forward(H, W, y, IGN)       # logits 512, -512, 480
    assert np.all(np.isfinite(loss)) and np.all(np.isfinite(lse))
    assert abs(lse[0] - (512.0 + math.log1p(math.exp(-32.0)))) < 1e-9
    assert abs(loss[1] - (lse[1] - 480.0)) < 1e-9


def test_out_of_range_label_raises():
    H, W, y, _ = _small()
    y[0] = W.shape[0]
    with pytest.raises(ValueError):
        O.forward(H, W, y, IGN)
    y[0] = -1
    with pytest.raises(ValueError):
        O.forward(H, W, y, IGN)


# ---------------------------------------------------------------- torch as a library pin

def _torch_ref(H, W, y, dl):
    Ht = torch.tensor(I.bf16_bits_to_f32(H), dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(I.bf16_bits_to_f32(W), dtype=torch.float64, requires_grad=True)
    yt = torch.tensor(y.astype(np.int64))
    loss = torch.nn.functional.cross_entropy(Ht @ Wt.T, yt, ignore_index=IGN, reduction="none")
    g = torch.tensor(np.where(y == IGN, 0.0, dl.astype(np.float64)))
    (loss * g).sum().backward()
    return loss.detach().numpy(), Ht.grad.numpy(), Wt.grad.numpy()


@pytest.mark.parametrize("shape", [(12, 8, 16), (33, 24, 130), (64, 16, 1000)])
def test_against_torch_cross_entropy_and_autograd(shape):
    N, D, V = shape
    H, W, y, dl = _small(N=N, D=D, V=V, ignore=(0, N // 2))
    loss_t, dH_t, dW_t = _torch_ref(H, W, y, dl)
    loss, _ = O.forward(H, W, y, IGN)
    dH, dW = O.backward(H, W, y, dl, IGN, row_block=7)
    assert np.allclose(loss, loss_t, atol=1e-12, rtol=0)
    assert np.allclose(dH, dH_t, atol=1e-12, rtol=0)
    assert np.allclose(dW, dW_t, atol=1e-12, rtol=0)


# ---------------------------------------------------------------- gradient pins

def test_grad_rows_sum_to_zero_and_bounded():
    H, W, y, dl = _small(N=20, D=8, V=40, ignore=(4, 5))
    G = O.grad_logits(H, W, y, dl, IGN)
    assert np.all(np.abs(G.sum(axis=1)) < 1e-14)
    assert np.all(np.abs(G) <= np.abs(np.where(y == IGN, 0, dl))[:, None] + 1e-15)
    assert np.all(G[4] == 0.0) and np.all(G[5] == 0.0)
    # the label entry is the only negative one in a valid row
    for i in range(20):
        if y[i] != IGN:
            neg = np.nonzero(G[i] < 0)[0]
            assert list(neg) == [y[i]]


def test_finite_differences_on_weighted_loss():
    """Central differences of sum_i dloss_i * loss_i in H and W (perturbing the widened
    values directly, in float64, through a scalar re-implementation of the loss)."""
    H, W, y, dl = _small(N=5, D=4, V=7, ignore=(3,))
    Hf = I.bf16_bits_to_f32(H).astype(np.float64)
    Wf = I.bf16_bits_to_f32(W).astype(np.float64)
    g = np.where(y == IGN, 0.0, dl.astype(np.float64))

    def total(Hx, Wx):
        t = 0.0
        for i in range(Hx.shape[0]):
            if y[i] == IGN:
                continue
            z = Wx @ Hx[i]
            t += g[i] * (math.log(np.exp(z - z.max()).sum()) + z.max() - z[y[i]])
        return t

    dH, dW = O.backward(H, W, y, dl, IGN)
    eps = 1e-6
    for (i, k) in [(0, 0), (1, 3), (3, 2), (4, 1)]:
        Hp, Hm = Hf.copy(), Hf.copy()
        Hp[i, k] += eps
        Hm[i, k] -= eps
        fd = (total(Hp, Wf) - total(Hm, Wf)) / (2 * eps)
        assert abs(fd - dH[i, k]) < 1e-8
    for (v, k) in [(0, 0), (int(y[0]), 1), (6, 3), (2, 2)]:
        Wp, Wm = Wf.copy(), Wf.copy()
        Wp[v, k] += eps
        Wm[v, k] -= eps
        fd = (total(Hf, Wp) - total(Hf, Wm)) / (2 * eps)
        assert abs(fd - dW[v, k]) < 1e-8
    assert np.all(dH[3] == 0.0)


def test_closed_form_at_zero_weight():
    """W = 0: softmax is uniform, so dH = 0 and dW[v] = sum_i dloss_i (1/V - 1[y_i = v]) h_i."""
    rng = np.random.default_rng(9)
    N, D, V = 9, 5, 6
    H = _bits(rng.standard_normal((N, D)))
    W = np.zeros((V, D), dtype=np.uint16)
    y = rng.integers(0, V, size=N).astype(np.int32)
    y[2] = IGN
    dl = rng.uniform(0.5, 1.5, size=N).astype(np.float32)
    dH, dW = O.backward(H, W, y, dl, IGN)
    assert np.all(np.abs(dH) < 1e-15)
    Hf = I.bf16_bits_to_f32(H).astype(np.float64)
    for v in range(V):
        acc = np.zeros(D)
        for i in range(N):
            if y[i] == IGN:
                continue
            acc += float(dl[i]) * (1.0 / V - (1.0 if y[i] == v else 0.0)) * Hf[i]
        assert np.allclose(dW[v], acc, atol=1e-14)


def test_dW_columns_sum_to_zero():
    H, W, y, dl = _small(N=30, D=6, V=25, ignore=(1,))
    _, dW = O.backward(H, W, y, dl, IGN)
    assert np.all(np.abs(dW.sum(axis=0)) < 1e-13)


def test_ignored_rows_are_inert_even_with_nan_dloss():
    H, W, y, dl = _small(N=10, D=6, V=12, ignore=(2, 7))
    dH0, dW0 = O.backward(H, W, y, dl, IGN)
    H2 = H.copy()
    H2[2] = _bits(np.full(6, 1e30))
    dl2 = dl.copy()
    dl2[2] = np.nan
    dl2[7] = np.inf
    dH1, dW1 = O.backward(H2, W, y, dl2, IGN)
    assert np.array_equal(dW0, dW1)
    assert np.all(dH1[2] == 0.0) and np.all(dH1[7] == 0.0)
    mask = np.ones(10, bool)
    mask[[2, 7]] = False
    assert np.array_equal(dH0[mask], dH1[mask])


def test_row_blocking_does_not_change_results():
    H, W, y, dl = _small(N=29, D=8, V=33, ignore=(0, 28))
    a = O.forward(H, W, y, IGN, row_block=1000)
    b = O.forward(H, W, y, IGN, row_block=5)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    dHa, dWa = O.backward(H, W, y, dl, IGN, row_block=1000)
    dHb, dWb = O.backward(H, W, y, dl, IGN, row_block=5)
    assert np.array_equal(dHa, dHb) and np.allclose(dWa, dWb, atol=1e-14)


def test_dweight_rows_matches_full_backward_and_torch():
    H, W, y, dl = _small(N=40, D=8, V=50, ignore=(3, 9))
    _, dW = O.backward(H, W, y, dl, IGN)
    rows = np.array([0, 7, 49, int(y[0])])
    got = O.dweight_rows(H, W, y, dl, rows, IGN, row_block=16)
    assert np.allclose(got, dW[rows], atol=1e-14)
    _, _, dW_t = _torch_ref(H, W, y, dl)
    assert np.allclose(got, dW_t[rows], atol=1e-12)


# ---------------------------------------------------------------- loss variants

def _torch_variant(H, W, y, dl, eps, lam):
    Ht = torch.tensor(I.bf16_bits_to_f32(H), dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(I.bf16_bits_to_f32(W), dtype=torch.float64, requires_grad=True)
    yt = torch.tensor(y.astype(np.int64))
    Z = Ht @ Wt.T
    ce = torch.nn.functional.cross_entropy(Z, yt, ignore_index=IGN, reduction="none", label_smoothing=eps)
    valid = torch.tensor(y != IGN)
    zl = torch.where(valid, lam * torch.logsumexp(Z, dim=-1) ** 2, torch.zeros((), dtype=torch.float64))
    loss = ce + zl
    g = torch.tensor(np.where(y == IGN, 0.0, dl.astype(np.float64)))
    (loss * g).sum().backward()
    return loss.detach().numpy(), Ht.grad.numpy(), Wt.grad.numpy()


@pytest.mark.parametrize("eps,lam", [(0.1, 0.0), (0.0, 1e-2), (0.2, 3e-3)])
def test_variants_against_torch_label_smoothing_and_logsumexp(eps, lam):
    H, W, y, dl = _small(N=21, D=8, V=37, ignore=(0, 11))
    loss_t, dH_t, dW_t = _torch_variant(H, W, y, dl, eps, lam)
    loss, lse = O.forward(H, W, y, IGN, label_smoothing=eps, z_loss=lam)
    dH, dW = O.backward(H, W, y, dl, IGN, row_block=8, label_smoothing=eps, z_loss=lam)
    assert np.allclose(loss, loss_t, atol=1e-12, rtol=0)
    assert np.allclose(dH, dH_t, atol=1e-12, rtol=0)
    assert np.allclose(dW, dW_t, atol=1e-12, rtol=0)
    rows = np.array([0, 36, int(y[1])])
    assert np.allclose(O.dweight_rows(H, W, y, dl, rows, IGN, label_smoothing=eps, z_loss=lam), dW_t[rows], atol=1e-12)
    # lse itself is not affected by the variants
    assert np.array_equal(lse, O.forward(H, W, y, IGN)[1])


def test_variants_closed_form_at_zero_weight():
    """W = 0: lse = ln V and mean logit 0, so loss = ln V + lambda ln^2 V for any eps; the logit
    gradient is (1 + 2 lambda ln V)/V - eps/V - (1 - eps) onehot."""
    V, D, N = 12, 4, 5
    eps, lam = 0.25, 0.05
    H = _bits(np.random.default_rng(2).standard_normal((N, D)))
    W = np.zeros((V, D), dtype=np.uint16)
    y = np.array([0, 3, 11, IGN, 5], dtype=np.int32)
    dl = np.full(N, 0.5, dtype=np.float32)
    loss, _ = O.forward(H, W, y, IGN, label_smoothing=eps, z_loss=lam)
    lnV = math.log(V)
    for i in range(N):
        assert abs(loss[i] - (0.0 if y[i] == IGN else lnV + lam * lnV * lnV)) < 1e-13
    G = O.grad_logits(H, W, y, dl, IGN, eps, lam)
    for i in range(N):
        for v in range(V):
            want = 0.0 if y[i] == IGN else 0.5 * ((1 + 2 * lam * lnV) / V - eps / V - (1 - eps) * (v == y[i]))
            assert abs(G[i, v] - want) < 1e-14


def test_variant_gradient_row_sums():
    """Rows of the smoothed gradient still sum to zero; the z-loss adds 2 lambda lse to each row sum."""
    H, W, y, dl = _small(N=9, D=6, V=20, ignore=(4,))
    G = O.grad_logits(H, W, y, np.ones(9, np.float32), IGN, label_smoothing=0.3)
    assert np.all(np.abs(G.sum(axis=1)) < 1e-13)
    _, lse = O.forward(H, W, y, IGN)
    G = O.grad_logits(H, W, y, np.ones(9, np.float32), IGN, z_loss=0.01)
    assert np.allclose(G.sum(axis=1), 2 * 0.01 * lse, atol=1e-13)


def test_variant_finite_differences():
    H, W, y, dl = _small(N=4, D=3, V=6, ignore=(2,))
    eps, lam = 0.15, 0.02
    Hf = I.bf16_bits_to_f32(H).astype(np.float64)
    Wf = I.bf16_bits_to_f32(W).astype(np.float64)
    g = np.where(y == IGN, 0.0, dl.astype(np.float64))

    def total(Hx, Wx):
        t = 0.0
        for i in range(4):
            if y[i] == IGN:
                continue
            z = Wx @ Hx[i]
            l = math.log(np.exp(z - z.max()).sum()) + z.max()
            t += g[i] * ((1 - eps) * (l - z[y[i]]) + eps * (l - z.mean()) + lam * l * l)
        return t

    dH, dW = O.backward(H, W, y, dl, IGN, label_smoothing=eps, z_loss=lam)
    h = 1e-6
    for (i, k) in [(0, 0), (1, 2), (3, 1)]:
        Hp, Hm = Hf.copy(), Hf.copy()
        Hp[i, k] += h
        Hm[i, k] -= h
        assert abs((total(Hp, Wf) - total(Hm, Wf)) / (2 * h) - dH[i, k]) < 1e-8
    for (v, k) in [(0, 0), (int(y[0]), 1), (5, 2)]:
        Wp, Wm = Wf.copy(), Wf.copy()
        Wp[v, k] += h
        Wm[v, k] -= h
        assert abs((total(Hf, Wp) - total(Hf, Wm)) / (2 * h) - dW[v, k]) < 1e-8


def test_mean_loss_counts_only_valid_rows():
    loss = np.array([1.0, 0.0, 3.0, 0.0, 5.0])
    y = np.array([4, IGN, 2, IGN, 0], dtype=np.int32)
    m, n = O.mean_loss(loss, y, IGN)
    assert n == 3 and abs(m - 3.0) < 1e-15
    assert O.mean_loss(np.zeros(2), np.array([IGN, IGN]), IGN) == (0.0, 0)
    yt = torch.tensor(y.astype(np.int64))
    Z = torch.randn(5, 6, dtype=torch.float64, generator=torch.Generator().manual_seed(0))
    per = torch.nn.functional.cross_entropy(Z, yt, ignore_index=IGN, reduction="none").numpy()
    ref = float(torch.nn.functional.cross_entropy(Z, yt, ignore_index=IGN, reduction="mean"))
    assert abs(O.mean_loss(per, y, IGN)[0] - ref) < 1e-14


def test_widen_bf16_exact():
    vals = np.array([0.0, 1.0, -2.5, 3.140625, 2.0 ** -126, -2.0 ** 100], dtype=np.float32)
    bits = (vals.view(np.uint32) >> 16).astype(np.uint16)     # all exactly representable
    assert np.array_equal(O.widen_bf16(bits), vals.astype(np.float64))
    with pytest.raises(TypeError):
        O.widen_bf16(vals)


# ---------------------------------------------------------------- the paper's printed numbers

def test_paper_memory_figures():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_memory_figures.txt")
    unit = {"GB": 1e9, "MB": 1e6, "MiB": float(1 << 20), "x": 1.0}
    n = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, B, N, X, val, u, tol, _cite = [t.strip() for t in line.split("|")]
        B, N, X, val, tol = int(B), int(N), int(X), float(val), float(tol)
        if key == "logits_bytes":
            got = O.logit_memory_bytes(B, N, X) / unit[u]
        elif key == "chunk_bytes":
            got = O.logit_memory_bytes(B, N, X) / unit[u]
        elif key == "reduction":
            got = O.chunk_reduction_factor(151936, X)
        else:
            raise AssertionError(key)
        assert abs(got - val) / val <= tol, (key, got, val)
        n += 1
    assert n == 5

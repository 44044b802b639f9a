"""Pins for the RMSNorm and AdamW oracles: torch's own implementations (float64, CPU, autograd),
closed forms, invariants and central finite differences.  Each would fail for a plausible
mistake (a dropped mean, eps inside / outside the root, coupled instead of decoupled decay,
a wrong bias correction)."""
import math

import numpy as np
import pytest
import torch

from oracle import adamw_oracle as A
from oracle import rmsnorm_oracle as R
from paper_2601_02609_amd import inputs as I


def _bits(x):
    return I.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def _f64(bits):
    return I.bf16_bits_to_f32(bits).astype(np.float64)


def _case(N=7, D=12, seed=0):
    rng = np.random.default_rng(seed)
    x = _bits(rng.standard_normal((N, D)) * 1.7)
    gamma = _bits(1.0 + 0.3 * rng.standard_normal(D))
    dy = _bits(rng.standard_normal((N, D)) * 0.01)
    return x, gamma, dy


# ------------------------------------------------------------------ RMSNorm
def test_round_bf16_matches_torch_and_breaks_ties_to_even():
    rng = np.random.default_rng(3)
    v = (rng.standard_normal(100000) * np.exp(rng.uniform(-20, 20, 100000))).astype(np.float32).astype(np.float64)
    ref = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(R.round_bf16(v), ref)
    b = np.arange(0x3F80, 0x3FA0, dtype=np.uint32)
    lo = (b << 16).view(np.float32).astype(np.float64)
    hi = ((b + 1) << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    assert np.array_equal(R.round_bf16((lo + hi) / 2), np.where(b % 2 == 0, b, b + 1).astype(np.uint16))
    assert np.array_equal(R.round_bf16(-(lo + hi) / 2), (np.where(b % 2 == 0, b, b + 1) | 0x8000).astype(np.uint16))
    # a value a hair above a tie goes up even when float32 cannot tell it from the tie
    assert R.round_bf16(np.array([(lo[0] + hi[0]) / 2 * (1 + 2.0 ** -40)]))[0] == b[0] + 1


def test_rmsnorm_residual_form():
    """h is torch's own bf16 sum (fp32 add, one rounding); y and the gradients are those of the
    plain norm applied to h; x and the residual receive the same gradient, plus what arrives
    through the residual stream."""
    rng = np.random.default_rng(4)
    x, gamma, dy = _case(N=9, D=16, seed=5)
    res = _bits(rng.standard_normal((9, 16)) * np.exp(rng.uniform(-6, 3, (9, 16))))
    h_bits, y, rstd = R.forward_residual(x, res, gamma, 1e-5)
    tx = torch.from_numpy(x.view(np.int16)).view(torch.bfloat16)
    tr = torch.from_numpy(res.view(np.int16)).view(torch.bfloat16)
    assert np.array_equal(h_bits, (tx + tr).view(torch.int16).numpy().view(np.uint16))
    y0, rstd0 = R.forward(h_bits, gamma, 1e-5)
    assert np.array_equal(y, y0) and np.array_equal(rstd, rstd0)
    # gradient through the fused form, by autograd on float64 copies of x and residual whose sum is h
    hx = torch.tensor(_f64(h_bits) - _f64(res), requires_grad=True)
    hr = torch.tensor(_f64(res), requires_grad=True)
    gt = torch.tensor(_f64(gamma), requires_grad=True)
    h = hx + hr
    out = torch.nn.functional.rms_norm(h, (16,), gt, 1e-5)
    d_res_in = _bits(rng.standard_normal((9, 16)) * 0.02)
    (out * torch.tensor(_f64(dy))).sum().backward(retain_graph=True)
    (h * torch.tensor(_f64(d_res_in))).sum().backward()
    dh, dgamma = R.backward_residual(h_bits, gamma, dy, 1e-5, d_res_in)
    assert np.allclose(dh, hx.grad.numpy(), atol=1e-14, rtol=0) and np.allclose(dh, hr.grad.numpy(), atol=1e-14, rtol=0)
    assert np.allclose(dgamma, gt.grad.numpy(), atol=1e-14, rtol=0)
    dh0, _ = R.backward_residual(h_bits, gamma, dy, 1e-5)
    assert np.allclose(dh - dh0, _f64(d_res_in), atol=1e-15)


@pytest.mark.parametrize("eps", [1e-6, 1e-2])
def test_rmsnorm_against_torch_and_autograd(eps):
    x, gamma, dy = _case()
    xt = torch.tensor(_f64(x), requires_grad=True)
    gt = torch.tensor(_f64(gamma), requires_grad=True)
    yt = torch.nn.functional.rms_norm(xt, (x.shape[1],), gt, eps)
    yt.backward(torch.tensor(_f64(dy)))
    y, rstd = R.forward(x, gamma, eps)
    dx, dgamma = R.backward(x, gamma, dy, eps)
    assert np.allclose(y, yt.detach().numpy(), atol=1e-13, rtol=0)
    assert np.allclose(dx, xt.grad.numpy(), atol=1e-14, rtol=0)
    assert np.allclose(dgamma, gt.grad.numpy(), atol=1e-14, rtol=0)
    assert np.allclose(rstd, 1.0 / np.sqrt((_f64(x) ** 2).mean(axis=1) + eps), atol=1e-15)


def test_rmsnorm_closed_forms():
    D = 8
    # a constant row c: r = sqrt(c^2 + eps), y = gamma c / r
    x = _bits(np.full((1, D), 3.0))
    gamma = _bits(np.arange(1, D + 1, dtype=np.float32))
    y, rstd = R.forward(x, gamma, 0.25)
    r = math.sqrt(9.0 + 0.25)
    assert abs(rstd[0] - 1.0 / r) < 1e-15
    assert np.allclose(y[0], np.arange(1, D + 1) * 3.0 / r, atol=1e-14)
    # a one-hot row e_k * a: mean square a^2 / D
    x = _bits(np.eye(D)[2:3] * 4.0)
    y, rstd = R.forward(x, _bits(np.ones(D)), 0.0)
    assert abs(rstd[0] - 1.0 / math.sqrt(16.0 / D)) < 1e-15
    assert abs(y[0, 2] - math.sqrt(D)) < 1e-14 and np.count_nonzero(y[0]) == 1


def test_rmsnorm_scale_invariance_and_orthogonality():
    """eps = 0: RMSNorm(a x) = RMSNorm(x) for a > 0, hence dx is orthogonal to x."""
    x, gamma, dy = _case(N=5, D=16, seed=3)
    x2 = _bits(_f64(x) * 4.0)             # exact in bf16
    y1, _ = R.forward(x, gamma, 0.0)
    y2, _ = R.forward(x2, gamma, 0.0)
    assert np.allclose(y1, y2, atol=1e-14)
    dx, _ = R.backward(x, gamma, dy, 0.0)
    assert np.abs((dx * _f64(x)).sum(axis=1)).max() < 1e-14


def test_rmsnorm_finite_differences():
    x, gamma, dy = _case(N=3, D=5, seed=5)
    eps = 1e-3
    xf, gf, dyf = _f64(x), _f64(gamma), _f64(dy)

    def total(xx, gg):
        t = 0.0
        for i in range(3):
            r = math.sqrt(sum(xx[i, j] ** 2 for j in range(5)) / 5 + eps)
            t += sum(dyf[i, j] * xx[i, j] / r * gg[j] for j in range(5))
        return t

    dx, dgamma = R.backward(x, gamma, dy, eps)
    h = 1e-6
    for (i, j) in [(0, 0), (1, 3), (2, 4)]:
        xp, xm = xf.copy(), xf.copy()
        xp[i, j] += h
        xm[i, j] -= h
        assert abs((total(xp, gf) - total(xm, gf)) / (2 * h) - dx[i, j]) < 1e-9
    for j in [0, 2, 4]:
        gp, gm = gf.copy(), gf.copy()
        gp[j] += h
        gm[j] -= h
        assert abs((total(xf, gp) - total(xf, gm)) / (2 * h) - dgamma[j]) < 1e-9


def test_rmsnorm_printed_backward_differs_unless_gamma_is_one():
    """The listing's rstd * gamma * (g - xhat c) equals the derivative only for gamma = 1 (documents
    the reading taken in the oracle's header)."""
    x, gamma, dy = _case(N=4, D=6, seed=7)
    eps = 1e-5
    xf, gf, g = _f64(x), _f64(gamma), _f64(dy)
    rstd = 1.0 / np.sqrt((xf * xf).mean(axis=1) + eps)
    xhat = xf * rstd[:, None]
    c = (g * gf * xhat).mean(axis=1)
    printed = rstd[:, None] * gf * (g - xhat * c[:, None])
    dx, _ = R.backward(x, gamma, dy, eps)
    assert np.abs(printed - dx).max() > 1e-6
    ones = _bits(np.ones(6))
    c1 = (g * xhat).mean(axis=1)
    printed1 = rstd[:, None] * (g - xhat * c1[:, None])
    assert np.allclose(printed1, R.backward(x, ones, dy, eps)[0], atol=1e-15)


# ------------------------------------------------------------------ AdamW

def test_adamw_against_torch_over_several_steps():
    rng = np.random.default_rng(1)
    p0 = rng.standard_normal(50)
    hp = dict(lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    pt = torch.tensor(p0.copy(), requires_grad=True)
    opt = torch.optim.AdamW([pt], **hp)
    p, m, v = p0.copy(), np.zeros(50), np.zeros(50)
    for step in range(1, 6):
        g = rng.standard_normal(50) * 0.3
        pt.grad = torch.tensor(g.copy())
        opt.step()
        p, m, v = A.adamw_step(p, g, m, v, step, hp["lr"], 0.9, 0.95, hp["eps"], hp["weight_decay"])
        assert np.allclose(p, pt.detach().numpy(), atol=1e-14, rtol=0), step
    st = opt.state[pt]
    assert np.allclose(m, st["exp_avg"].numpy(), atol=1e-15)
    assert np.allclose(v, st["exp_avg_sq"].numpy(), atol=1e-15)


def test_adamw_first_step_closed_form():
    """Step 1 from zero moments: m/bc1 = g, v/bc2 = g^2, so p <- p (1 - lr wd) - lr g / (|g| + eps)."""
    p = np.array([1.0, -2.0, 0.5])
    g = np.array([0.3, -0.7, 0.0])
    lr, wd, eps = 0.01, 0.1, 1e-8
    pn, m, v = A.adamw_step(p, g, np.zeros(3), np.zeros(3), 1, lr, 0.9, 0.999, eps, wd)
    want = p * (1 - lr * wd) - lr * g / (np.abs(g) + eps)
    assert np.allclose(pn, want, atol=1e-15)
    assert np.allclose(m, 0.1 * g, atol=1e-16) and np.allclose(v, 0.001 * g * g, atol=1e-18)


def test_adamw_decay_is_decoupled():
    """With g = 0 the parameters only shrink by (1 - lr wd): the decay never meets sqrt(v)."""
    p = np.array([2.0, -4.0])
    pn, m, v = A.adamw_step(p, np.zeros(2), np.zeros(2), np.full(2, 9.0), 3, 0.1, 0.9, 0.99, 1e-8, 0.5)
    assert np.allclose(pn, p * 0.95, atol=1e-15)


def test_clip_coef_against_torch_and_closed_form():
    rng = np.random.default_rng(2)
    g1, g2 = rng.standard_normal(30), rng.standard_normal((4, 5))
    t1 = torch.zeros(30, dtype=torch.float64, requires_grad=True)
    t2 = torch.zeros(4, 5, dtype=torch.float64, requires_grad=True)
    t1.grad, t2.grad = torch.tensor(g1.copy()), torch.tensor(g2.copy())
    norm = float(torch.nn.utils.clip_grad_norm_([t1, t2], max_norm=1.5))
    c = A.clip_coef([g1, g2], 1.5, 1e-6)
    assert abs(c - min(1.0, 1.5 / (norm + 1e-6))) < 1e-15
    assert np.allclose(t1.grad.numpy(), g1 * c, atol=1e-15)
    # 3-4-5: norm 5
    assert abs(A.clip_coef([np.array([3.0]), np.array([4.0])], 1.0, 0.0) - 0.2) < 1e-16
    assert A.clip_coef([np.array([0.1])], 1.0) == 1.0
    # the clipped gradient enters the moments
    p, m, v = A.adamw_step(np.zeros(1), np.array([10.0]), np.zeros(1), np.zeros(1), 1, 0.0, 0.9, 0.999, 1e-8, 0.0, clip=0.2)
    assert abs(m[0] - 0.1 * 2.0) < 1e-15 and abs(v[0] - 0.001 * 4.0) < 1e-16

"""GPU parity of the steps around the LM head -- RMSNorm forward/backward, global-norm clipping
coefficient, fused AdamW -- against their fp64 oracles, element by element.

Tolerances, from the arithmetic: the kernels compute in fp32 and round bf16 outputs once, so a
bf16 output is within 2^-8 relative of the oracle per element (plus fp32 noise on values near 0);
fp32 outputs (rstd, dgamma, parameters, moments) within a few 1e-6 relative.
"""
import numpy as np
import pytest
import torch

from oracle import adamw_oracle as A
from oracle import rmsnorm_oracle as R
from paper_2601_02609_amd import inputs as I
from tests.gpu_util import bf16_dev, bf16_host, rel_fro

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2601_02609_amd import binding
    binding.lib()
    return binding


def _norm_case(N, D, seed):
    rng = np.random.default_rng(seed)
    x = I.f32_to_bf16_bits((rng.standard_normal((N, D)) * 1.5).astype(np.float32))
    gamma = I.f32_to_bf16_bits((1.0 + 0.2 * rng.standard_normal(D)).astype(np.float32))
    dy = I.f32_to_bf16_bits((rng.standard_normal((N, D)) * 1e-3).astype(np.float32))
    return x, gamma, dy


@pytest.mark.parametrize("shape", [(1, 64), (7, 896), (1001, 896), (300, 2048), (130, 4096), (5, 8192), (2500, 192),
                                   # several trips per workgroup with the row shared by 2 / 4 wavefronts,
                                   # a last trip only some workgroups (and only some of their rows) take
                                   (2101, 2048), (4301, 1536), (3000, 3584), (1100, 4096), (2060, 8192)])
def test_rmsnorm_matches_oracle(B, shape):
    N, D = shape
    eps = 1e-6
    x, gamma, dy = _norm_case(N, D, seed=N + D)
    print(f"[rmsnorm] N={N} D={D}", flush=True)
    y, rstd = B.cce_rmsnorm_forward(bf16_dev(x), bf16_dev(gamma), eps)
    dx, dgamma = B.cce_rmsnorm_backward(bf16_dev(x), bf16_dev(gamma), rstd, bf16_dev(dy))
    torch.cuda.synchronize()
    o_y, o_rstd = R.forward(x, gamma, eps)
    o_dx, o_dgamma = R.backward(x, gamma, dy, eps)
    assert np.abs(rstd.cpu().numpy() / o_rstd - 1.0).max() <= 2e-6
    yh, dxh = bf16_host(y), bf16_host(dx)
    # one bf16 rounding of an fp32 result: 2^-8 relative, with an absolute floor for values near zero
    assert np.all(np.abs(yh - o_y) <= 2.0 ** -8 * np.abs(o_y) + 1e-6)
    assert np.all(np.abs(dxh - o_dx) <= 2.0 ** -8 * np.abs(o_dx) + 1e-8)
    assert rel_fro(yh, o_y) <= 3e-3 and rel_fro(dxh, o_dx) <= 3e-3
    assert np.abs(dgamma.cpu().numpy() - o_dgamma).max() <= 1e-5 * np.abs(o_dgamma).max() + 1e-9


@pytest.mark.parametrize("shape", [(3, 64), (1001, 896), (130, 4096), (5, 8192), (2101, 2048), (1100, 4096)])
def test_rmsnorm_residual_form_matches_oracle(B, shape):
    """Fused residual add: the stored residual stream h is the oracle's bf16 sum bit for bit
    (byte work: one rounding of an exact or harmlessly rounded fp32 sum); y, rstd and the
    gradient of h (with a gradient arriving through the residual stream) as for the plain norm."""
    N, D = shape
    eps = 1e-6
    rng = np.random.default_rng(N * 7 + D)
    x, gamma, dy = _norm_case(N, D, seed=N + D + 1)
    res = I.f32_to_bf16_bits((rng.standard_normal((N, D)) * np.exp(rng.uniform(-8, 3, (N, D)))).astype(np.float32))
    d_res = I.f32_to_bf16_bits((rng.standard_normal((N, D)) * 2e-3).astype(np.float32))
    print(f"[rmsnorm+residual] N={N} D={D}", flush=True)
    xd, rd = bf16_dev(x), bf16_dev(res)
    y, rstd = B.cce_rmsnorm_residual_forward(xd, rd, bf16_dev(gamma), eps)
    dh, dgamma = B.cce_rmsnorm_residual_backward(rd, bf16_dev(gamma), rstd, bf16_dev(dy), bf16_dev(d_res))
    dh0, _ = B.cce_rmsnorm_residual_backward(rd, bf16_dev(gamma), rstd, bf16_dev(dy), None)
    dx_plain, _ = B.cce_rmsnorm_backward(rd, bf16_dev(gamma), rstd, bf16_dev(dy))
    torch.cuda.synchronize()
    o_h, o_y, o_rstd = R.forward_residual(x, res, gamma, eps)
    h_bits = rd.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(h_bits, o_h)
    assert np.array_equal(xd.view(torch.int16).cpu().numpy().view(np.uint16), x)          # x untouched
    assert np.abs(rstd.cpu().numpy() / o_rstd - 1.0).max() <= 2e-6
    yh = bf16_host(y)
    assert np.all(np.abs(yh - o_y) <= 2.0 ** -8 * np.abs(o_y) + 1e-6)
    o_dh, o_dgamma = R.backward_residual(o_h, gamma, dy, eps, d_res)
    dhh = bf16_host(dh)
    assert np.all(np.abs(dhh - o_dh) <= 2.0 ** -8 * np.abs(o_dh) + 1e-8)
    assert np.abs(dgamma.cpu().numpy() - o_dgamma).max() <= 1e-5 * np.abs(o_dgamma).max() + 1e-9
    assert torch.equal(dh0, dx_plain)                      # no residual gradient: the plain backward
    assert rel_fro(dhh - bf16_host(dh0), I.bf16_bits_to_f32(d_res).astype(np.float64)) <= 2e-2


def test_rmsnorm_dgamma_accumulates_and_is_reproducible(B):
    x, gamma, dy = _norm_case(700, 896, seed=3)
    xd, gd, dyd = bf16_dev(x), bf16_dev(gamma), bf16_dev(dy)
    _, rstd = B.cce_rmsnorm_forward(xd, gd, 1e-6)
    dx1, dg1 = B.cce_rmsnorm_backward(xd, gd, rstd, dyd)
    dx2, dg2 = B.cce_rmsnorm_backward(xd, gd, rstd, dyd)
    assert torch.equal(dx1, dx2) and torch.equal(dg1, dg2)
    acc = torch.ones_like(dg1)
    B.cce_rmsnorm_backward(xd, gd, rstd, dyd, dgamma=acc, accumulate_dgamma=True)
    torch.cuda.synchronize()
    assert torch.allclose(acc, dg1 + 1.0, atol=1e-6, rtol=0)


def test_rmsnorm_feeds_the_lm_head(B):
    """The normalised rows are what cce_forward consumes: unit RMS when gamma = 1."""
    x, _, _ = _norm_case(256, 896, seed=9)
    ones = I.f32_to_bf16_bits(np.ones(896, dtype=np.float32))
    y, _ = B.cce_rmsnorm_forward(bf16_dev(x), bf16_dev(ones), 0.0)
    rms = np.sqrt((bf16_host(y) ** 2).mean(axis=1))
    assert np.abs(rms - 1.0).max() <= 2e-3


def test_rmsnorm_argument_errors(B):
    L = B.lib()
    x = torch.zeros(4, 64, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(64, dtype=torch.bfloat16, device="cuda")
    y = torch.empty_like(x)
    r = torch.empty(4, device="cuda")
    assert L.cce_rmsnorm_forward(None, g.data_ptr(), 4, 64, 1e-6, y.data_ptr(), r.data_ptr(), None) == B.CCE_ERR_INVALID
    assert L.cce_rmsnorm_forward(x.data_ptr(), g.data_ptr(), 4, 48, 1e-6, y.data_ptr(), r.data_ptr(), None) == B.CCE_ERR_UNSUPPORTED
    assert L.cce_rmsnorm_forward(x.data_ptr(), g.data_ptr(), 0, 64, 1e-6, y.data_ptr(), r.data_ptr(), None) == B.CCE_ERR_INVALID


@pytest.mark.parametrize("n", [1, 3, 1000, 4099, 896 * 3001])
def test_sumsq_and_clip_coef(B, n):
    rng = np.random.default_rng(n)
    g = (rng.standard_normal(n) * 0.05).astype(np.float32)
    g2 = (rng.standard_normal(777) * 0.5).astype(np.float32)
    gd, g2d = torch.from_numpy(g).cuda(), torch.from_numpy(g2).cuda()
    s = B.cce_grad_sumsq(gd)
    assert abs(float(s.item()) / float((g.astype(np.float64) ** 2).sum()) - 1.0) <= 1e-6
    B.cce_grad_sumsq(g2d, sumsq=s, accumulate=True)
    for max_norm in (0.5, 1e6):
        c = B.cce_clip_coef(s, max_norm, 1e-6)
        want = A.clip_coef([g, g2], max_norm, 1e-6)
        assert abs(float(c.item()) - want) <= 2e-6 * want
        if max_norm == 1e6:
            assert float(c.item()) == 1.0


@pytest.mark.parametrize("n", [1, 5, 4096, 896 * 1201 + 3])
def test_adamw_matches_oracle_over_steps(B, n):
    rng = np.random.default_rng(n)
    p0 = (rng.standard_normal(n) * 0.1).astype(np.float32)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    pd = torch.from_numpy(p0.copy()).cuda()
    md, vd = torch.zeros_like(pd), torch.zeros_like(pd)
    pb = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    p, m, v = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for step in range(1, 5):
        g = (rng.standard_normal(n) * 0.02).astype(np.float32)
        clip = 0.37 if step == 2 else 1.0
        cd = torch.tensor([clip], dtype=torch.float32, device="cuda") if step % 2 == 0 else None
        B.cce_adamw_step(pd, torch.from_numpy(g).cuda(), md, vd, step, param_bf16=pb, clip_coef=cd, **hp)
        p, m, v = A.adamw_step(p, g, m, v, step, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                               clip=clip if cd is not None else 1.0)
    torch.cuda.synchronize()
    gp, gm, gv = pd.cpu().numpy().astype(np.float64), md.cpu().numpy().astype(np.float64), vd.cpu().numpy().astype(np.float64)
    # fp32 arithmetic against fp64: a few ulp per step on p, m, v
    assert np.abs(gp - p).max() <= 2e-6 * np.abs(p).max() + 1e-9
    assert np.abs(gm - m).max() <= 2e-6 * np.abs(m).max() + 1e-12
    assert np.abs(gv - v).max() <= 2e-6 * np.abs(v).max() + 1e-14
    # the bf16 copy is the fp32 parameter rounded to nearest even
    want_bits = I.f32_to_bf16_bits(pd.cpu().numpy())
    got_bits = pb.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(want_bits, got_bits)


def test_adamw_consumes_the_weight_gradient_of_the_backward(B):
    """dW of cce_backward -> clipping coefficient -> AdamW -> bf16 weights for the next forward."""
    from tests.gpu_util import dev_inputs
    w = I.make_workload(I.custom_spec(300, 128, 900, seed=31, ignore_frac=0.1))
    H, W, y = dev_inputs(w)
    loss, lse = B.cce_forward(H, W, y, -100)
    dH, dW = B.cce_backward(H, W, y, lse, torch.from_numpy(w.dloss_mean).cuda(), -100)
    s = B.cce_grad_sumsq(dW.view(-1))
    coef = B.cce_clip_coef(s, 0.01)
    master = W.float().view(-1).clone()
    m, v = torch.zeros_like(master), torch.zeros_like(master)
    Wn = torch.empty_like(W)
    B.cce_adamw_step(master, dW.view(-1), m, v, 1, lr=1e-2, weight_decay=0.0, param_bf16=Wn.view(-1), clip_coef=coef)
    loss2, _ = B.cce_forward(H, Wn, y, -100)
    torch.cuda.synchronize()
    g = dW.cpu().numpy().astype(np.float64).ravel()
    c = A.clip_coef([g], 0.01)
    p_ref, _, _ = A.adamw_step(W.float().cpu().numpy().ravel(), g, np.zeros_like(g), np.zeros_like(g), 1,
                               1e-2, 0.9, 0.999, 1e-8, 0.0, clip=c)
    assert np.abs(master.cpu().numpy() - p_ref).max() <= 1e-6
    assert float(loss2.sum()) < float(loss.sum())          # one descent step lowers the loss


def test_adamw_argument_errors(B):
    L = B.lib()
    t = torch.zeros(8, device="cuda")
    assert L.cce_adamw_step(t.data_ptr(), None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 8,
                            1e-3, 0.9, 0.999, 1e-8, 0.0, 0, None, None) == B.CCE_ERR_INVALID      # step 0
    assert L.cce_adamw_step(t.data_ptr(), None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 8,
                            1e-3, 1.0, 0.999, 1e-8, 0.0, 1, None, None) == B.CCE_ERR_INVALID      # beta1 = 1
    assert L.cce_adamw_step(None, None, t.data_ptr(), t.data_ptr(), t.data_ptr(), 8,
                            1e-3, 0.9, 0.999, 1e-8, 0.0, 1, None, None) == B.CCE_ERR_INVALID

"""Pins for the oracle's two comparison modes: the master-weight step (Sec. 3.1 "Quantization-Aware
Training with Master Weights"; Sec. 4.1 baselines) and the exact, stored-error injection of
Appendix A.  Comparators: torch's optimizers, the exact-equivalence theorem of Appendix A, and the
master-weight closed form of Appendix C."""
import numpy as np
import pytest
import torch

import oracle
from oracle import (FMT_ADDNOISE, FMT_E4M3, FMT_INT4, MODE_ECO, MODE_EXACT, MODE_MASTER, MODE_NAIVE, OPT_ADAM, OPT_SGDM,
                    ROUND_RTN, ROUND_SR, StepConfig)


@pytest.mark.parametrize("fmt", [FMT_E4M3, FMT_INT4])
def test_master_weight_step_is_the_plain_optimizer_plus_a_quantizer(o64, fmt):
    """The master copy follows torch's Adam exactly whatever the quantizer does; the quantized weights are
    q(master) (the separately pinned round-to-nearest quantizer); the momentum is not touched."""
    rng = np.random.default_rng(0)
    n, bs, T = 96, 32, 12
    theta0 = rng.standard_normal(n) * 0.05
    p = torch.nn.Parameter(torch.tensor(theta0))
    opt = torch.optim.Adam([p], lr=1e-2, betas=(0.9, 0.999), eps=1e-8)
    master = theta0.copy()
    codes, scales = o64.quantize_rtn(fmt, theta0, block_size=bs)
    m, v = np.zeros(n), np.zeros(n)
    for k in range(1, T + 1):
        g = rng.standard_normal(n) * 1e-2
        p.grad = torch.tensor(g)
        opt.step()
        cfg = StepConfig(fmt=fmt, round=ROUND_RTN, mode=MODE_MASTER, lr=1e-2, step=k, block_size=bs)
        assert o64.eco_step(cfg, n, m, v, codes=codes, scales=scales, grad_real=g, aux=master) == 0
        np.testing.assert_allclose(master, p.detach().numpy(), rtol=1e-12, atol=1e-15)
        rc, rs = o64.quantize_rtn(fmt, master, block_size=bs)
        assert np.array_equal(rc, codes) and np.array_equal(rs, scales)
    np.testing.assert_allclose(m, opt.state[p]["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(v, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-12)
    assert o64.eco_step(StepConfig(fmt=fmt, mode=MODE_MASTER), n, m, v, codes=codes, scales=scales, grad_real=g) != 0


def test_master_weight_quadratic_closed_form(o64):
    """Appendix C, master weights: E[x^2] = L eta s^2 (1+b) / (2(1+b) - L eta (1-b)) for the master iterate and
    E[x^2] + s^2 for the quantized one (x^ = x + xi, gradient taken at x^)."""
    rng = np.random.default_rng(1)
    L, sigma, beta, eta = 1.0, 0.01, 0.9, 0.2
    n, burn, T = 8192, 1500, 1500
    u = L * eta * sigma ** 2 * (1 + beta) / (2 * (1 + beta) - L * eta * (1 - beta))
    x = np.zeros(n)                       # master
    xq = rng.standard_normal(n) * sigma   # quantized
    m = np.zeros(n)
    acc_m = acc_q = 0.0
    for k in range(1, burn + T + 1):
        xi = rng.standard_normal(n) * sigma
        g = L * xq
        cfg = StepConfig(fmt=FMT_ADDNOISE, opt=OPT_SGDM, mode=MODE_MASTER, lr=eta, beta1=beta, step=k)
        assert o64.eco_step(cfg, n, m, None, wreal=xq, grad_real=g, xi=xi, aux=x) == 0
        if k > burn:
            acc_m += float(np.mean(x * x))
            acc_q += float(np.mean(xq * xq))
    assert abs(acc_m / T / u - 1) < 0.04
    assert abs(acc_q / T / (u + sigma ** 2) - 1) < 0.04


@pytest.mark.parametrize("fmt", [FMT_E4M3, FMT_INT4])
@pytest.mark.parametrize("rnd", [ROUND_RTN, ROUND_SR])
def test_exact_injection_reproduces_master_weight_sgdm(o64, fmt, rnd):
    """Appendix A (exact equivalence): with e_0 = theta_0 - q(theta_0) and m_0 = m_0^MW - e_0/(eta beta), SGDM
    without master weights and with m <- m~ + e_t/eta - e_{t+1}/(eta beta) produces the same quantized
    iterates as SGDM with master weights; theta^ + e is the master copy and m + e/(eta beta) its momentum."""
    rng = np.random.default_rng(2)
    n, bs, T, lr, beta = 64, 16, 60, 0.05, 0.9
    theta0 = rng.standard_normal(n) * 0.3
    m0 = rng.standard_normal(n) * 0.1
    A = rng.standard_normal(n) * 0.5 + 1.0          # gradient of a separable quadratic, taken at the QUANTIZED iterate
    bvec = rng.standard_normal(n) * 0.1

    # master-weight run
    master = theta0.copy()
    c_mw, s_mw = o64.quantize_rtn(fmt, theta0, block_size=bs)
    m_mw = m0.copy()
    # injected run
    c_im, s_im = o64.quantize_rtn(fmt, theta0, block_size=bs)
    err = theta0 - o64.dequantize(fmt, c_im, s_im, n, bs)
    m_im = m0 - err / (lr * beta)
    moved = 0
    for k in range(1, T + 1):
        q_mw = o64.dequantize(fmt, c_mw, s_mw, n, bs)
        q_im = o64.dequantize(fmt, c_im, s_im, n, bs)
        # same codes; the two scales are the same real number computed along two routes (last-bit differences)
        assert np.array_equal(c_mw, c_im), k
        np.testing.assert_allclose(q_im, q_mw, rtol=1e-12, atol=0)
        g = A * q_mw + bvec
        before = c_mw.copy()
        common = dict(fmt=fmt, opt=OPT_SGDM, round=rnd, lr=lr, beta1=beta, step=k, seed=11, tensor_id=4, block_size=bs)
        assert o64.eco_step(StepConfig(mode=MODE_MASTER, **common), n, m_mw, None, codes=c_mw, scales=s_mw,
                            grad_real=g, aux=master) == 0
        assert o64.eco_step(StepConfig(mode=MODE_EXACT, **common), n, m_im, None, codes=c_im, scales=s_im,
                            grad_real=g, aux=err) == 0
        moved += int(np.any(before != c_mw))
        np.testing.assert_allclose(o64.dequantize(fmt, c_im, s_im, n, bs) + err, master, rtol=0, atol=1e-12)
        np.testing.assert_allclose(m_im + err / (lr * beta), m_mw, rtol=0, atol=1e-10)
    assert moved > 5
    assert np.array_equal(c_mw, c_im)

    # the memory-free rule (Alg. 2) is NOT this: it replaces e_t by e_{t+1}; same start, different iterates
    c_eco, s_eco = o64.quantize_rtn(fmt, theta0, block_size=bs)
    m_eco = m0.copy()
    for k in range(1, 11):
        g = A * o64.dequantize(fmt, c_eco, s_eco, n, bs) + bvec
        cfg = StepConfig(fmt=fmt, opt=OPT_SGDM, round=rnd, mode=MODE_ECO, lr=lr, beta1=beta, step=k, seed=11,
                         tensor_id=4, block_size=bs)
        assert o64.eco_step(cfg, n, m_eco, None, codes=c_eco, scales=s_eco, grad_real=g) == 0
    assert np.all(np.isfinite(m_eco))


def test_exact_injection_is_sgdm_only(o64):
    n = 32
    codes, scales = o64.quantize_rtn(FMT_E4M3, np.ones(n), block_size=32)
    m, v, e, g = np.zeros(n), np.zeros(n), np.zeros(n), np.zeros(n)
    assert o64.eco_step(StepConfig(opt=OPT_ADAM, mode=MODE_EXACT, block_size=32), n, m, v, codes=codes, scales=scales,
                        grad_real=g, aux=e) != 0
    assert o64.eco_step(StepConfig(opt=OPT_SGDM, mode=MODE_EXACT, block_size=32), n, m, None, codes=codes,
                        scales=scales, grad_real=g, aux=None) != 0
    assert o64.eco_step(StepConfig(opt=OPT_SGDM, mode=MODE_EXACT, block_size=32), n, m, None, codes=codes,
                        scales=scales, grad_real=g, aux=e) == 0

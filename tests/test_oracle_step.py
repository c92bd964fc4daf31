"""Pins for the oracle's optimizer step (Alg. 1-3 of the paper).

Nothing here compares the oracle with itself only: the comparators are torch's
own Adam / SGD (library routines), identities the paper proves (Lemma 3.4 and
the one-step relation in its proof, which hold for ANY quantizer), the
closed-form stationary moments of Appendix C, and exact rational arithmetic.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import (FMT_ADDNOISE, FMT_BF16_PLAIN, FMT_E4M3, FMT_IDENTITY, FMT_INT4, OPT_ADAM, OPT_SGDM, ROUND_RTN,
                    ROUND_SR, StepConfig)


def torch_adam_reference(theta0, grads, lr, b1, b2, eps, wd=0.0, m0=None, v0=None, k0=0):
    """Plain Adam(W) by torch.optim in float64, optionally resumed from (m0, v0) after k0 steps."""
    p = torch.nn.Parameter(torch.tensor(theta0, dtype=torch.float64))
    cls = torch.optim.AdamW if wd else torch.optim.Adam
    opt = cls([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    if m0 is not None:
        opt.state[p] = {"step": torch.tensor(float(k0)), "exp_avg": torch.tensor(m0, dtype=torch.float64).clone(),
                        "exp_avg_sq": torch.tensor(v0, dtype=torch.float64).clone()}
    for g in grads:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
    st = opt.state[p]
    return p.detach().numpy().copy(), st["exp_avg"].numpy().copy(), st["exp_avg_sq"].numpy().copy()


def test_identity_quantizer_is_plain_adam(o64, o32):
    """With q = id the error is zero and the injection adds nothing (Alg. 3): the step is Adam.
    Note torch divides sqrt(v) by sqrt(1-b2^k) where the paper divides v by (1-b2^k): same value."""
    rng = np.random.default_rng(0)
    n, T = 257, 25
    theta0 = rng.standard_normal(n) * 0.02
    grads = [rng.standard_normal(n) * 1e-3 * (1 + k % 3) for k in range(T)]
    lr, b1, b2, eps = 1e-3, 0.9, 0.999, 1e-8
    ref_t, ref_m, ref_v = torch_adam_reference(theta0, grads, lr, b1, b2, eps)

    for o, tol in ((o64, 1e-12), (o32, 2e-5)):
        w = theta0.astype(o.dtype).copy()
        m = np.zeros(n, o.dtype)
        v = np.zeros(n, o.dtype)
        for k, g in enumerate(grads, start=1):
            cfg = StepConfig(fmt=FMT_IDENTITY, lr=lr, beta1=b1, beta2=b2, eps=eps, step=k, block_size=64)
            err = np.ones(n, o.dtype)
            assert o.eco_step(cfg, n, m, v, wreal=w, grad_real=g.astype(o.dtype), dbg_err=err) == 0
            assert np.all(err == 0)
        np.testing.assert_allclose(w, ref_t, rtol=tol, atol=tol * 1e-2)
        np.testing.assert_allclose(m, ref_m, rtol=tol, atol=tol * 1e-5)
        np.testing.assert_allclose(v, ref_v, rtol=tol, atol=tol * 1e-8)


def test_identity_quantizer_with_decoupled_decay_is_adamw(o64):
    rng = np.random.default_rng(1)
    n, T = 64, 10
    theta0 = rng.standard_normal(n)
    grads = [rng.standard_normal(n) * 1e-2 for _ in range(T)]
    ref_t, ref_m, ref_v = torch_adam_reference(theta0, grads, 1e-2, 0.9, 0.98, 1e-9, wd=0.1)
    w, m, v = theta0.copy(), np.zeros(n), np.zeros(n)
    for k, g in enumerate(grads, start=1):
        cfg = StepConfig(fmt=FMT_IDENTITY, lr=1e-2, beta1=0.9, beta2=0.98, eps=1e-9, weight_decay=0.1, step=k)
        assert o64.eco_step(cfg, n, m, v, wreal=w, grad_real=g) == 0
    np.testing.assert_allclose(w, ref_t, rtol=1e-12)
    np.testing.assert_allclose(m, ref_m, rtol=1e-12)


def test_identity_quantizer_is_plain_sgdm(o64):
    """EMA-form momentum m = b m + (1-b) g (Eq. m_tilde) is torch SGD with dampening = b."""
    rng = np.random.default_rng(2)
    n, T, lr, beta = 50, 30, 0.05, 0.9
    theta0 = rng.standard_normal(n)
    grads = [rng.standard_normal(n) for _ in range(T)]
    p = torch.nn.Parameter(torch.tensor(theta0))
    opt = torch.optim.SGD([p], lr=lr, momentum=beta, dampening=beta)
    opt.state[p]["momentum_buffer"] = torch.zeros(n, dtype=torch.float64)   # start from m = 0, not from g
    w, m = theta0.copy(), np.zeros(n)
    for k, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g)
        opt.step()
        cfg = StepConfig(fmt=FMT_IDENTITY, opt=OPT_SGDM, lr=lr, beta1=beta, step=k)
        assert o64.eco_step(cfg, n, m, None, wreal=w, grad_real=g) == 0
    np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12)
    np.testing.assert_allclose(m, opt.state[p]["momentum_buffer"].numpy(), rtol=1e-12)


@pytest.mark.parametrize("fmt", [FMT_E4M3, FMT_INT4])
@pytest.mark.parametrize("rnd", [ROUND_SR, ROUND_RTN])
def test_sgdm_virtual_sequence_invariant(o64, fmt, rnd):
    """Lemma 3.4: theta_t := theta^_t - (eta b/(1-b)) m^_t obeys theta_{t+1} = theta_t - eta g_t
    exactly, whatever the quantizer.  Summed over T steps this fixes sign and size of alpha."""
    rng = np.random.default_rng(3)
    n, bs, T, lr, beta = 64, 8, 100, 0.02, 0.9
    C = lr * beta / (1 - beta)
    x0 = rng.standard_normal(n) * 0.5
    codes, scales = o64.quantize_rtn(fmt, x0, block_size=bs)
    m = rng.standard_normal(n) * 0.1
    virt0 = o64.dequantize(fmt, codes, scales, n, bs) - C * m
    gsum = np.zeros(n)
    changed = 0
    for k in range(1, T + 1):
        g = rng.standard_normal(n)
        gsum += g
        before = codes.copy()
        cfg = StepConfig(fmt=fmt, opt=OPT_SGDM, round=rnd, lr=lr, beta1=beta, step=k, seed=17, block_size=bs)
        assert o64.eco_step(cfg, n, m, None, codes=codes, scales=scales, grad_real=g) == 0
        changed += int(np.any(before != codes))
    virt = o64.dequantize(fmt, codes, scales, n, bs) - C * m
    np.testing.assert_allclose(virt - virt0, -lr * gsum, rtol=0, atol=1e-11)
    assert changed >= 5                          # the weights really moved on the grid

    # without injection the invariant must fail (the test has teeth)
    codes, scales = o64.quantize_rtn(fmt, x0, block_size=bs)
    m = np.zeros(n)
    virt0 = o64.dequantize(fmt, codes, scales, n, bs)
    gsum[:] = 0
    for k in range(1, 21):
        g = rng.standard_normal(n)
        gsum += g
        cfg = StepConfig(fmt=fmt, opt=OPT_SGDM, round=rnd, inject=False, lr=lr, beta1=beta, step=k, seed=17,
                         block_size=bs)
        assert o64.eco_step(cfg, n, m, None, codes=codes, scales=scales, grad_real=g) == 0
    virt = o64.dequantize(fmt, codes, scales, n, bs) - C * m
    assert np.abs(virt - virt0 + lr * gsum).max() > 1e-4


@pytest.mark.parametrize("fmt", [FMT_E4M3, FMT_INT4])
def test_sgdm_one_step_relation(o64, fmt):
    """Proof of Lemma 3.4: theta^_{t+1} = theta^_t - eta m^_{t+1} - e_{t+1}/beta."""
    rng = np.random.default_rng(4)
    n, bs, lr, beta = 32, 8, 0.1, 0.8
    x0 = rng.standard_normal(n)
    codes, scales = o64.quantize_rtn(fmt, x0, block_size=bs)
    th_hat = o64.dequantize(fmt, codes, scales, n, bs)
    m = rng.standard_normal(n)
    g = rng.standard_normal(n)
    e = np.zeros(n)
    tt = np.zeros(n)
    cfg = StepConfig(fmt=fmt, opt=OPT_SGDM, lr=lr, beta1=beta, step=1, seed=5, block_size=bs)
    m_in = m.copy()
    assert o64.eco_step(cfg, n, m, None, codes=codes, scales=scales, grad_real=g, dbg_err=e, dbg_theta=tt) == 0
    new_hat = o64.dequantize(fmt, codes, scales, n, bs)
    np.testing.assert_allclose(new_hat, th_hat - lr * m - e / beta, atol=1e-12)
    # and the pieces are what Eqs. (m_tilde)-(error) say they are
    m_tilde = beta * m_in + (1 - beta) * g
    np.testing.assert_allclose(tt, th_hat - lr * m_tilde, atol=1e-14)
    np.testing.assert_allclose(e, tt - new_hat, atol=1e-14)
    assert np.abs(e).max() > 1e-3


@pytest.mark.parametrize("fmt,rho", [(FMT_E4M3, 448.0), (FMT_INT4, 7.0)])
@pytest.mark.parametrize("rnd", [ROUND_SR, ROUND_RTN])
def test_adam_eco_step_against_library_adam(o64, fmt, rho, rnd):
    """One Adam-ECO step from a mid-training state, taken apart with torch's Adam as comparator:
    theta~ and v are the plain Adam results from theta^; the new weights are grid neighbours of
    theta~ on the new abs-max scale; and the element-wise analogue of the one-step relation holds,
    theta^' = theta^ - eta_t m^' - e/beta1 with eta_t the adaptive step of Sec. 3.2."""
    rng = np.random.default_rng(5)
    n, bs, k = 64, 16, 7
    lr, b1, b2, eps = 1e-2, 0.9, 0.999, 1e-8
    x0 = rng.standard_normal(n) * 0.05
    codes, scales = o64.quantize_rtn(fmt, x0, block_size=bs)
    th_hat = o64.dequantize(fmt, codes, scales, n, bs)
    m0 = rng.standard_normal(n) * 1e-2
    v0 = rng.uniform(0.5, 2.0, n) * 1e-4
    g = rng.standard_normal(n) * 1e-2
    ref_t, ref_m, ref_v = torch_adam_reference(th_hat, [g], lr, b1, b2, eps, m0=m0, v0=v0, k0=k - 1)

    m, v = m0.copy(), v0.copy()
    e, tt = np.zeros(n), np.zeros(n)
    cfg = StepConfig(fmt=fmt, round=rnd, lr=lr, beta1=b1, beta2=b2, eps=eps, step=k, seed=9, block_size=bs)
    assert o64.eco_step(cfg, n, m, v, codes=codes, scales=scales, grad_real=g, dbg_err=e, dbg_theta=tt) == 0
    new_hat = o64.dequantize(fmt, codes, scales, n, bs)

    np.testing.assert_allclose(tt, ref_t, rtol=1e-12, atol=1e-15)       # OPTIM_STEP is Adam
    np.testing.assert_allclose(v, ref_v, rtol=1e-13)                    # v is returned unchanged by ECO_QUANTIZE
    np.testing.assert_allclose(e, tt - new_hat, atol=1e-15)
    table = np.abs(o64.decode_table(fmt))
    grid = np.unique(table[~np.isnan(table)])
    grid = grid[grid <= rho]
    for b in range(n // bs):
        sl = slice(b * bs, (b + 1) * bs)
        a = np.abs(tt[sl]).max()
        np.testing.assert_allclose(scales[b], a / rho, rtol=1e-15)
        y = np.abs(tt[sl]) / scales[b]
        got = np.abs(new_hat[sl]) / scales[b]
        for yy, gg in zip(y, got):
            j = np.searchsorted(grid, min(yy, rho), side="right") - 1
            nb = {grid[j], grid[min(j + 1, grid.size - 1)]}
            assert any(abs(gg - c) < 1e-9 for c in nb), (yy, gg, nb)
        assert np.isclose(np.abs(new_hat[sl]).max(), a, rtol=1e-12)     # the largest element lands on rho
    d = np.sqrt(ref_v / (1 - b2 ** k)) + eps
    eta_t = lr / ((1 - b1 ** k) * d)
    np.testing.assert_allclose(new_hat, th_hat - eta_t * m - e / b1, atol=1e-13)
    # which is Alg. 3's injection, m^ = m~ + (1/eta_t)(1 - 1/b1) e, in another form
    np.testing.assert_allclose(m - ref_m, (1 / eta_t) * (1 - 1 / b1) * e, rtol=1e-9, atol=1e-16)
    assert np.abs(e).max() > 0

    # naive master-weight removal: same step, momentum left alone
    codes2, scales2 = o64.quantize_rtn(fmt, x0, block_size=bs)
    m2, v2 = m0.copy(), v0.copy()
    cfg.inject = False
    assert o64.eco_step(cfg, n, m2, v2, codes=codes2, scales=scales2, grad_real=g) == 0
    np.testing.assert_allclose(m2, ref_m, rtol=1e-13)
    assert np.array_equal(codes2, codes) and np.array_equal(scales2, scales)


def test_bookkeeping_in_exact_rationals(o32):
    """8-element tensors, block sizes 8 and 4, fp32 build: take the step apart with exact rational
    arithmetic on the fp32 outputs.  Every relation below holds up to the rounding of the few
    fp32 operations between the quantities it links."""
    rng = np.random.default_rng(6)
    table = o32.decode_table(FMT_E4M3)
    for bs in (8, 4):
        for trial in range(20):
            x0 = (rng.standard_normal(8) * 0.02).astype(np.float32)
            codes, scales = o32.quantize_rtn(FMT_E4M3, x0, block_size=bs)
            th_hat = o32.dequantize(FMT_E4M3, codes, scales, 8, bs)
            m0 = (rng.standard_normal(8) * 1e-3).astype(np.float32)
            v0 = (rng.uniform(0.5, 2, 8) * 1e-6).astype(np.float32)
            gb = torch.tensor(rng.standard_normal(8) * 1e-3).to(torch.bfloat16)
            g16 = gb.view(torch.int16).numpy().view(np.uint16).copy()
            g = gb.float().numpy()
            lr, b1, b2, eps, k = 1e-3, 0.9, 0.999, 1e-8, 3
            m, v = m0.copy(), v0.copy()
            e, tt = np.zeros(8, np.float32), np.zeros(8, np.float32)
            cfg = StepConfig(lr=lr, beta1=b1, beta2=b2, eps=eps, step=k, seed=trial, block_size=bs)
            assert o32.eco_step(cfg, 8, m, v, codes=codes, scales=scales, grad_bf16=g16, dbg_err=e, dbg_theta=tt) == 0
            F = lambda a: [Fraction(float(t)) for t in a]
            Fm0, Fv0, Fg, Fth, Ftt, Fe, Fm, Fv = map(F, (m0, v0, g, th_hat, tt, e, m, v))
            B1, B2, LR, EPS = Fraction(b1), Fraction(b2), Fraction(lr), Fraction(eps)
            bc1, bc2 = 1 - B1 ** k, 1 - B2 ** k
            for i in range(8):
                mt = B1 * Fm0[i] + (1 - B1) * Fg[i]
                vt = B2 * Fv0[i] + (1 - B2) * Fg[i] ** 2
                assert abs(Fv[i] - vt) <= abs(vt) * Fraction(3, 2 ** 24)
                d = Fraction(float(np.sqrt(float(vt / bc2)))) + EPS
                th = Fth[i] - LR / bc1 * mt / d
                assert abs(Ftt[i] - th) <= abs(th) * Fraction(1, 2 ** 22) + Fraction(1, 10 ** 9)
                s_new = Fraction(float(scales[i // bs]))
                q = Fraction(float(table[codes[i]])) * s_new
                assert abs((Ftt[i] - q) - Fe[i]) <= abs(Ftt[i]) * Fraction(1, 2 ** 22)      # e = theta~ - theta^'
                inj = (bc1 / LR) * (1 - 1 / B1) * d * Fe[i]
                assert abs(Fm[i] - (mt + inj)) <= (abs(mt) + abs(inj)) * Fraction(3, 2 ** 21)   # ~12 fp32 roundings
                assert inj == 0 or (inj > 0) == (Fe[i] < 0)                                  # kappa < 0
            for b in range(8 // bs):
                blk = Ftt[b * bs:(b + 1) * bs]
                a = max(abs(t) for t in blk)
                assert abs(Fraction(float(scales[b])) * 448 - a) <= a * Fraction(1, 2 ** 23)
                kmax = max(range(bs), key=lambda j: abs(blk[j]))
                assert codes[b * bs + kmax] & 0x7F == 0x7E


def test_quadratic_stationary_moments(o64):
    """Appendix C: f(x) = L x^2/2, q(x) = x + xi with E xi^2 = sigma^2.  Stationary E[x^2] of the
    quantized iterate: ECO 2 s^2 / (2(1-b^2) - L eta (1-b)^2); naive removal
    s^2 ((1-b^2) + 2 b L eta) / (L eta (2(1-b^2) - L eta (1-b)^2))."""
    rng = np.random.default_rng(8)
    L, sigma, beta = 1.0, 0.01, 0.9
    n, burn, T = 8192, 1500, 1500
    for eta in (0.2, 0.05):
        den = 2 * (1 - beta ** 2) - L * eta * (1 - beta) ** 2
        closed = {True: 2 * sigma ** 2 / den,
                  False: sigma ** 2 * ((1 - beta ** 2) + 2 * beta * L * eta) / (L * eta * den)}
        for inject in (True, False):
            x = np.zeros(n)
            m = np.zeros(n)
            acc = 0.0
            for k in range(1, burn + T + 1):
                xi = rng.standard_normal(n) * sigma
                g = L * x
                cfg = StepConfig(fmt=FMT_ADDNOISE, opt=OPT_SGDM, inject=inject, lr=eta, beta1=beta, step=k)
                assert o64.eco_step(cfg, n, m, None, wreal=x, grad_real=g, xi=xi) == 0
                if k > burn:
                    acc += float(np.mean(x * x))
            est = acc / T
            assert abs(est / closed[inject] - 1) < 0.04, (eta, inject, est, closed[inject])
    # Sec. 3.4: at the smaller learning rate naive removal is already well above ECO (it grows like 1/eta)
    assert closed[False] / closed[True] > 2.5


def test_elem_offset_and_threads_do_not_change_results(o32):
    """A span stepped on its own, with its offset in the tensor, gives the same bytes as the same
    span stepped as part of the whole tensor; and the thread count is irrelevant."""
    rng = np.random.default_rng(9)
    n = 128 * 9 + 40                                  # ragged tail
    x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    g16 = (rng.integers(0, 2 ** 16, n).astype(np.uint16) & 0xBFFF) | 0x3000     # finite, |g| ~ 1e-10..2
    g16 = (g16 & 0x8FFF) | 0x3000
    cfg = StepConfig(step=4, seed=123, tensor_id=3)

    def run(lo, hi, threads):
        o32.set_threads(threads)
        codes, scales = o32.quantize_rtn(FMT_E4M3, x0)
        c, s = codes[lo:hi].copy(), scales[lo // 128:(hi + 127) // 128].copy()
        m = np.full(hi - lo, 1e-4, np.float32)
        v = np.full(hi - lo, 1e-8, np.float32)
        cc = StepConfig(**{**cfg.__dict__, "elem_offset": lo})
        assert o32.eco_step(cc, hi - lo, m, v, codes=c, scales=s, grad_bf16=g16[lo:hi].copy()) == 0
        return c, s, m, v

    full = run(0, n, 8)
    one = run(0, n, 1)
    for a, b in zip(full, one):
        assert np.array_equal(a, b)
    part = run(256, 768, 3)
    assert np.array_equal(part[0], full[0][256:768]) and np.array_equal(part[1], full[1][2:6])
    assert np.array_equal(part[2], full[2][256:768]) and np.array_equal(part[3], full[3][256:768])
    tail = run(1024, n, 2)
    assert np.array_equal(tail[0], full[0][1024:]) and np.array_equal(tail[2], full[2][1024:])
    o32.set_threads(8)


def test_bf16_plain_is_adam_with_bf16_weights(o32):
    """Norm weights are not quantized (Sec. 4.2: the method is applied to linear layers only):
    ordinary Adam, weights rounded to bfloat16 on store, momentum untouched."""
    rng = np.random.default_rng(10)
    n = 512
    w0 = torch.tensor(1 + rng.standard_normal(n) * 0.1).to(torch.bfloat16).float().numpy()
    g = torch.tensor(rng.standard_normal(n) * 1e-3).to(torch.bfloat16)
    g16 = g.view(torch.int16).numpy().view(np.uint16).copy()
    ref_t, ref_m, ref_v = torch_adam_reference(w0, [g.double().numpy()], 1e-3, 0.9, 0.999, 1e-8)
    w, m, v = w0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    cfg = StepConfig(fmt=FMT_BF16_PLAIN, step=1)
    assert o32.eco_step(cfg, n, m, v, wreal=w, grad_bf16=g16) == 0
    np.testing.assert_allclose(m, ref_m, rtol=1e-6)
    np.testing.assert_allclose(v, ref_v, rtol=1e-6)
    want = torch.tensor(ref_t).to(torch.bfloat16).float().numpy()
    # equal to the bf16 rounding of exact Adam except where fp32 rounding sits on a bf16 tie
    assert (w != want).mean() < 0.01
    assert np.all(np.abs(w - ref_t) <= np.abs(ref_t) * 2.0 ** -8)


def test_bf16_state_and_scale(o32):
    """bf16 optimizer state and bf16 scales: every stored value is a bfloat16, and the stored
    scale is the bfloat16 nearest to max|theta~|/rho."""
    rng = np.random.default_rng(11)
    n = 256
    x0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    codes, scales = o32.quantize_rtn(FMT_INT4, x0, scale_bf16=True)
    isbf = lambda a: not np.any(np.ascontiguousarray(a, np.float32).view(np.uint32) & 0xFFFF)
    assert isbf(scales)
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    g16 = torch.tensor(rng.standard_normal(n) * 1e-4).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    tt = np.zeros(n, np.float32)
    cfg = StepConfig(fmt=FMT_INT4, lr=1e-5, state_bf16=True, scale_bf16=True, step=1, seed=2)
    assert o32.eco_step(cfg, n, m, v, codes=codes, scales=scales, grad_bf16=g16, dbg_theta=tt) == 0
    assert isbf(m) and isbf(v) and isbf(scales)
    for b in range(2):
        a = np.abs(tt[b * 128:(b + 1) * 128]).max()
        want = torch.tensor(np.float32(a) / np.float32(7)).to(torch.bfloat16).float().item()
        assert scales[b] == want


def test_invalid_arguments_are_rejected(o32):
    n = 128
    codes, scales = o32.quantize_rtn(FMT_E4M3, np.ones(n, np.float32))
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    g = np.zeros(n, np.uint16)
    ok = StepConfig()
    assert o32.eco_step(ok, n, m, v, codes=codes, scales=scales, grad_bf16=g) == 0
    for bad in (dict(step=0), dict(lr=0.0), dict(beta1=0.0), dict(beta1=1.0), dict(block_size=0),
                dict(elem_offset=64)):
        cfg = StepConfig(**{**ok.__dict__, **bad})
        assert o32.eco_step(cfg, n, m, v, codes=codes, scales=scales, grad_bf16=g) != 0, bad
    assert o32.eco_step(ok, n, m, None, codes=codes, scales=scales, grad_bf16=g) != 0
    assert o32.eco_step(ok, n, m, v, codes=None, scales=scales, grad_bf16=g) != 0


@pytest.mark.parametrize("fmt,rho", [(FMT_E4M3, 448.0), (FMT_INT4, 7.0)])
def test_step_gives_every_element_its_documented_random_field(o32, fmt, rho):
    """Inside the step, element i of the tensor (span offset included) rounds with the 16-bit field i & 7 of
    Philox call q = i >> 3, counter (q, step, tensor_id), key = seed: the new codes are recomputed here from
    theta~ with an independent big-integer Philox and the separately pinned encoder."""
    from test_oracle_random import philox_bigint
    rng = np.random.default_rng(11)
    n, bs, off = 96, 32, 64
    seed, step, tid = 0xFEDCBA9876543210, 5, 9
    w0 = (rng.standard_normal(n) * 0.05).astype(np.float32)
    codes, scales = o32.quantize_rtn(fmt, w0, block_size=bs)
    g = (rng.standard_normal(n) * 1e-2).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (rng.random(n) * 1e-4).astype(np.float32)
    theta = np.zeros(n, np.float32)
    cfg = StepConfig(fmt=fmt, opt=OPT_ADAM, round=ROUND_SR, block_size=bs, lr=1e-2, step=step, seed=seed,
                     tensor_id=tid, elem_offset=off)
    assert o32.eco_step(cfg, n, m, v, codes=codes, scales=scales, grad_real=g, dbg_theta=theta) == 0
    r16 = np.zeros(n, np.uint16)
    for i in range(n):
        gi = off + i
        words = philox_bigint([gi >> 3, 0, step, tid], [seed & 0xFFFFFFFF, seed >> 32])
        word = words[(gi & 7) >> 1]
        r16[i] = (word >> 16) if gi & 1 else (word & 0xFFFF)
    expect = np.zeros(n, np.uint8)
    for b in range(n // bs):
        th = theta[b * bs:(b + 1) * bs]
        inv = np.float32(rho) / np.abs(th).max()
        expect[b * bs:(b + 1) * bs] = o32.encode(fmt, ROUND_SR, (th * inv).astype(np.float32), r16[b * bs:(b + 1) * bs])
    got = codes if fmt == FMT_E4M3 else np.stack([codes & 15, codes >> 4], axis=1).reshape(-1)[:n]
    assert np.array_equal(got, expect)
    # the decision really depends on the field: other random bits give other codes somewhere
    assert not np.array_equal(o32.encode(fmt, ROUND_SR, (theta * (np.float32(rho) / np.abs(theta[:bs]).max())).astype(np.float32)[:bs],
                                         np.roll(r16[:bs], 1)), expect[:bs])

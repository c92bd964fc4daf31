"""Pins for the oracle's bfloat16 branches (the INT4 fine-tuning configuration keeps bf16 scales and bf16
optimizer state).

bf16 scales.  Sec. 3.1 defines the scale as s = max|x|/rho and the reconstruction as x^ = s*y: the codes y
belong to the scale that is STORED.  With a bf16 scale the stored value s' = bf16(max|x|/rho) differs from
max|x|/rho, so the codes are round(x * fl(1/s')) -- relative to s', not to the unrounded quotient -- and when
s' was rounded down the largest element lands beyond rho and saturates.  The test recomputes every code in
exact rational arithmetic from theta~ and the stored scale.

bf16 state.  Alg. 3 computes d and m^ from m~ and v~ (lines 1-5) and returns them (line 6); storing in bf16 is
one rounding of the returned values.  So a step with bf16 state must produce the same theta~, codes, scales and
error as the same step with fp32 state, and its stored m and v must be the nearest-even bf16 of the fp32 step's
m and v (torch's cast is the library routine that says what "nearest-even bf16" is).
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import FMT_E4M3, FMT_INT4, OPT_ADAM, OPT_SGDM, ROUND_RTN, ROUND_SR, StepConfig


def rn_f32(fr: Fraction) -> np.float32:
    """The fp32 nearest to an exact rational (ties to the even significand)."""
    c = np.float32(float(fr))
    cands = [np.nextafter(c, np.float32(-np.inf)), c, np.nextafter(c, np.float32(np.inf))]
    best = min(cands, key=lambda x: (abs(Fraction(float(x)) - fr), int(np.float32(x).view(np.uint32)) & 1))
    return np.float32(best)


def bf16_nearest(x) -> np.ndarray:
    return torch.tensor(np.asarray(x, np.float32)).to(torch.bfloat16).float().numpy()


def grid_of(fmt):
    """Non-negative grid magnitudes, from the format definitions (OCP E4M3: bias 7, subnormals, max 448)."""
    if fmt == FMT_INT4:
        return [Fraction(k) for k in range(8)]
    g = []
    for code in range(127):
        E, M = code >> 3, code & 7
        g.append(Fraction(M, 512) if E == 0 else Fraction(8 + M, 8) * Fraction(2) ** (E - 7))
    return g


def exact_code(grid, y: np.float32, rnd, r16: int) -> int:
    """Signed grid index of round(y): nearest with ties to the even index, or the centred 16-bit stochastic rule."""
    ay = abs(Fraction(float(y)))
    neg = bool(np.signbit(y))
    if ay >= grid[-1]:
        j = len(grid) - 1
    else:
        j = max(i for i, gv in enumerate(grid) if gv <= ay)
        lo, hi = grid[j], grid[j + 1]
        if rnd == ROUND_RTN:
            below, above = ay - lo, hi - ay
            j += int(below > above or (below == above and j & 1))
        else:
            F = round((ay - lo) / (hi - lo) * 2 ** 20)
            j += int(F + 16 * r16 + 8 >= 2 ** 20)
    return -j if neg else j


def stored_index(fmt, codes, n):
    """Signed grid index of every stored code."""
    if fmt == FMT_E4M3:
        c = codes[:n].astype(np.int64)
        return np.where(c & 0x80, -(c & 0x7F), c & 0x7F)
    nib = np.stack([codes & 15, codes >> 4], axis=1).reshape(-1)[:n].astype(np.int64)
    return np.where(nib & 8, nib - 16, nib)


@pytest.mark.parametrize("rnd", [ROUND_RTN, ROUND_SR])
@pytest.mark.parametrize("fmt,rho", [(FMT_E4M3, 448), (FMT_INT4, 7)])
def test_bf16_scale_codes_are_relative_to_the_stored_scale(o32, fmt, rho, rnd):
    rng = np.random.default_rng(21 + fmt + 2 * rnd)
    n, bs = 2048, 128
    seed, step, tid = 77, 3, 4
    w0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    codes, scales = o32.quantize_rtn(fmt, w0, block_size=bs, scale_bf16=True)
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (rng.random(n) * 1e-5).astype(np.float32)
    g16 = torch.tensor(rng.standard_normal(n) * 3e-3).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
    theta, err = np.zeros(n, np.float32), np.zeros(n, np.float32)
    cfg = StepConfig(fmt=fmt, opt=OPT_ADAM, round=rnd, block_size=bs, scale_bf16=True, lr=2e-3, step=step, seed=seed,
                     tensor_id=tid)
    assert o32.eco_step(cfg, n, m, v, codes=codes, scales=scales, grad_bf16=g16, dbg_theta=theta, dbg_err=err) == 0
    r16 = o32.random16(seed, step, tid, n)          # pinned separately (test_oracle_random)
    grid = grid_of(fmt)
    got = stored_index(fmt, codes, n)
    down_and_saturated = up_and_inside = 0
    for b in range(n // bs):
        th = theta[b * bs:(b + 1) * bs]
        a = np.abs(th).max()
        s = np.float32(scales[b])
        assert s == bf16_nearest(np.float32(a) / np.float32(rho)), "stored scale = bf16(max|theta~| / rho)"
        inv = rn_f32(1 / Fraction(float(s)))
        imax = int(np.abs(th).argmax())
        for j in range(bs):
            y = rn_f32(Fraction(float(th[j])) * Fraction(float(inv)))
            want = exact_code(grid, y, rnd, int(r16[b * bs + j]))
            assert got[b * bs + j] == want, (b, j, float(y), int(got[b * bs + j]), want)
            # the error is measured against the value the stored pair (code, scale) reconstructs
            recon = rn_f32(grid[abs(want)] * (-1 if want < 0 else 1) * Fraction(float(s)))
            assert err[b * bs + j] == rn_f32(Fraction(float(th[j])) - Fraction(float(recon)))
        ymax = Fraction(float(a)) * Fraction(float(inv))
        if Fraction(float(s)) * rho < Fraction(float(a)):
            # the scale was rounded down: the largest element lies beyond rho and saturates
            assert ymax > rho and abs(got[b * bs + imax]) == len(grid) - 1
            down_and_saturated += 1
        elif Fraction(float(s)) * rho > Fraction(float(a)) and ymax < rho:
            up_and_inside += 1
    assert down_and_saturated >= 3 and up_and_inside >= 3, "the sample must contain scales rounded either way"


@pytest.mark.parametrize("opt", [OPT_ADAM, OPT_SGDM])
@pytest.mark.parametrize("fmt", [FMT_E4M3, FMT_INT4])
def test_bf16_state_is_one_rounding_of_the_fp32_step(o32, fmt, opt):
    rng = np.random.default_rng(31 + fmt + 2 * opt)
    n, bs = 1024, 128
    w0 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    codes0, scales0 = o32.quantize_rtn(fmt, w0, block_size=bs, scale_bf16=True)
    m0 = bf16_nearest(rng.standard_normal(n) * 1e-3)          # the state a previous bf16 step would have left
    v0 = bf16_nearest(rng.random(n) * 1e-5)
    for step in (1, 2, 7):
        g16 = torch.tensor(rng.standard_normal(n) * 2e-3).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()
        out = {}
        for state_bf16 in (False, True):
            c, s, m, v = codes0.copy(), scales0.copy(), m0.copy(), v0.copy()
            th, er = np.zeros(n, np.float32), np.zeros(n, np.float32)
            cfg = StepConfig(fmt=fmt, opt=opt, round=ROUND_SR, block_size=bs, state_bf16=state_bf16, scale_bf16=True,
                             lr=1e-3, step=step, seed=5, tensor_id=1)
            assert o32.eco_step(cfg, n, m, v if opt == OPT_ADAM else None, codes=c, scales=s, grad_bf16=g16,
                                dbg_theta=th, dbg_err=er) == 0
            out[state_bf16] = (c, s, th, er, m, v)
        f, h = out[False], out[True]
        for k, name in enumerate(("codes", "scales", "theta~", "error")):
            assert np.array_equal(f[k], h[k]), f"{name} must not depend on the storage type of the state"
        assert np.array_equal(h[4], bf16_nearest(f[4])), "stored m = bf16(m^ of the fp32 step)"
        # the rounding is a real one: the fp32 values are not bfloat16 already
        assert np.mean(f[4] != bf16_nearest(f[4])) > 0.9
        if opt == OPT_ADAM:
            assert np.array_equal(h[5], bf16_nearest(f[5])), "stored v = bf16(v~ of the fp32 step)"
            assert np.mean(f[5] != bf16_nearest(f[5])) > 0.9
        codes0, scales0, m0, v0 = h[0], h[1], h[4], h[5]      # go on from the bf16 state

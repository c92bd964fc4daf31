"""Pins for the oracle's number formats: OCP E4M3, INT4, bfloat16.

What fixes them, other than the oracle itself: the format definition written as
exact rationals, the anchor encodings of the OCP specification
(tests/golden/e4m3_anchor_values.txt), and torch's own CPU casts
(torch.float8_e4m3fn, torch.bfloat16) as a library cross-check.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import FMT_E4M3, FMT_INT4, ROUND_RTN, ROUND_SR

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def e4m3_exact(c: int):
    """Value of code c from the format definition, as an exact rational (None for NaN)."""
    s, E, M = c >> 7, (c >> 3) & 15, c & 7
    if E == 15 and M == 7:
        return None
    mag = Fraction(M, 8) * Fraction(1, 64) if E == 0 else (1 + Fraction(M, 8)) * Fraction(2) ** (E - 7)
    return -mag if s else mag


@pytest.mark.parametrize("real", ["f32", "f64"])
def test_e4m3_decode_matches_definition(real):
    t = oracle.get(real).decode_table(FMT_E4M3)
    for c in range(256):
        ex = e4m3_exact(c)
        if ex is None:
            assert np.isnan(t[c])
        else:
            assert Fraction(float(t[c])) == ex, c
            if ex == 0:
                assert np.signbit(t[c]) == bool(c >> 7)


def test_e4m3_anchor_values(o32):
    t = o32.decode_table(FMT_E4M3)
    for line in open(os.path.join(GOLDEN, "e4m3_anchor_values.txt")):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        c, v = int(code, 16), float(val)
        assert t[c] == v and np.signbit(t[c]) == np.signbit(v), line


def test_e4m3_decode_matches_torch(o32):
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
    t = o32.decode_table(FMT_E4M3)
    assert np.array_equal(np.isnan(ref), np.isnan(t))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok].view(np.uint32), t[ok].view(np.uint32))


def test_e4m3_monotone_in_sign_magnitude(o32):
    t = o32.decode_table(FMT_E4M3)
    assert np.all(np.diff(t[0:127]) > 0)
    assert np.all(np.diff(t[128:255]) < 0)


@pytest.mark.parametrize("real", ["f32", "f64"])
def test_e4m3_all_codes_round_trip(real):
    o = oracle.get(real)
    t = o.decode_table(FMT_E4M3)
    codes = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    assert len(codes) == 254
    for rnd in (ROUND_RTN, ROUND_SR):
        # on-grid values are fixed points of both rounding modes, whatever the random bits
        for r in (0, 1, 0x8000, 0xFFFF):
            back = o.encode(FMT_E4M3, rnd, t[codes], np.full(codes.size, r, dtype=np.uint16))
            assert np.array_equal(back, codes), (rnd, r)


def test_e4m3_rtn_boundaries(o32):
    t = o32.decode_table(FMT_E4M3).astype(np.float32)
    for sign in (1.0, -1.0):
        sbit = 0 if sign > 0 else 0x80
        for j in range(126):
            lo, hi = np.float32(t[j]), np.float32(t[j + 1])
            mid = np.float32((np.float64(lo) + np.float64(hi)) / 2)      # exact in fp32
            assert np.float64(mid) * 2 == np.float64(lo) + np.float64(hi)
            below = np.nextafter(mid, np.float32(0), dtype=np.float32)
            above = np.nextafter(mid, np.float32(1e9), dtype=np.float32)
            got = o32.encode(FMT_E4M3, ROUND_RTN, sign * np.array([below, mid, above], dtype=np.float32))
            even = j if j % 2 == 0 else j + 1
            assert list(got) == [sbit | j, sbit | even, sbit | (j + 1)], (j, sign)
    # saturation: anything at or beyond rho encodes to +-448, never to NaN
    big = np.array([448.0, 448.00003, 464.0, 480.0, 1e6, 3e38], dtype=np.float32)
    assert np.all(o32.encode(FMT_E4M3, ROUND_RTN, big) == 0x7E)
    assert np.all(o32.encode(FMT_E4M3, ROUND_RTN, -big) == 0xFE)
    assert np.all(o32.encode(FMT_E4M3, ROUND_SR, big, np.full(big.size, 0xFFFF, np.uint16)) == 0x7E)


def test_e4m3_rtn_matches_torch_cast(o32):
    g = torch.Generator().manual_seed(11)
    # a wide log-uniform sweep that covers the subnormal range, the normal range and both signs
    mag = torch.exp(torch.rand(400000, generator=g) * 16.0 - 9.5)           # ~[7e-5, 665]
    x = (mag * torch.sign(torch.randn(400000, generator=g))).clamp(-448, 448).float()
    ref = x.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = o32.encode(FMT_E4M3, ROUND_RTN, x.numpy())
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("real", ["f32", "f64"])
def test_int4_codec(real):
    o = oracle.get(real)
    t = o.decode_table(FMT_INT4)
    assert list(t) == [0, 1, 2, 3, 4, 5, 6, 7, -8, -7, -6, -5, -4, -3, -2, -1]
    vals = np.arange(-7, 8).astype(o.dtype)
    for rnd in (ROUND_RTN, ROUND_SR):
        c = o.encode(FMT_INT4, rnd, vals, np.full(vals.size, 0xFFFF, np.uint16))
        assert np.array_equal(t[c], vals)
        assert not np.any(c == 8)                                  # -8 is never produced
    # ties go to the even integer; beyond +-7 saturates
    y = np.array([0.5, 1.5, 2.5, 3.5, 6.5, -0.5, -1.5, -6.5, 7.4, 9.0, -100.0, 0.49999, 0.50001], dtype=o.dtype)
    c = o.encode(FMT_INT4, ROUND_RTN, y)
    assert list(t[c]) == [0, 2, 2, 4, 6, 0, -2, -6, 7, 7, -7, 0, 1]


def test_int4_nibble_order_and_dequantize(o32):
    x = np.array([1, -2, 3, -4, 5, -6, 7, 0], dtype=np.float32)      # abs-max 7 -> scale exactly 1
    codes, scales = o32.quantize_rtn(FMT_INT4, x, block_size=8)
    assert scales[0] == 1.0
    # element 2j in the low nibble, 2j+1 in the high nibble
    assert list(codes) == [0x1 | (0xE << 4), 0x3 | (0xC << 4), 0x5 | (0xA << 4), 0x7 | (0x0 << 4)]
    assert np.array_equal(o32.dequantize(FMT_INT4, codes, scales, 8, block_size=8), x)


def test_bf16_round_matches_torch(o32):
    g = torch.Generator().manual_seed(5)
    x = torch.randn(200000, generator=g) * torch.exp(torch.randn(200000, generator=g) * 8)
    edge = torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, 3.3895e38, 3.4e38,
                         1e-40, 9.1835e-41, 4.6e-41, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20], dtype=torch.float32)
    x = torch.cat([x.float(), edge])
    ref = x.to(torch.bfloat16).float().numpy()
    got = np.array([o32.bf16_round(float(v)) for v in x.numpy()], dtype=np.float32)
    assert np.array_equal(ref.view(np.uint32), got.view(np.uint32))


def test_quantizer_scale_and_max_element(o32):
    """s = max|x| / rho; the largest element lands on +-rho; codes are a function of x/max|x| only."""
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(1024) * 0.02).astype(np.float32)
    for fmt, rho in ((FMT_E4M3, 448.0), (FMT_INT4, 7.0)):
        codes, scales = o32.quantize_rtn(fmt, x, block_size=128)
        deq = o32.dequantize(fmt, codes, scales, x.size, block_size=128)
        for b in range(8):
            blk = x[b * 128:(b + 1) * 128]
            a = np.abs(blk).max()
            assert scales[b] == np.float32(a) / np.float32(rho)
            k = np.abs(blk).argmax()
            assert abs(deq[b * 128 + k]) == np.float32(rho) * scales[b]
            # round-to-nearest error is at most half a grid step: for E4M3 half of 2^-3 relative
            # above the subnormal range, for INT4 half a unit of the scale
            err = np.abs(deq[b * 128:(b + 1) * 128] - blk)
            if fmt == FMT_INT4:
                assert np.all(err <= 0.5 * scales[b] * (1 + 1e-6))
            else:
                assert np.all(err <= np.maximum(np.abs(blk) / 16, scales[b] * 2.0 ** -10) * (1 + 1e-5))
        # a permutation of a block permutes its codes and keeps its scale
        perm = rng.permutation(128)
        xp = x.copy()
        xp[:128] = x[:128][perm]
        cp, sp = o32.quantize_rtn(fmt, xp, block_size=128)
        assert sp[0] == scales[0]
        dp = o32.dequantize(fmt, cp, sp, x.size, block_size=128)
        assert np.array_equal(dp[:128], deq[:128][perm])


def test_zero_and_tiny_blocks(o32):
    x = np.zeros(256, dtype=np.float32)
    x[128:] = 1e-38                                  # rho / max overflows fp32 -> stored as a zero block
    for fmt in (FMT_E4M3, FMT_INT4):
        codes, scales = o32.quantize_rtn(fmt, x, block_size=128)
        assert np.all(scales == 0) and np.all(codes == 0)


def test_ragged_last_block(o32):
    rng = np.random.default_rng(4)
    x = rng.standard_normal(300).astype(np.float32)
    codes, scales = o32.quantize_rtn(FMT_E4M3, x, block_size=128)
    assert scales.size == 3
    assert scales[2] == np.float32(np.abs(x[256:]).max()) / np.float32(448.0)
    full, _ = o32.quantize_rtn(FMT_E4M3, x[256:], block_size=128)
    assert np.array_equal(codes[256:], full)

"""Pins for the oracle's random numbers and stochastic rounding.

Philox4x32-10 is fixed by the published algorithm (Salmon et al., SC'11): the
known-answer vectors in tests/golden/philox4x32_10_kat.txt and an independent
big-integer implementation written here from the paper's description.
Stochastic rounding is fixed by its definition in the paper's Sec. 3.1
("Quantization": the probability of either neighbour is proportional to the
distance to the other one; the result is an unbiased estimator).
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import FMT_E4M3, FMT_INT4, ROUND_SR

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M32 = 0xFFFFFFFF


def philox_bigint(ctr, key, rounds=10):
    """Philox-4x32 as published: two 32x32->64 multiplies per round, Weyl key schedule."""
    c = list(ctr)
    k = list(key)
    for r in range(rounds):
        if r:
            k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & M32, (p0 >> 32) ^ c[3] ^ k[1], p0 & M32]
    return c


def test_philox_known_answers(o32):
    n = 0
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(x, 16) for x in line.split()]
        assert list(o32.philox(w[0:4], w[4:6])) == w[6:10]
        assert philox_bigint(w[0:4], w[4:6]) == w[6:10]
        n += 1
    assert n == 3


def test_philox_matches_bigint_on_random_and_edge_counters(o32, o64):
    rng = np.random.default_rng(1)
    cases = [([0, 0, 0, 0], [0, 0]), ([1, 0, 0, 0], [0, 0]), ([M32, 0, 0, 0], [1, 2]),
             ([0, 1, 0, 0], [1, 2]), ([5, 6, 7, 8], [M32, M32])]
    cases += [(list(rng.integers(0, 2 ** 32, 4)), list(rng.integers(0, 2 ** 32, 2))) for _ in range(200)]
    for ctr, key in cases:
        ref = philox_bigint([int(x) for x in ctr], [int(x) for x in key])
        assert list(o32.philox(ctr, key)) == ref
        assert list(o64.philox(ctr, key)) == ref


def test_stream_layout(o32):
    """Counter = (q lo, q hi, step lo, tensor_id), key = (seed lo, seed hi); element i uses the
    16-bit field i & 7 of call q = i >> 3."""
    seed, step, tid = 0x0123456789ABCDEF, 7, 42
    words = o32.philox_fill(seed, step, tid, 64)
    for q in range(16):
        ref = philox_bigint([q, 0, step, tid], [seed & M32, seed >> 32])
        assert list(words[4 * q:4 * q + 4]) == ref
    r = o32.random16(seed, step, tid, 128)
    for i in range(128):
        w = int(words[(i >> 3) * 4 + ((i & 7) >> 1)])
        assert int(r[i]) == ((w >> 16) if i & 1 else (w & 0xFFFF))
    # sub-ranges and the 2^32 carry into the second counter word
    assert np.array_equal(o32.philox_fill(seed, step, tid, 16, first_word=20), words[20:36])
    big = (1 << 34) + 8                      # word index; call index 2^32 + 2
    hi = o32.philox_fill(seed, step, tid, 4, first_word=big)
    assert list(hi) == philox_bigint([2, 1, step, tid], [seed & M32, seed >> 32])
    # a different step, tensor or seed gives a different stream
    for other in (o32.philox_fill(seed, step + 1, tid, 64), o32.philox_fill(seed, step, tid + 1, 64),
                  o32.philox_fill(seed + 1, step, tid, 64)):
        assert not np.array_equal(other, words)


def test_philox_bit_balance(o32):
    w = o32.philox_fill(99, 1, 0, 1 << 18)
    bits = np.unpackbits(w.view(np.uint8))
    n = bits.size
    assert abs(bits.mean() - 0.5) < 5 * 0.5 / np.sqrt(n)
    per_bit = np.unpackbits(w.view(np.uint8).reshape(-1, 4), axis=1).mean(axis=0)
    assert np.all(np.abs(per_bit - 0.5) < 5 * 0.5 / np.sqrt(w.size))
    # 16-bit fields are uniform: chi-square over 256 buckets of the high byte
    r = o32.random16(99, 1, 0, 1 << 19)
    cnt = np.bincount(r >> 8, minlength=256)
    chi2 = ((cnt - r.size / 256) ** 2 / (r.size / 256)).sum()
    assert chi2 < 255 + 6 * np.sqrt(2 * 255)


def _neighbours(grid, ay):
    j = max(i for i, gval in enumerate(grid) if gval <= ay)
    return j, grid[j], grid[j + 1]


@pytest.mark.parametrize("fmt", [FMT_E4M3, FMT_INT4])
def test_sr_exhaustive_over_random_field(o32, fmt):
    """For fixed y, sweep all 2^16 values of the element's random field: only the two neighbours
    occur, and the number of 'up' outcomes is exactly floor((F + 8) / 16), F = f * 2^20 rounded to nearest
    even: the probability of rounding up is the distance from the lower neighbour (Sec. 3.1) rounded to the
    nearest multiple of 2^-16 -- within 2^-17 of it and in neither direction preferentially -- and values
    whose F is a multiple of 16 (f = 1/2, 1/4, 1/16 below) hit it exactly."""
    table = o32.decode_table(fmt)
    grid = sorted(Fraction(float(v)) for v in (table[:127] if fmt == FMT_E4M3 else table[:8]))
    rho = grid[-1]
    rng = np.random.default_rng(7)
    ys = list(rng.uniform(0, float(rho), 12).astype(np.float32))
    ys += [np.float32(2.0 ** -12), np.float32(0.0123), np.float32(float(rho) - 1e-3), np.float32(1.0),
           np.float32(3.0 + 2.0 ** -20), np.float32(1.5 - 2.0 ** -20),
           np.float32(1.0625), np.float32(2.5), np.float32(3.25), np.float32(5.0625), np.float32(6.5)]
    # fractions with every residue of F modulo 16 just above a grid point (1.0 is on both grids; the next
    # grid point is 1.125 for E4M3 and 2 for INT4, so one unit of F is 2^-23 resp. 2^-20)
    unit = 2.0 ** -23 if fmt == FMT_E4M3 else 2.0 ** -20
    ys += [np.float32(1.0 + k * unit) for k in list(range(1, 34)) + [2 ** 20 - 9, 2 ** 20 - 8, 2 ** 20 - 1]]
    r = np.arange(65536, dtype=np.uint16)
    seen_residues = set()
    for y in ys:
        for sign in (1, -1):
            codes = o32.encode(fmt, ROUND_SR, np.full(65536, sign * y, dtype=np.float32), r)
            vals = np.abs(table[codes].astype(np.float64))
            j, lo, hi = _neighbours(grid, Fraction(float(y)))
            assert set(np.unique(vals)) <= {float(lo), float(hi)}
            f = (Fraction(float(y)) - lo) / (hi - lo)
            F = round(f * 2 ** 20)                     # Python rounds exact halves to even, like the definition
            seen_residues.add(F % 16)
            ups = int((vals == float(hi)).sum()) if hi != lo else 0
            assert ups == (F + 8) // 16, (float(y), ups, float(f * 65536))
            assert abs(ups - f * 65536) <= Fraction(1, 2) + Fraction(1, 32)     # nearest multiple (F itself is rounded below 2^-6)
            if f == 0:
                assert ups == 0
            # the up outcomes are the LARGEST random fields: up iff F + 16 r + 8 >= 2^20
            if 0 < ups < 65536:
                assert np.all(vals[65536 - ups:] == float(hi)) and np.all(vals[:65536 - ups] == float(lo))
            # sign symmetry: the magnitude decision does not depend on the sign
            if sign == -1:
                pos = o32.encode(fmt, ROUND_SR, np.full(65536, y, dtype=np.float32), r)
                assert np.array_equal(np.abs(table[pos]), np.abs(table[codes]))
    assert seen_residues == set(range(16))


def test_sr_resolution_has_no_preferred_direction():
    """The 16-bit resolution of the random field: P(up) - f, averaged over the 16 residues of F modulo 16, is
    2^-21 of a grid step (a rule that truncates F/16 instead would pull every value toward zero by 15/32 of
    2^-16, on every element at every step).  Stated for the rule itself, in exact rationals."""
    for base in (0, 16, 4096, 2 ** 20 - 16):
        bias = [Fraction((F + 8) // 16, 2 ** 16) - Fraction(F, 2 ** 20) for F in range(base, base + 16)]
        assert abs(sum(bias) / 16) <= Fraction(1, 2 ** 21)
        assert max(abs(b) for b in bias) <= Fraction(1, 2 ** 17)
        trunc = [Fraction(F // 16, 2 ** 16) - Fraction(F, 2 ** 20) for F in range(base, base + 16)]
        assert sum(trunc) / 16 == -Fraction(15, 2 ** 21)


@pytest.mark.parametrize("fmt,rho", [(FMT_E4M3, 448.0), (FMT_INT4, 7.0)])
def test_sr_unbiased_with_philox_bits(o32, fmt, rho):
    """E[dec(SR(y))] = y (Sec. 3.1: stochastic rounding is an unbiased estimator; Assumption 3.2), checked with
    the oracle's own Philox-driven random fields, on single values and on a spread of values."""
    table = o32.decode_table(fmt).astype(np.float64)
    n = 1 << 20
    r = o32.random16(2024, 3, 5, n)
    for y in (0.3141, 1.7, 5.55, 0.0071, -2.9):
        y32 = np.float32(y * rho / 7.0)
        codes = o32.encode(fmt, ROUND_SR, np.full(n, y32, dtype=np.float32), r)
        vals = table[codes]
        step = np.ptp(vals)                       # distance between the two neighbours
        assert step > 0
        # standard error of a two-point variable is at most step/2/sqrt(n); 5 sigma
        assert abs(vals.mean() - float(y32)) <= 5 * step / 2 / np.sqrt(n)
    # many different values inside one grid cell: the mean error over them is zero within 5 sigma as well
    lo, hi = (1.0, 1.125) if fmt == FMT_E4M3 else (1.0, 2.0)
    ys = np.random.default_rng(5).uniform(lo, hi, n).astype(np.float32)
    err = table[o32.encode(fmt, ROUND_SR, ys, r)] - ys.astype(np.float64)
    assert abs(err.mean()) <= 5 * (hi - lo) / 2 / np.sqrt(n)

"""Pins for the oracle's number formats and random numbers (CPU only).

Each check compares the C oracle with something it does not compute itself:
the printed E2M1 value table, the bit-field formula of the format, an exact
rational nearest-value search, closed forms for the E8M0 rule, and statistical
properties of the counter hash.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

E2M1_SET = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def _read_pairs(path):
    rows = []
    with open(path) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                a, b = line.split()
                rows.append((a, b))
    return rows


# ---------------------------------------------------------------- E2M1 codec
def test_e2m1_decode_matches_printed_table(golden_dir):
    rows = _read_pairs(os.path.join(golden_dir, "e2m1_values.txt"))
    assert len(rows) == 16
    for code_hex, val in rows:
        got = oracle.e2m1_decode(int(code_hex, 16))
        want = float(val)
        assert got == want and math.copysign(1.0, got) == math.copysign(1.0, want)


def test_e2m1_decode_matches_bitfield_formula():
    # sign | 2-bit exponent (bias 1) | 1-bit mantissa; exponent 0 is subnormal
    for code in range(16):
        s, e, m = code >> 3, (code >> 1) & 3, code & 1
        mag = m * 0.5 if e == 0 else 2.0 ** (e - 1) * (1 + m / 2)
        assert oracle.e2m1_decode(code) == (-mag if s else mag)
    assert sorted({abs(oracle.e2m1_decode(c)) for c in range(16)}) == E2M1_SET


def test_e2m1_round_trip_all_codes():
    for code in range(16):
        assert oracle.e2m1_encode_rne(oracle.e2m1_decode(code)) == code
        # an exactly representable value never moves under stochastic rounding either
        for r in (0, 1, 0x7FFFFFFF, 0xFFFFFFFF, 0x12345678):
            assert oracle.e2m1_encode_sr(oracle.e2m1_decode(code), r) == code


def test_e2m1_rne_tie_table(golden_dir):
    for mag, want in _read_pairs(os.path.join(golden_dir, "e2m1_rne_ties.txt")):
        for sign in (1.0, -1.0):
            code = oracle.e2m1_encode_rne(sign * float(mag))
            assert abs(oracle.e2m1_decode(code)) == float(want), (mag, want)
            assert (code >> 3) == (1 if sign < 0 else 0)


def _rne_by_thresholds(t: float) -> int:
    """Independent formulation: count decision thresholds passed, in exact rationals.
    Midpoints between neighbours; at a midpoint the even code wins."""
    a = abs(Fraction(t))
    grid = [Fraction(v) for v in E2M1_SET]
    code = 0
    for c in range(7):
        mid = (grid[c] + grid[c + 1]) / 2
        upper_is_even = ((c + 1) % 2) == 0
        if a > mid or (a == mid and upper_is_even):
            code = c + 1
    return (8 if math.copysign(1.0, t) < 0 else 0) | code


def test_e2m1_rne_every_bf16_input():
    # all finite bf16 values, at three scalings so that every one lands in the
    # interesting range [0, 8) for some scaling
    bits = np.arange(65536, dtype=np.uint32)
    vals = (bits << 16).astype(np.uint32).view(np.float32)
    finite = np.isfinite(vals)
    checked = 0
    for k in (0, -3, 2):
        for v in vals[finite][::1]:
            t = math.ldexp(float(v), k)
            if abs(t) > 16:
                continue
            assert oracle.e2m1_encode_rne(t) == _rne_by_thresholds(t)
            checked += 1
    assert checked > 90000


def test_e2m1_rne_negative_zero_and_tiny_keep_sign():
    assert oracle.e2m1_encode_rne(-0.0) == 8
    assert oracle.e2m1_encode_rne(-1e-30) == 8
    assert oracle.e2m1_encode_rne(1e-30) == 0


# ---------------------------------------------------------------- E8M0 rule
def test_e8m0_closed_form_every_bf16_amax():
    # amax = m * 2^k with m in [1,2): byte = k + 125, and amax * 2^-(byte-127) in [4, 8)
    for h in range(0x0080, 0x7F80):  # all positive normal bf16
        bits = h << 16
        v = float(np.array([bits], dtype=np.uint32).view(np.float32)[0])
        m, e = math.frexp(v)  # v = m * 2^e, m in [0.5, 1)
        k = e - 1
        want = min(max(k + 125, 0), 254)
        got = oracle.e8m0_from_amax_bits(bits)
        assert got == want
        if 0 < k + 125 <= 254:
            scaled = math.ldexp(v, -(got - 127))
            assert 4.0 <= scaled < 8.0


def test_e8m0_edges():
    assert oracle.e8m0_from_amax_bits(0) == 0                      # all-zero block
    assert oracle.e8m0_from_amax_bits(0x00000001) == 0             # subnormal amax
    assert oracle.e8m0_from_amax_bits(0x007FFFFF) == 0
    assert oracle.e8m0_from_amax_bits(0x00800000) == 0             # 2^-126 -> clamp(1-2)
    assert oracle.e8m0_from_amax_bits(0x01000000) == 0             # 2^-125
    assert oracle.e8m0_from_amax_bits(0x01800000) == 1             # 2^-124
    assert oracle.e8m0_from_amax_bits(0x3F800000) == 125           # 1.0
    assert oracle.e8m0_from_amax_bits(0x40C00000) == 127           # 6.0 -> scale 1
    assert oracle.e8m0_from_amax_bits(0x7F7FFFFF) == 252           # FLT_MAX
    assert oracle.e8m0_from_amax_bits(0x7F800000) == 0xFF          # inf
    assert oracle.e8m0_from_amax_bits(0x7FC00000) == 0xFF          # NaN


# ---------------------------------------------------------------- bf16
def test_bf16_widening_is_exact():
    L = oracle.lib()
    for h in (0x0000, 0x8000, 0x3F80, 0xBF80, 0x4049, 0x0001, 0x7F7F, 0x42C8):
        f = L.orc_bf16_to_f32(h)
        assert np.array([f], dtype=np.float32).view(np.uint32)[0] == (h << 16)
    assert L.orc_bf16_to_f32(0x42C8) == 100.0 and L.orc_bf16_to_f32(0x3F80) == 1.0


def test_f32_to_bf16_rne_against_torch():
    import torch
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32),
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.4e38, 1e-40], dtype=np.float32)])
    got = oracle.f32_to_bf16_rne(x)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, want)


# ---------------------------------------------------------------- counter hash
def test_rand32_is_a_pure_function():
    a = oracle.rand32_array(7, 1000, 4096)
    b = oracle.rand32_array(7, 1000, 4096)
    assert np.array_equal(a, b)
    assert a[5] == oracle.rand32(7, 1005)
    assert not np.array_equal(a, oracle.rand32_array(8, 1000, 4096))
    # the high halves of seed and index matter too
    assert oracle.rand32(7, 5) != oracle.rand32(7 + (1 << 32), 5)
    assert oracle.rand32(7, 5) != oracle.rand32(7, 5 + (1 << 32))


def test_rand32_uniform_buckets_chi_square():
    n = 1 << 20
    r = oracle.rand32_array(12345, 0, n)
    for shift in (24, 0, 9):  # top byte, bottom byte, and the bits SR consumes first
        counts = np.bincount((r >> shift) & 0xFF, minlength=256)
        chi2 = float(((counts - n / 256) ** 2 / (n / 256)).sum())
        # 255 dof: mean 255, sd ~22.6; 6 sd
        assert chi2 < 255 + 6 * 22.6, (shift, chi2)


def test_rand32_avalanche():
    n = 1 << 14
    base = oracle.rand32_array(99, 0, n)
    for bit in range(0, 32, 3):
        # flipping one index bit: consecutive-index array vs the same indices xor (1<<bit)
        flipped = np.array([oracle.rand32(99, i ^ (1 << bit)) for i in range(0, n, 8)], dtype=np.uint32)
        diff = base[::8] ^ flipped
        frac = np.unpackbits(diff.view(np.uint8)).mean()
        assert abs(frac - 0.5) < 0.02, (bit, frac)
    for bit in (0, 13, 31, 40, 63):  # seed bits
        other = oracle.rand32_array(99 ^ (1 << bit), 0, n)
        frac = np.unpackbits((base ^ other).view(np.uint8)).mean()
        assert abs(frac - 0.5) < 0.02, (bit, frac)


def test_rand32_neighbouring_counters_uncorrelated():
    r = oracle.rand32_array(3, 0, 1 << 18).astype(np.float64) / 2**32
    c = np.corrcoef(r[:-1], r[1:])[0, 1]
    assert abs(c) < 0.01


# ---------------------------------------------------------------- stochastic rounding
@pytest.mark.parametrize("a", [0.1, 0.25, 0.6, 1.3, 1.9, 2.2, 3.75, 4.5, 5.9])
def test_sr_is_unbiased(a):
    n = 1 << 17
    r = oracle.rand32_array(2024, 0, n)
    vals = np.array([abs(oracle.e2m1_decode(oracle.e2m1_encode_sr(a, int(x)))) for x in r])
    lo = max(v for v in E2M1_SET if v <= a)
    hi = min(v for v in E2M1_SET if v >= a)
    assert set(np.unique(vals)) <= {lo, hi}
    p = (a - lo) / (hi - lo)
    sigma = (hi - lo) * math.sqrt(p * (1 - p) / n)
    assert abs(vals.mean() - a) < 4 * sigma + 2**-22


def test_sr_saturates_and_keeps_sign():
    for r in (0, 0xFFFFFFFF, 0x80000000):
        assert oracle.e2m1_encode_sr(6.5, r) == 7
        assert oracle.e2m1_encode_sr(-100.0, r) == 15
        assert oracle.e2m1_encode_sr(-0.0, r) == 8
    # u is never 0: a vanishing fraction never rounds up, even with r = 0
    assert oracle.e2m1_encode_sr(1e-20, 0) == 0
    # and never reaches 1: a fraction just below 1 rounds up with the largest u ...
    # u_max = 1 - 2^-24 ; f = 1 - 2^-25 > u_max
    assert oracle.e2m1_encode_sr(0.5 * (1 - 2.0**-25), 0xFFFFFFFF) == 1


def test_sr_uses_the_top_23_bits():
    # the decision is u < f with u = (2*(r>>9)+1) / 2^24
    a = 0.25  # f = 0.5 between 0 and 0.5
    thr = 1 << 22  # (2n+1)/2^24 < 1/2  <=>  n < 2^22 (n integer: 2n+1 < 2^23)
    for n in (0, 1, thr - 1, thr, thr + 1, (1 << 23) - 1):
        r = (n << 9) | 0x1FF
        want = 1 if (2 * n + 1) < (1 << 23) else 0
        assert oracle.e2m1_encode_sr(a, r) == want

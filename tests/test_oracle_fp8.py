"""Pins for the oracle's MXFP8 (E4M3) pieces (CPU only): the codec against the format's definition, the
scale rule, the block quantiser against invariants, and the mixed-format GEMM against exact arithmetic."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2605_09825_amd import synth
from test_oracle_quantize import bf16_bits, bits_to_f64

GOLD = os.path.join(os.path.dirname(__file__), "golden", "e4m3_values.txt")


def all_e4m3():
    return [(c, oracle.e4m3_decode(c)) for c in range(256)]


def test_decode_matches_the_printed_values_and_the_bit_field_formula():
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        code, val = line.split()
        got = oracle.e4m3_decode(int(code, 16))
        assert got == float(val) and math.copysign(1.0, got) == math.copysign(1.0, float(val)), line
    for c, v in all_e4m3():
        e, m, sgn = (c >> 3) & 15, c & 7, -1.0 if c & 0x80 else 1.0
        if e == 15 and m == 7:
            assert math.isnan(v)
        elif e == 0:
            assert v == sgn * m * 2.0 ** -9
        else:
            assert v == sgn * (8 + m) * 2.0 ** (e - 10)
    finite = [v for _, v in all_e4m3() if not math.isnan(v)]
    assert max(finite) == 448.0 and min(finite) == -448.0 and len(set(map(abs, finite))) == 127


def test_encode_round_trips_every_code_and_rounds_to_nearest_even():
    for c, v in all_e4m3():
        if not math.isnan(v):
            assert oracle.e4m3_encode_rne(v) == c
    mags = sorted(v for c, v in all_e4m3() if c < 0x7F)
    for lo, hi in zip(mags, mags[1:]):
        mid = (lo + hi) / 2  # exact in double
        c_lo, c_hi = oracle.e4m3_encode_rne(lo), oracle.e4m3_encode_rne(hi)
        even = c_lo if c_lo % 2 == 0 else c_hi
        assert oracle.e4m3_encode_rne(mid) == even, (lo, hi)
        assert oracle.e4m3_encode_rne(math.nextafter(mid, 0.0)) == c_lo
        assert oracle.e4m3_encode_rne(math.nextafter(mid, math.inf)) == c_hi
        assert oracle.e4m3_encode_rne(-mid) == even | 0x80
    # brute-force nearest on a dense sweep with exact rational distances
    rng = np.random.default_rng(0)
    for t in np.concatenate([rng.uniform(0, 2, 300), rng.uniform(0, 500, 300), rng.uniform(0, 0.02, 200)]):
        d = [(abs(Fraction(t) - Fraction(m)), i) for i, m in enumerate(mags)]
        best = min(d)[0]
        cands = [i for dist, i in d if dist == best]
        want = cands[0] if len(cands) == 1 else [i for i in cands if i % 2 == 0][0]
        assert oracle.e4m3_encode_rne(float(t)) == want  # code of magnitude i is i
    # saturation and sign of zero
    for t in (448.0, 449.0, 464.0, 480.0, 1e30, math.inf):
        assert oracle.e4m3_encode_rne(t) == 0x7E and oracle.e4m3_encode_rne(-t) == 0xFE
    assert oracle.e4m3_encode_rne(-0.0) == 0x80 and oracle.e4m3_encode_rne(-1e-9) == 0x80


def test_scale_rule_closed_form():
    # amax = m * 2^k, 1 <= m < 2  ->  byte = k - 8 + 127: the scaled maximum lands in [256, 512)
    for k in range(-100, 100):
        for m in (1.0, 1.5, 1.9921875):
            bits = int(np.float32(m * 2.0 ** k).view(np.uint32))
            byte = oracle.e8m0_from_amax_bits_fp8(bits)
            assert byte == k + 119
            assert 256 <= m * 2.0 ** k / 2.0 ** (byte - 127) < 512
    assert oracle.e8m0_from_amax_bits_fp8(0) == 0
    assert oracle.e8m0_from_amax_bits_fp8(0x7F800000) == 0xFF and oracle.e8m0_from_amax_bits_fp8(0x7FC00000) == 0xFF


def decode_fp8(q, s):
    lut = np.array([oracle.e4m3_decode(c) for c in range(256)])
    return lut[q] * np.exp2(s.astype(np.float64) - 127).repeat(32, axis=1)


def test_hand_computed_blocks():
    x = np.ones((1, 32))
    x[0, 0] = 100.0  # floor(log2 100) = 6 -> exponent -2 -> byte 125: 100*4 = 400 (0x7C), 1*4 = 4 (0x48)
    q, s = oracle.quantize_fp8(bf16_bits(x))
    assert s.tolist() == [[125]]
    assert q[0, 0] == 0x7C and set(q[0, 1:].tolist()) == {0x48}
    z = np.zeros((1, 64))
    z[0, 40] = np.nan
    q, s = oracle.quantize_fp8(bf16_bits(z))
    assert s.tolist() == [[0, 0xFF]] and not q.any()


@pytest.mark.parametrize("had", [oracle.HAD_NONE, oracle.HAD_DET, oracle.HAD_DET16])
def test_block_quantiser_invariants(had):
    x = synth.as_u16(synth.student_t3(64, 256, 1.0, 2, synth.STREAM_X))
    q, s = oracle.quantize_fp8(x, oracle.AXIS_LAST, had)
    # scale bytes: exactly 6 above the MXFP4 bytes of the same blocks (8 - 2), rotation included
    _, s4 = oracle.quantize(x, oracle.AXIS_LAST, had)
    assert np.array_equal(s.astype(int), s4.astype(int) - 6)
    # transposed operand = last-axis quantisation of the transpose
    xt = np.ascontiguousarray(x.T)
    a = oracle.quantize_fp8(x, oracle.AXIS_FIRST, had)
    b = oracle.quantize_fp8(xt, oracle.AXIS_LAST, had)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    if had == oracle.HAD_NONE:
        xv, dq = bits_to_f64(x), decode_fp8(q, s)
        scale = np.exp2(s.astype(np.float64) - 127).repeat(32, axis=1)
        a_ = np.abs(xv) / scale
        # unsaturated normal range: relative error at most 2^-4 (3 mantissa bits); subnormal: absolute 2^-10
        ok = a_ <= 448
        err = np.abs(xv - dq) / scale
        assert np.all(err[ok] <= np.maximum(a_[ok] * 2.0 ** -4, 2.0 ** -10))
        assert np.all(np.abs(dq[~ok]) == 448 * scale[~ok])
        # idempotent on its own output grid (values exactly representable in bf16 need not be: compare codes)
        assert a_.reshape(64, 8, 32).max(axis=2).min() >= 256.0


def test_mixed_format_gemm_is_the_exact_sum():
    rng = np.random.default_rng(3)
    Ra, Rb, C = 5, 7, 64
    a8 = rng.integers(0, 127, size=(Ra, C), dtype=np.uint8) | (rng.integers(0, 2, size=(Ra, C), dtype=np.uint8) << 7)
    b8 = rng.integers(0, 127, size=(Rb, C), dtype=np.uint8) | (rng.integers(0, 2, size=(Rb, C), dtype=np.uint8) << 7)
    a4 = rng.integers(0, 256, size=(Ra, C // 2), dtype=np.uint8)
    b4 = rng.integers(0, 256, size=(Rb, C // 2), dtype=np.uint8)
    sa = rng.integers(120, 134, size=(Ra, C // 32), dtype=np.uint8)
    sb = rng.integers(120, 134, size=(Rb, C // 32), dtype=np.uint8)

    def dec(q, s, fmt):
        out = [[None] * C for _ in range(q.shape[0])]
        for r in range(q.shape[0]):
            for c in range(C):
                if fmt == oracle.FMT_E4M3:
                    v = Fraction(oracle.e4m3_decode(int(q[r, c])))
                else:
                    byte = int(q[r, c // 2])
                    v = Fraction(oracle.e2m1_decode((byte >> 4) if c & 1 else (byte & 15)))
                out[r][c] = v * Fraction(2) ** (int(s[r, c // 32]) - 127)
        return out

    for (aq, af), (bq, bf) in (((a8, 1), (b8, 1)), ((a8, 1), (b4, 0)), ((a4, 0), (b8, 1)), ((a4, 0), (b4, 0))):
        A, B = dec(aq, sa, af), dec(bq, sb, bf)
        out, ab = oracle.gemm_fmt(aq, sa, af, bq, sb, bf)
        for i in range(Ra):
            for j in range(Rb):
                exact = sum(A[i][c] * B[j][c] for c in range(C))
                assert abs(Fraction(out[i, j]) - exact) <= abs(exact) * Fraction(1, 2 ** 45) + Fraction(1, 2 ** 200)
                assert ab[i, j] >= abs(out[i, j])
        ii, jj = np.array([0, 4, 2]), np.array([6, 0, 3])
        o2, _ = oracle.gemm_at_fmt(aq, sa, af, bq, sb, bf, ii, jj)
        assert np.array_equal(o2, out[ii, jj])
    # the two-format entry with both operands E2M1 is the plain GEMM
    o4, _ = oracle.gemm(a4, sa, b4, sb)
    assert np.array_equal(o4, oracle.gemm_fmt(a4, sa, 0, b4, sb, 0)[0])

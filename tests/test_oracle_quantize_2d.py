"""Pins for the oracle's 2D (32 x 32) block quantiser of App. D (CPU only).  The 1D quantiser is
pinned on its own; here the 2D one is tied to it and to the properties the paper names: one scale per
32 x 32 region, and invariance under transposition."""
import numpy as np
import pytest

import oracle
from paper_2605_09825_amd import synth
from test_oracle_quantize import bf16_bits, bits_to_f64, unpack

HADS = [oracle.HAD_NONE, oracle.HAD_DET, oracle.HAD_RANDSIGN, oracle.HAD_DET16, oracle.HAD_RANDSIGN16]
E2M1 = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6, -0.0, -0.5, -1, -1.5, -2, -3, -4, -6])


def test_hand_computed_region():
    # a 32 x 32 region of ones with a single 100: floor(log2 100) = 6 -> exponent 4 -> byte 131 for all
    # 32 rows; 100/16 = 6.25 saturates to 6 (code 7); 1/16 rounds to 0 everywhere else
    x = np.ones((32, 32))
    x[17, 5] = 100.0
    q, s = oracle.quantize_2d(bf16_bits(x))
    assert s.tolist() == [[131]] * 32
    codes = unpack(q)
    want = np.zeros((32, 32), dtype=np.uint8)
    want[17, 5] = 7
    assert np.array_equal(codes, want)
    # the same tensor in 1D: only row 17 sees the outlier, the other rows keep byte 125 and code 6
    q1, s1 = oracle.quantize(bf16_bits(x))
    assert s1[17, 0] == 131 and set(np.delete(s1[:, 0], 17).tolist()) == {125}
    assert set(np.delete(unpack(q1), 17, axis=0).reshape(-1).tolist()) == {6}


def test_two_regions_are_independent():
    x = np.ones((32, 64))
    x[3, 40] = 8.0  # second region only: floor(log2 8) = 3 -> exponent 1 -> byte 128; 1/2 -> code 1, 8/2 = 4 -> code 6
    q, s = oracle.quantize_2d(bf16_bits(x))
    assert np.all(s[:, 0] == 125) and np.all(s[:, 1] == 128)
    codes = unpack(q)
    assert np.all(codes[:, :32] == 6)
    want = np.full((32, 32), 1)
    want[3, 8] = 6
    assert np.array_equal(codes[:, 32:], want)


@pytest.mark.parametrize("axis", [oracle.AXIS_LAST, oracle.AXIS_FIRST])
@pytest.mark.parametrize("had", HADS)
@pytest.mark.parametrize("rnd", [oracle.RNE, oracle.SR])
def test_region_scale_is_the_largest_1d_scale_and_matching_blocks_keep_their_codes(axis, had, rnd):
    # the E8M0 rule is monotone in the maximum, so the region's byte is the largest of its 32 block bytes;
    # a block whose own byte equals the region's is quantised exactly as in 1D (same counters for SR)
    x = synth.as_u16(synth.student_t3(96, 160, 1.0, 11, synth.STREAM_X))
    q1, s1 = oracle.quantize(x, axis, had, rnd, seed=5)
    q2, s2 = oracle.quantize_2d(x, axis, had, rnd, seed=5)
    R, nb = s1.shape
    want = s1.reshape(R // 32, 32, nb).max(axis=1, keepdims=True).repeat(32, axis=1).reshape(R, nb)
    assert np.array_equal(s2, want)
    same = s1 == s2
    assert 0.02 < same.mean() < 0.9  # both kinds of block occur
    c1, c2 = unpack(q1).reshape(R, nb, 32), unpack(q2).reshape(R, nb, 32)
    assert np.array_equal(c1[same], c2[same])
    assert not np.array_equal(c1[~same], c2[~same])


def test_transposition_invariance_without_rotation():
    # "transpose-invariant": quantising X and X^T gives the same codes and scales, transposed
    x = synth.as_u16(synth.normal_with_outlier_channels(64, 96, 3, synth.STREAM_X, fraction=0.05))
    ql, sl = oracle.quantize_2d(x, oracle.AXIS_LAST)
    qf, sf = oracle.quantize_2d(x, oracle.AXIS_FIRST)
    assert np.array_equal(unpack(qf), unpack(ql).T)
    # one byte per region in both outputs: sl[32*rb + i][cb] == sf[32*cb + j][rb] for all i, j
    for rb in range(2):
        for cb in range(3):
            assert len(set(sl[rb * 32:(rb + 1) * 32, cb].tolist())) == 1
            assert len(set(sf[cb * 32:(cb + 1) * 32, rb].tolist())) == 1
            assert sl[rb * 32, cb] == sf[cb * 32, rb]
    # and AXIS_FIRST is AXIS_LAST of the transposed tensor, in every mode
    xt = np.ascontiguousarray(x.T)
    for had in HADS:
        a = oracle.quantize_2d(x, oracle.AXIS_FIRST, had, oracle.SR, seed=3)
        b = oracle.quantize_2d(xt, oracle.AXIS_LAST, had, oracle.SR, seed=3)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("had", [oracle.HAD_NONE])
def test_error_bound_of_the_format(had):
    # unsaturated elements: |x - DQ(Q(x))| <= half the local grid spacing times 2^E
    x = synth.as_u16(synth.normal(64, 128, 1.0, 4, synth.STREAM_X))
    q, s = oracle.quantize_2d(x, oracle.AXIS_LAST, had)
    xv = bits_to_f64(x)
    dq = oracle.dequantize(q, s)
    scale = np.exp2(s.astype(np.float64) - 127).repeat(32, axis=1)
    a = np.abs(xv) / scale
    assert a.max() < 8.0  # the region maximum lands in [4, 8)
    spacing = np.where(a < 2, 0.5, np.where(a < 4, 1.0, 2.0))
    unsat = a <= 6
    assert np.all(np.abs(xv - dq)[unsat] <= (spacing * scale / 2)[unsat])
    assert np.all(np.abs(dq[~unsat]) == (6 * scale)[~unsat])
    # every region uses its top octave
    assert np.all(a.reshape(2, 32, 4, 32).max(axis=(1, 3)) >= 4.0)


def test_non_finite_value_marks_its_whole_region_only():
    x = np.ones((64, 64))
    x[40, 10] = np.nan
    q, s = oracle.quantize_2d(bf16_bits(x))
    assert np.all(s[32:, 0] == 0xFF) and np.all(q[32:, :16] == 0)
    assert np.all(s[:32] == 125) and np.all(s[32:, 1] == 125)


def test_leading_dimension_and_shape_errors():
    base = synth.as_u16(synth.normal(96, 160, 1.0, 8, synth.STREAM_X))
    view = base[32:96, 32:128]
    a = oracle.quantize_2d(view, oracle.AXIS_LAST, oracle.HAD_DET)
    b = oracle.quantize_2d(np.ascontiguousarray(view), oracle.AXIS_LAST, oracle.HAD_DET)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    with pytest.raises(ValueError):
        oracle.quantize_2d(base[:48], oracle.AXIS_LAST)

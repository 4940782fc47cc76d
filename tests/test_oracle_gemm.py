"""Pins for the oracle's GEMM and linear-layer compositions (CPU only): brute force
in exact rational arithmetic on tiny shapes, exactly representable inputs for
which quantisation is the identity, and the stage/axis conventions of App. C."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from paper_2605_09825_amd import synth

E2M1 = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]


def frac_decode(q, s):
    R, C = q.shape[0], q.shape[1] * 2
    out = [[None] * C for _ in range(R)]
    for r in range(R):
        for c in range(C):
            byte = int(q[r, c // 2])
            code = (byte >> 4) if (c & 1) else (byte & 15)
            mag = E2M1[code & 7] * Fraction(2) ** (int(s[r, c // 32]) - 127)
            out[r][c] = -mag if code & 8 else mag
    return out


def test_gemm_equals_exact_rational_brute_force():
    rng = np.random.default_rng(0)
    Ra, Rb, C = 16, 12, 64
    aq = rng.integers(0, 256, size=(Ra, C // 2), dtype=np.uint8)
    bq = rng.integers(0, 256, size=(Rb, C // 2), dtype=np.uint8)
    as_ = rng.integers(110, 140, size=(Ra, C // 32), dtype=np.uint8)
    bs = rng.integers(100, 150, size=(Rb, C // 32), dtype=np.uint8)
    out, ab = oracle.gemm(aq, as_, bq, bs)
    A, B = frac_decode(aq, as_), frac_decode(bq, bs)
    for i in range(Ra):
        for j in range(Rb):
            exact = sum(A[i][c] * B[j][c] for c in range(C))
            absum = sum(abs(A[i][c] * B[j][c]) for c in range(C))
            # every term is a dyadic rational of few bits; 64 terms: double may round, but barely
            assert abs(Fraction(out[i, j]) - exact) <= Fraction(1, 2**45) * absum
            assert abs(Fraction(ab[i, j]) - absum) <= Fraction(1, 2**45) * absum


def test_gemm_is_not_symmetric_in_its_operands_layout():
    # out is [Ra][Rb]; swapping operands transposes it (catches a transposed write)
    rng = np.random.default_rng(1)
    aq = rng.integers(0, 256, size=(8, 16), dtype=np.uint8)
    bq = rng.integers(0, 256, size=(24, 16), dtype=np.uint8)
    as_ = np.full((8, 1), 127, dtype=np.uint8)
    bs = np.full((24, 1), 126, dtype=np.uint8)
    o1 = oracle.gemm(aq, as_, bq, bs, want_absum=False)
    o2 = oracle.gemm(bq, bs, aq, as_, want_absum=False)
    assert o1.shape == (8, 24) and np.array_equal(o1, o2.T)


def test_gemm_at_matches_full_gemm():
    rng = np.random.default_rng(2)
    aq = rng.integers(0, 256, size=(40, 48), dtype=np.uint8)
    bq = rng.integers(0, 256, size=(24, 48), dtype=np.uint8)
    as_ = rng.integers(120, 130, size=(40, 3), dtype=np.uint8)
    bs = rng.integers(120, 130, size=(24, 3), dtype=np.uint8)
    out, ab = oracle.gemm(aq, as_, bq, bs)
    ii = rng.integers(0, 40, size=100)
    jj = rng.integers(0, 24, size=100)
    o, a = oracle.gemm_at(aq, as_, bq, bs, ii, jj)
    assert np.array_equal(o, out[ii, jj]) and np.array_equal(a, ab[ii, jj])
    with pytest.raises(RuntimeError):
        oracle.gemm_at(aq, as_, bq, bs, np.array([40]), np.array([0]))


def grid_tensor(rows, cols, seed, axis_last=True):
    """Values on the MXFP4 grid: each 32-block along the chosen axis has elements
    code*2^e with one element of magnitude 4 or 6 (so the block's shared exponent is e
    and quantisation reproduces every element exactly)."""
    rng = np.random.default_rng(seed)
    R, C = (rows, cols) if axis_last else (cols, rows)
    mags = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6])
    v = mags[rng.integers(0, 8, size=(R, C))] * rng.choice([-1.0, 1.0], size=(R, C))
    e = rng.integers(-6, 5, size=(R, C // 32))
    pos = rng.integers(0, 32, size=(R, C // 32))
    for r in range(R):
        for b in range(C // 32):
            v[r, b * 32 + pos[r, b]] = rng.choice([4.0, 6.0, -4.0, -6.0])
    v = v * np.repeat(2.0**e, 32, axis=1)
    return v if axis_last else np.ascontiguousarray(v.T)


def to_bits(v):
    t = torch.from_numpy(v.astype(np.float32)).to(torch.bfloat16)
    assert np.array_equal(t.to(torch.float64).numpy(), v)  # exactly representable
    return synth.as_u16(t).copy()


def test_linear_fwd_is_exact_on_grid_inputs():
    M, N, K = 24, 40, 96
    X, W = grid_tensor(M, K, 3), grid_tensor(N, K, 4)
    (xq, xs), (wq, ws) = oracle.linear_fwd_operands(to_bits(X), to_bits(W))
    assert np.array_equal(oracle.dequantize(xq, xs), X) and np.array_equal(oracle.dequantize(wq, ws), W)
    y, _ = oracle.linear_fwd(to_bits(X), to_bits(W))
    assert y.shape == (M, N) and np.array_equal(y, X @ W.T)            # Y = X W^T (App. C.1)


def test_linear_bwd_is_exact_on_grid_inputs():
    M, N, K = 64, 32, 96
    # Dgrad contracts N: dY blocks along its rows (last axis), W blocks down its columns (first axis)
    dY, W = grid_tensor(M, N, 5), grid_tensor(N, K, 6, axis_last=False)
    (gq, gs), (wtq, wts) = oracle.linear_dgrad_operands(to_bits(dY), to_bits(W))
    assert wtq.shape == (K, N // 2)
    dx, _ = oracle.gemm(gq, gs, wtq, wts)
    assert dx.shape == (M, K) and np.array_equal(dx, dY @ W)           # dX = dY W (App. C.2)
    # Wgrad contracts tokens M: both operands blocked down their first axis
    dY2, X2 = grid_tensor(M, N, 7, axis_last=False), grid_tensor(M, K, 8, axis_last=False)
    (gtq, gts), (xtq, xts) = oracle.linear_wgrad_operands(to_bits(dY2), to_bits(X2))
    assert gtq.shape == (N, M // 2) and xtq.shape == (K, M // 2)
    dw, _ = oracle.gemm(gtq, gts, xtq, xts)
    assert dw.shape == (N, K) and np.array_equal(dw, dY2.T @ X2)       # dW = dY^T X (App. C.3)
    # and the composed call agrees with the pieces
    (dx2, _), (dw2, _) = oracle.linear_bwd(to_bits(dY2), to_bits(X2), to_bits(W))
    assert dx2.shape == (M, K) and dw2.shape == (N, K) and np.array_equal(dw2, dw)


@pytest.mark.parametrize("had", [oracle.HAD_NONE, oracle.HAD_DET, oracle.HAD_RANDSIGN, oracle.HAD_DET16,
                                 oracle.HAD_RANDSIGN16])
def test_quantised_linear_approximates_the_real_product(had):
    # the rotation must cancel inside the contraction (App. C): a missing normalisation, a
    # rotation along the wrong axis or a one-sided sign flip would leave an O(1) relative error
    M, N, K = 64, 96, 256
    x = synth.normal(M, K, 1.0, seed=1, stream=synth.STREAM_X)
    w = synth.normal(N, K, 0.02, seed=1, stream=synth.STREAM_W)
    dy = synth.normal(M, N, 1e-3, seed=1, stream=synth.STREAM_DY)
    X, W, dY = (t.to(torch.float64).numpy() for t in (x, w, dy))
    xb, wb, dyb = (synth.as_u16(t) for t in (x, w, dy))
    y, _ = oracle.linear_fwd(xb, wb, had=had, seed=3)
    (dx, _), (dw, _) = oracle.linear_bwd(dyb, xb, wb, had=had, seed=3)
    for got, want in ((y, X @ W.T), (dx, dY @ W), (dw, dY.T @ X)):
        rel = np.linalg.norm(got - want) / np.linalg.norm(want)
        assert rel < 0.2, rel


def test_hadamard_helps_with_outlier_channels():
    # App. A.2: rotation spreads concentrated energy; with 1 hot channel in a block the
    # un-rotated quantiser zeroes its neighbours
    M, N, K = 64, 64, 1024
    x = synth.normal_with_outlier_channels(M, K, seed=2, stream=synth.STREAM_X, fraction=0.004)
    w = synth.normal(N, K, 0.02, seed=2, stream=synth.STREAM_W)
    X, W = x.to(torch.float64).numpy(), w.to(torch.float64).numpy()
    errs = {}
    for had in (oracle.HAD_NONE, oracle.HAD_DET):
        y, _ = oracle.linear_fwd(synth.as_u16(x), synth.as_u16(w), had=had)
        errs[had] = np.linalg.norm(y - X @ W.T) / np.linalg.norm(X @ W.T)
    assert errs[oracle.HAD_DET] < errs[oracle.HAD_NONE]

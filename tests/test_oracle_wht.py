"""Pins for the oracle's Walsh-Hadamard butterflies and for the cancellation
identities of App. C (CPU only)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def sylvester(n):
    return np.array([[(-1) ** bin(i & j).count("1") for j in range(n)] for i in range(n)], dtype=np.int64)


def dense_from_butterfly(n):
    # column j of H is the transform of the unit vector e_j
    cols = [oracle.wht(np.eye(n, dtype=np.float32)[j]) for j in range(n)]
    return np.stack(cols, axis=1)


@pytest.mark.parametrize("n", [16, 32])
def test_butterfly_is_the_sylvester_hadamard_matrix(n):
    H = dense_from_butterfly(n)
    assert set(np.unique(H)) == {-1.0, 1.0}                       # entries +-1 (App. A.2)
    assert np.array_equal(H.astype(np.int64), sylvester(n))
    assert np.array_equal(H, H.T)
    Hi = H.astype(np.int64)
    assert np.array_equal(Hi @ Hi.T, n * np.eye(n, dtype=np.int64))  # H H^T = n I  (App. C)
    assert np.array_equal(Hi.T @ Hi, n * np.eye(n, dtype=np.int64))


@pytest.mark.parametrize("n", [16, 32])
def test_butterfly_equals_dense_product_on_integers(n):
    rng = np.random.default_rng(n)
    H = sylvester(n)
    for _ in range(50):
        x = rng.integers(-1000, 1001, size=n)
        got = oracle.wht(x.astype(np.float32))
        assert np.array_equal(got.astype(np.int64), H @ x)          # all sums < 2^24: exact


def test_butterfly_error_bound_on_reals():
    # five roundings per output at most: |fl(Hx) - Hx| <= 5 * 2^-24 * sum|x| (first order)
    rng = np.random.default_rng(0)
    H = sylvester(32)
    for _ in range(20):
        x = rng.standard_normal(32).astype(np.float32) * np.float32(10.0) ** rng.integers(-3, 4)
        got = oracle.wht(x)
        exact = [sum(Fraction(int(H[i, j])) * Fraction(float(x[j])) for j in range(32)) for i in range(32)]
        bound = 5.5 * 2.0**-24 * float(np.abs(x).astype(np.float64).sum())
        for i in range(32):
            assert abs(Fraction(float(got[i])) - exact[i]) <= bound


def test_parseval_after_normalisation():
    rng = np.random.default_rng(1)
    x = rng.standard_normal(32).astype(np.float32)
    y = oracle.wht(x).astype(np.float64) / np.sqrt(32.0)
    assert abs((y**2).sum() - (x.astype(np.float64) ** 2).sum()) < 1e-5 * (x.astype(np.float64) ** 2).sum()


def rot_rows(a):
    """Apply the unnormalised 32-point butterfly to every 32-block of every row."""
    out = np.empty_like(a, dtype=np.float32)
    for r in range(a.shape[0]):
        for b in range(0, a.shape[1], 32):
            out[r, b:b + 32] = oracle.wht(a[r, b:b + 32].astype(np.float32))
    return out.astype(np.int64)


def test_cancellation_fprop_dgrad_wgrad_exact_on_integers():
    # App. C.1-C.3 with the +-1 matrix: (A H)(B H)^T = 32 A B^T when A and B are rotated
    # along their shared (contraction) axis.  Small integers keep everything exact.
    rng = np.random.default_rng(2)
    M, N, K = 64, 96, 128
    X = rng.integers(-8, 9, size=(M, K))
    W = rng.integers(-8, 9, size=(N, K))
    dY = rng.integers(-8, 9, size=(M, N))
    # Fprop: contract K; X[M,K] and W[N,K] rotated along K
    assert np.array_equal(rot_rows(X) @ rot_rows(W).T, 32 * (X @ W.T))
    # Dgrad: contract N; dY[M,N] along N and W^T[K,N] along N
    assert np.array_equal(rot_rows(dY) @ rot_rows(W.T.copy()).T, 32 * (dY @ W))
    # Wgrad: contract tokens M; dY^T[N,M] and X^T[K,M] along M
    assert np.array_equal(rot_rows(dY.T.copy()) @ rot_rows(X.T.copy()).T, 32 * (dY.T @ X))


def test_cancellation_with_random_signs_exact_on_integers():
    # (X D H)(W D H)^T = 32 X W^T for any +-1 diagonal D shared by both operands
    rng = np.random.default_rng(3)
    X = rng.integers(-8, 9, size=(32, 64))
    W = rng.integers(-8, 9, size=(48, 64))
    mask = oracle.sign_mask(77)
    d = np.array([-1 if (mask >> i) & 1 else 1 for i in range(32)])
    D = np.tile(d, 2)
    assert np.array_equal(rot_rows(X * D) @ rot_rows(W * D).T, 32 * (X @ W.T))
    assert 4 < (d < 0).sum() < 28  # the mask is not degenerate


def test_cancellation_with_random_signs_and_16_point_rotations_exact_on_integers():
    # (X D (H16 + H16))(W D (H16 + H16))^T = 16 X W^T: the randomised rotation of Table 1 (size 16) cancels too
    rng = np.random.default_rng(4)
    X = rng.integers(-8, 9, size=(32, 64))
    W = rng.integers(-8, 9, size=(48, 64))
    mask = oracle.sign_mask(78)
    D = np.tile(np.array([-1 if (mask >> i) & 1 else 1 for i in range(32)]), 2)

    def rot16(a):
        return np.stack([np.concatenate([oracle.wht(r[i:i + 16].astype(np.float32)) for i in range(0, 64, 16)])
                         for r in a]).astype(np.int64)
    assert np.array_equal(rot16(X * D) @ rot16(W * D).T, 16 * (X @ W.T))

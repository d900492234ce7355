"""Pins for the oracle's dense products (the plain definition CSB-MVM must equal)."""
from fractions import Fraction

import numpy as np
import pytest

import csb_inputs
import oracle


def _exact_matvec(A, x):
    """Brute force in exact rational arithmetic (every float is a rational)."""
    R, C = A.shape
    return [float(sum(Fraction(float(A[i, j])) * Fraction(float(x[j])) for j in range(C)))
            for i in range(R)]


@pytest.mark.parametrize("R,C", [(1, 1), (3, 5), (12, 7), (8, 12)])
def test_matvec_brute_force_exact(R, C):
    rng = np.random.default_rng(R * 31 + C)
    A = rng.normal(size=(R, C)).astype(np.float32)
    A[rng.random((R, C)) < 0.5] = 0.0
    x = rng.uniform(-1, 1, size=C).astype(np.float32)
    got = oracle.matvec(A, x)
    ref = _exact_matvec(A, x)
    # float64 accumulation of at most 12 products of float32 pairs (each exact in float64)
    assert np.allclose(got, ref, rtol=0, atol=12 * 2.0 ** -52 * max(1.0, np.abs(ref).max()))


def test_matvec_is_numpy_float64_product():
    m = csb_inputs.small_matrix(3, 200, 150, 16, 16, rate=6.0)
    x = csb_inputs.make_vectors(3, 150, 1)
    ref = m.A.astype(np.float64) @ x.astype(np.float64)
    assert np.allclose(oracle.matvec(m.A, x), ref, rtol=1e-13, atol=1e-15)
    X = csb_inputs.make_vectors(4, 150, 9)
    refm = m.A.astype(np.float64) @ X.astype(np.float64)
    Y = oracle.matmat(m.A, X)
    assert np.allclose(Y, refm, rtol=1e-13, atol=1e-15)
    # column k of the mat-mat product is the mat-vec with right-hand side k
    for k in (0, 4, 8):
        assert np.array_equal(Y[:, k], oracle.matvec(m.A, np.ascontiguousarray(X[:, k])))
    rows = [0, 17, 199]
    assert np.array_equal(oracle.matmat_rows(m.A, rows, X), Y[rows])
    # |.|-sum used by the rounding bound
    refa = np.abs(m.A.astype(np.float64)) @ np.abs(x.astype(np.float64))
    assert np.allclose(oracle.matvec_abs(m.A, x), refa, rtol=1e-13)


def test_matvec_identity_permutation_linearity():
    n = 37
    rng = np.random.default_rng(5)
    x = rng.uniform(-1, 1, n).astype(np.float32)
    w = rng.uniform(-1, 1, n).astype(np.float32)
    assert np.array_equal(oracle.matvec(np.eye(n, dtype=np.float32), x), x.astype(np.float64))
    perm = rng.permutation(n)
    P = np.zeros((n, n), np.float32)
    P[np.arange(n), perm] = 1.0
    assert np.array_equal(oracle.matvec(P, x), x[perm].astype(np.float64))
    A = rng.normal(size=(11, n)).astype(np.float32)
    # alpha, beta powers of two and x+w exact in float32 only by luck; use float64 reference
    lhs = oracle.matvec(A, (0.5 * x).astype(np.float32)) + oracle.matvec(A, (2.0 * w).astype(np.float32))
    rhs = 0.5 * oracle.matvec(A, x) + 2.0 * oracle.matvec(A, w)
    assert np.allclose(lhs, rhs, rtol=1e-14, atol=1e-15)


def test_transposed_operand_would_fail():
    """A non-square, non-symmetric case: A x differs from what A^T-style indexing gives."""
    A = np.arange(6, dtype=np.float32).reshape(2, 3)
    x = np.array([1, 10, 100], np.float32)
    assert oracle.matvec(A, x).tolist() == [210.0, 543.0]
    X = np.array([[1, 0], [0, 1], [1, 1]], np.float32)
    assert oracle.matmat(A, X).tolist() == [[2.0, 3.0], [8.0, 9.0]]

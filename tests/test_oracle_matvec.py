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


# ---- the float32 CSB-MVM on the encoded arrays (the benchmark's like-for-like CPU baseline) ----

def test_csb_matvec_f32_hand_worked_example():
    """The two-block example of tests/golden: y = [10, 25, -8, 35] for x = 1..8."""
    A = np.array([[0, 1, 0, 2, 0, 0, 0, 0],
                  [0, 0, 0, 0, 5, 0, 0, 0],
                  [0, 3, 0, 4, -6, 0, 0, 0],
                  [0, 0, 0, 0, 7, 0, 0, 0]], np.float32)
    x = np.arange(1, 9, dtype=np.float32)
    y = oracle.csb_matvec_f32(oracle.csb_encode(A, 4, 4), x)
    assert y.dtype == np.float32 and np.array_equal(y, np.array([10, 25, -8, 35], np.float32))


@pytest.mark.parametrize("R,C,br,bc", [(1, 1, 1, 1), (12, 7, 4, 3), (37, 53, 8, 8), (130, 257, 32, 32), (70, 300, 16, 64)])
def test_csb_matvec_f32_exact_on_small_integers(R, C, br, bc):
    """Small integer entries make every float32 product and sum exact, so the walk over the
    encoded arrays must reproduce the float64 product of the dense matrix bit for bit: a wrong
    offset, a swapped index array or a missed block cannot hide behind rounding."""
    rng = np.random.default_rng(R * 7 + C)
    A = rng.integers(-8, 9, size=(R, C)).astype(np.float32)
    A[rng.random((R, C)) < 0.6] = 0.0
    A[:, rng.random(C) < 0.2] = 0.0                       # whole columns and rows pruned away
    A[rng.random(R) < 0.2, :] = 0.0
    x = rng.integers(-8, 9, size=C).astype(np.float32)
    y = oracle.csb_matvec_f32(oracle.csb_encode(A, br, bc), x)
    assert np.array_equal(y.astype(np.float64), oracle.matvec(A, x))


def test_csb_matvec_f32_within_the_float32_dot_product_bound():
    m = csb_inputs.small_matrix(9, 300, 421, 32, 32, rate=5.0)
    x = csb_inputs.make_vectors(9, 421, 1)
    y = oracle.csb_matvec_f32(oracle.csb_encode(m.A, 32, 32), x).astype(np.float64)
    ref, scale = oracle.matvec(m.A, x), oracle.matvec_abs(m.A, x)
    k = np.count_nonzero(m.A, axis=1)
    assert np.all(np.abs(y - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * scale + 1e-30)
    assert np.any(y != ref)                               # it does round: a float32 path, as claimed
    Z = np.zeros((40, 48), np.float32)
    assert np.array_equal(oracle.csb_matvec_f32(oracle.csb_encode(Z, 16, 16), x[:48]), np.zeros(40, np.float32))

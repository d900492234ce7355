"""Pins for the oracle's CSB projection (the pruning step inside Algorithm 1, Sec. 3.2.2).

The oracle takes its ranking decisions in float32 with a fixed summation order; these
tests pin it to things that do not depend on that arithmetic: a hand-worked example, an
exact-integer brute force (small integer entries make every sum exact, so the ranking is a
matter of integers), and invariants the description fixes (kept counts per block-column and
block-row, the cross-point pattern, untouched survivors, rate 1 = identity, nesting)."""
from fractions import Fraction
import math

import numpy as np
import pytest

import oracle
from helpers import read_golden


def prune_count(n, rate):
    return min(n, max(0, math.floor(n * (1.0 - 1.0 / math.sqrt(rate)) + 0.5)))


def brute_force_project(W, br, bc, rate):
    """Same procedure with exact rational sums and Python's sort on (sum, position)."""
    R, C = W.shape
    Z = [[Fraction(int(v)) for v in row] for row in W]
    for c0 in range(0, C, bc):
        cols = range(c0, min(C, c0 + bc))
        order = sorted(range(R), key=lambda i: (sum(Z[i][c] ** 2 for c in cols), i))
        for i in order[:prune_count(R, rate)]:
            for c in cols:
                Z[i][c] = Fraction(0)
    for r0 in range(0, R, br):
        rows = range(r0, min(R, r0 + br))
        order = sorted(range(C), key=lambda c: (sum(Z[i][c] ** 2 for i in rows), c))
        for c in order[:prune_count(C, rate)]:
            for i in rows:
                Z[i][c] = Fraction(0)
    return np.array([[float(v) for v in row] for row in Z], dtype=np.float32)


def test_hand_worked_projection():
    g = read_golden("projection_example.txt")
    W = np.array(g["A"], dtype=np.float32)
    br, bc, rate = int(g["br"][0]), int(g["bc"][0]), g["rate"][0]
    Z = oracle.csb_project(W, br, bc, rate)
    expect = np.array([g[f"z_{i}"] for i in range(W.shape[0])], dtype=np.float32)
    assert np.array_equal(Z, expect)
    enc = oracle.csb_encode(Z, br, bc)
    assert list(enc.nrows) == [int(v) for v in g["nrows"]]
    assert list(enc.ncols) == [int(v) for v in g["ncols"]]
    # the fixture also records the state after RowPrune: ColumnPrune only removes from it
    rows_only = np.array([g[f"after_rows_{i}"] for i in range(W.shape[0])], dtype=np.float32)
    assert not np.any((Z != 0) & (rows_only == 0))
    assert np.array_equal(Z[Z != 0], rows_only[Z != 0])


@pytest.mark.parametrize("seed", range(12))
def test_projection_matches_exact_integer_brute_force(seed):
    rng = np.random.default_rng(seed)
    R, C = int(rng.integers(1, 13)), int(rng.integers(1, 13))
    br, bc = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    rate = float(rng.choice([1.0, 1.5, 2.0, 4.0, 9.0, 16.0]))
    W = rng.integers(-4, 5, size=(R, C)).astype(np.float32)      # many ties, many zeros
    assert np.array_equal(oracle.csb_project(W, br, bc, rate), brute_force_project(W, br, bc, rate))


@pytest.mark.parametrize("R,C,br,bc,rate", [(64, 96, 16, 16, 4.0), (100, 70, 32, 8, 10.0), (37, 53, 8, 16, 2.5),
                                            (128, 128, 32, 32, 16.0)])
def test_projection_invariants(R, C, br, bc, rate):
    rng = np.random.default_rng(R + C)
    W = rng.normal(0, 1, (R, C)).astype(np.float32)
    Z = oracle.csb_project(W, br, bc, rate)
    keep = Z != 0
    assert np.array_equal(Z[keep], W[keep])                       # survivors keep their bits
    kr, kc = prune_count(R, rate), prune_count(C, rate)
    # RowPrune: in every block-column exactly R - kr row segments survive it; after ColumnPrune a
    # row segment is non-zero only if it survived RowPrune (Gaussian entries: no accidental zeros)
    for c0 in range(0, C, bc):
        seg = keep[:, c0:c0 + bc].any(axis=1)
        assert seg.sum() <= R - kr
    for r0 in range(0, R, br):
        seg = keep[r0:r0 + br, :].any(axis=0)
        assert seg.sum() <= C - kc
    # inside every block the survivors are exactly the cross-points of kept rows and columns
    for r0 in range(0, R, br):
        for c0 in range(0, C, bc):
            b = keep[r0:r0 + br, c0:c0 + bc]
            assert np.array_equal(b, np.outer(b.any(axis=1), b.any(axis=0)))
    # overall density close to 1 / rate (both passes hit their counts exactly; the product of
    # the two kept shares is what the rate promises)
    assert abs(keep.mean() - (1 - kr / R) * (1 - kc / C)) < 0.08
    # rate 1 prunes nothing; a higher rate keeps a subset of the row segments a lower one keeps
    assert np.array_equal(oracle.csb_project(W, br, bc, 1.0), W)
    Z_hi = oracle.csb_project(W, br, bc, rate * 2)
    for c0 in range(0, C, bc):
        lo_rows = keep[:, c0:c0 + bc].any(axis=1)
        hi_rows = (Z_hi[:, c0:c0 + bc] != 0).any(axis=1)
        assert not np.any(hi_rows & ~lo_rows)


def test_projection_by_construction():
    """Magnitudes that make the answer obvious: row i of every block-column carries i + 1, so
    RowPrune removes the first rows; afterwards every column of a block-row has the same sum
    except those scaled up on purpose, so ColumnPrune removes the earliest unscaled ones."""
    R, C, br, bc = 8, 8, 4, 4
    W = np.tile((np.arange(R, dtype=np.float32) + 1)[:, None], (1, C))
    W[:, [1, 6]] *= 3.0
    Z = oracle.csb_project(W, br, bc, 4.0)                         # each pass removes half
    assert not Z[:4].any()                                         # rows 0-3 are the weakest in both block-columns
    kept_cols = np.flatnonzero(Z[4:].any(axis=0))
    # block-row 1: columns 1 and 6 are strongest; among the equal rest the earlier positions go
    assert list(kept_cols) == [1, 5, 6, 7]
    # block-row 0 is all zero after RowPrune: ties by position, columns 0-3 are "pruned", nothing to see
    assert np.array_equal(Z[4:, kept_cols], W[4:, kept_cols])


# ---- the float32 reading against the plain float64 definition ------------------------------------

GAUSS_CASES = [(4, 6, 2, 3, 4.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0), (130, 257, 32, 32, 10.0),
               (96, 96, 32, 16, 1.0), (70, 300, 16, 64, 16.0), (300, 40, 128, 8, 2.0), (513, 100, 256, 256, 12.0),
               (1, 1, 1, 1, 4.0), (1025, 3, 64, 2, 25.0)]


def differing_decisions(W, br, bc, rate):
    """Entries kept by one of the two projections and removed by the other."""
    return int(np.count_nonzero((oracle.csb_project(W, br, bc, rate) != 0) != (oracle.csb_project_f64(W, br, bc, rate) != 0)))


@pytest.mark.parametrize("seed", range(6))
def test_float64_projection_matches_exact_integer_brute_force(seed):
    rng = np.random.default_rng(100 + seed)
    R, C = int(rng.integers(1, 13)), int(rng.integers(1, 13))
    br, bc = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    rate = float(rng.choice([1.5, 2.0, 4.0, 9.0]))
    W = rng.integers(-4, 5, size=(R, C)).astype(np.float32)
    assert np.array_equal(oracle.csb_project_f64(W, br, bc, rate), brute_force_project(W, br, bc, rate))


def test_float32_decisions_equal_float64_decisions_on_the_tested_inputs():
    """The projection is specified here with its ranking sums in float32 (the device's
    arithmetic).  On every Gaussian input the device tests use (same seeds, same shapes) the
    plain float64 definition takes the same decisions: zero differing entries.  The count is
    what the design notes quote."""
    total = 0
    for R, C, br, bc, rate in GAUSS_CASES:
        rng = np.random.default_rng(R * 7 + C)
        total += differing_decisions(rng.normal(0, 0.05, (R, C)).astype(np.float32), br, bc, rate)
    total += differing_decisions(np.random.default_rng(11).normal(0, 0.05, (512, 640)).astype(np.float32), 32, 32, 10.0)
    total += differing_decisions(np.random.default_rng(0).normal(0, 0.05, (2048, 2048)).astype(np.float32), 32, 32, 12.0)
    assert total == 0


def test_float32_and_float64_readings_part_only_at_a_near_tie():
    """Two segments whose sums differ by less than one float32 unit in the last place: float32
    sees a tie and removes the earlier position, float64 removes the smaller sum."""
    W = np.array([[1.0, 2.0 ** -13], [1.0, 0.0]], dtype=np.float32)       # sums 1 + 2^-26 and 1
    Z32 = oracle.csb_project(W, 2, 2, 4.0)                                 # each pass removes one of two
    Z64 = oracle.csb_project_f64(W, 2, 2, 4.0)
    assert not Z32[0].any() and Z32[1].any()
    assert Z64[0].any() and not Z64[1].any()

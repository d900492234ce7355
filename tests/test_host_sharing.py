"""csb_sharing_model (host only) against the oracle's brute force on small matrices: cycle
counts without sharing and with one-directional sharing are exact optima and must agree
exactly, and so must the 2-D figure on grids of at most four PEGroups, where the library
searches exhaustively; on larger grids the 2-D figure is an upper bound on the optimum that
must lie between the exact 2-D optimum and the better one-directional one."""
import numpy as np
import pytest

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbError


def counts(A, br, bc):
    enc = oracle.csb_encode(A, br, bc)
    nbr, nbc = -(-A.shape[0] // br), -(-A.shape[1] // bc)
    return np.asarray(enc.nrows).reshape(nbr, nbc), np.asarray(enc.ncols).reshape(nbr, nbc)


@pytest.mark.parametrize("R,C,br,bc,P,Q,K,L,rate", [(24, 32, 8, 8, 2, 2, 2, 2, 2.0), (40, 24, 8, 8, 2, 2, 2, 2, 1.5), (30, 50, 6, 10, 2, 3, 2, 2, 2.0),
                                                    (16, 64, 8, 8, 2, 2, 1, 3, 1.3), (64, 16, 8, 8, 2, 2, 3, 1, 1.3), (36, 36, 12, 12, 4, 4, 2, 2, 1.2)])
def test_against_brute_force(R, C, br, bc, P, Q, K, L, rate):
    for seed in range(2):
        A = csb_inputs.small_matrix(seed + R, R, C, br, bc, rate=rate).A
        nr, nc = counts(A, br, bc)
        ref = oracle.sharing_model(nr, nc, P, Q, K, L, exact_2d=True)
        got = CsbMatrix(A, br, bc).sharing_model(P, Q, K, L)
        for k in ("work", "iterations", "cycles_none", "cycles_horizontal", "cycles_vertical"):
            assert got[k] == ref[k], (k, got[k], ref[k])
        assert got["exact_2d"] == (1 if K * L <= 4 else 0)
        assert got["cycles_2d"] == ref["cycles_2d"], (got["cycles_2d"], ref["cycles_2d"])      # every grid here has at most four PEGroups
        for k in ("none", "horizontal", "vertical", "2d"):
            assert abs(got["eff_" + k] - ref["eff_" + k]) < 1e-12


def test_2d_figure_is_the_optimum_on_small_grids():
    for seed in range(6):
        A = csb_inputs.small_matrix(100 + seed, 32, 32, 8, 8, rate=1.6).A
        nr, nc = counts(A, 8, 8)
        ref = oracle.sharing_model(nr, nc, 2, 2, 2, 2, exact_2d=True)
        got = CsbMatrix(A, 8, 8).sharing_model(2, 2, 2, 2)
        assert got["exact_2d"] == 1 and got["cycles_2d"] == ref["cycles_2d"] and got["eff_2d"] == ref["eff_2d"]


def test_2d_figure_on_a_larger_grid_is_a_bound():
    """Six PEGroups: the library improves one PEGroup's choice at a time, so its time is never
    below the optimum (brute force) and never above the one-directional schedules'."""
    for seed in range(3):
        A = csb_inputs.small_matrix(200 + seed, 8, 12, 4, 4, rate=1.4).A
        nr, nc = counts(A, 4, 4)
        ref = oracle.sharing_model(nr, nc, 2, 2, 2, 3, exact_2d=True)
        got = CsbMatrix(A, 4, 4).sharing_model(2, 2, 2, 3)
        assert got["exact_2d"] == 0
        assert ref["cycles_2d"] <= got["cycles_2d"] <= min(ref["cycles_horizontal"], ref["cycles_vertical"])


def test_workload_shape_and_errors():
    m = csb_inputs.make_rnn(csb_inputs.CONFIGS["cfg2"], T=1).W[0]
    M = CsbMatrix(m.A, m.br, m.bc)
    r = M.sharing_model()                                  # the paper's evaluation: 4 x 4 PEGroups of 4 x 4 PEs
    assert r["work"] == int(M.view()["nnz"]) and r["iterations"] == 16 * 6
    assert 0 < r["eff_none"] <= r["eff_horizontal"] <= 1 and r["eff_none"] <= r["eff_vertical"] <= 1
    assert max(r["eff_horizontal"], r["eff_vertical"]) <= r["eff_2d"] <= 1 and r["exact_2d"] == 0
    for bad in ((0, 4, 4, 4), (4, 4, 9, 4), (4, 4, 4, 0)):
        with pytest.raises(CsbError):
            M.sharing_model(*bad)

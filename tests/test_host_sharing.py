"""csb_sharing_model (host only) against the oracle's brute force on small matrices: cycle
counts without sharing and with one-directional sharing are exact optima and must agree
exactly; the 2-D figure is an upper bound on the optimum that must lie between the exact 2-D
optimum and the better one-directional one."""
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
        assert ref["cycles_2d"] <= got["cycles_2d"] <= min(ref["cycles_horizontal"], ref["cycles_vertical"])
        for k in ("none", "horizontal", "vertical"):
            assert abs(got["eff_" + k] - ref["eff_" + k]) < 1e-12


def test_2d_figure_is_close_to_the_optimum():
    """The 2-D schedule is found by local improvement, so its time is an upper bound on the
    optimum: never below it, and within 15 % of it on these small cases."""
    for seed in range(6):
        A = csb_inputs.small_matrix(100 + seed, 32, 32, 8, 8, rate=1.6).A
        nr, nc = counts(A, 8, 8)
        ref = oracle.sharing_model(nr, nc, 2, 2, 2, 2, exact_2d=True)
        got = CsbMatrix(A, 8, 8).sharing_model(2, 2, 2, 2)
        assert ref["cycles_2d"] <= got["cycles_2d"] <= 1.15 * ref["cycles_2d"]


def test_workload_shape_and_errors():
    m = csb_inputs.make_rnn(csb_inputs.CONFIGS["cfg2"], T=1).W[0]
    M = CsbMatrix(m.A, m.br, m.bc)
    r = M.sharing_model()                                  # the paper's evaluation: 4 x 4 PEGroups of 4 x 4 PEs
    assert r["work"] == int(M.view()["nnz"]) and r["iterations"] == 16 * 6
    assert 0 < r["eff_none"] <= r["eff_horizontal"] <= 1 and r["eff_none"] <= r["eff_vertical"] <= 1
    assert max(r["eff_horizontal"], r["eff_vertical"]) <= r["eff_2d"] <= 1
    for bad in ((0, 4, 4, 4), (4, 4, 9, 4), (4, 4, 4, 0)):
        with pytest.raises(CsbError):
            M.sharing_model(*bad)

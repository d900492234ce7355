"""csb_spmv_static (the entry point that allocates nothing: its partial sums of shared row
tiles go through a device array built into the library) against csb_spmv with a caller's
workspace: the same kernels, so the results must be equal bit for bit; and both against the
oracle at the bar of csb_spmv.  Two calls in a row, the second on a smaller matrix, so the
second sees what the first left in the buffer."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix
from paper_2005_05758_amd.binding import CsbError, lib
from helpers import rel_max_err

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def one_case(R, C, br, bc, rate, n_chunks, seed):
    say(f"[spmv_static] {R}x{C} block {br}x{bc} rate {rate} n_chunks {n_chunks}")
    m = csb_inputs.small_matrix(seed, R, C, br, bc, rate=rate)
    x = csb_inputs.make_vectors(seed + 1, C, 1)
    M = CsbMatrix(m.A, br, bc)
    st = M.plan(n_chunks, 2)                 # equal split: row tiles shared between workgroups, merged through memory
    assert st["n_shared_tiles"] > 0 and M.workspace_bytes(1) > 0, "the case must use the buffer"
    assert M.workspace_bytes(1) <= int(lib().csb_spmv_static_limit())
    M.validate()
    M.upload()
    xd = torch.from_numpy(x).cuda()
    y_ws = M.spmv(xd)                        # caller's workspace
    y_st = M.spmv_static(xd)                 # built-in buffer
    y_st2 = M.spmv_static(xd)                # again: the buffer holds the previous call's words
    torch.cuda.synchronize()
    assert torch.equal(y_ws, y_st) and torch.equal(y_st, y_st2)
    D = oracle.csb_decode(oracle.csb_encode(m.A, br, bc))
    ref = oracle.matvec(D, x)
    got = y_st.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert rel_max_err(got, ref) <= 1e-5
    k = np.count_nonzero(D, axis=1)
    bound = 2.0 * np.maximum(k, 1) * 2.0 ** -24 * oracle.matvec_abs(D, x) + 1e-30
    assert np.all(np.abs(got - ref) <= bound)
    return M


def test_spmv_static_two_calls_second_smaller():
    keep = one_case(1500, 900, 32, 32, 6.0, 48, 21)      # larger first
    one_case(300, 257, 16, 32, 4.0, 24, 22)              # then a smaller one on the same buffer
    # and the first matrix once more, after another matrix has used the buffer
    x = torch.from_numpy(csb_inputs.make_vectors(22, 900, 1)).cuda()
    a, b = keep.spmv(x), keep.spmv_static(x)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_spmv_static_row_owned_plan_and_errors():
    m = csb_inputs.small_matrix(5, 200, 150, 16, 16, rate=4.0)
    x = torch.from_numpy(csb_inputs.make_vectors(6, 150, 1)).cuda()
    M = CsbMatrix(m.A, 16, 16)
    with pytest.raises(CsbError):
        M.spmv_static(x)                     # not planned
    M.plan()
    M.upload()
    a, b = M.spmv(x), M.spmv_static(x)       # row-owned layout: no partial sums in memory
    torch.cuda.synchronize()
    assert torch.equal(a, b)

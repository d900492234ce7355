"""Parity of csb_project (through the C ABI) against the oracle's projection: the result is a
matter of integer decisions (which segments go) and copied bits, so the bar is bit-exact."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, project
from helpers import rel_max_err

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_project(W, br, bc, rate, tag="", f64_too=False):
    say(f"[project] {tag} shape={W.shape} block={br}x{bc} rate={rate}")
    ref = oracle.csb_project(W, br, bc, rate)
    Wd = torch.from_numpy(W).cuda()
    Z = project(Wd, br, bc, rate)
    torch.cuda.synchronize()
    got = Z.cpu().numpy()
    assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), int(np.count_nonzero(got != ref))
    assert np.array_equal(Wd.cpu().numpy().view(np.uint32), W.view(np.uint32))   # the input is untouched
    if f64_too:
        # no two ranking sums at a cut are close enough on these inputs for float32 and float64
        # to rank them differently (counted on the CPU side), so the device result is also the
        # plain float64 definition's, bit for bit
        ref64 = oracle.csb_project_f64(W, br, bc, rate)
        assert np.array_equal(got.view(np.uint32), ref64.view(np.uint32)), int(np.count_nonzero(got != ref64))
    return got


@pytest.mark.parametrize("R,C,br,bc,rate", [
    (4, 6, 2, 3, 4.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0), (130, 257, 32, 32, 10.0),
    (96, 96, 32, 16, 1.0), (70, 300, 16, 64, 16.0), (300, 40, 128, 8, 2.0), (513, 100, 256, 256, 12.0),
    (1, 1, 1, 1, 4.0), (1025, 3, 64, 2, 25.0),
    # the 16-byte forms of the kernels: whole blocks of 16 / 32 / 64 columns, with a ragged last
    # group of rows, more than 256 blocks in a row, and row counts that are no multiple of 8
    (100, 128, 16, 32, 5.0), (72, 320, 8, 64, 9.0), (40, 9600, 8, 32, 12.0), (24, 4800, 8, 16, 7.0),
    (264, 544, 24, 32, 10.0)])
def test_project_small_shapes(R, C, br, bc, rate):
    rng = np.random.default_rng(R * 7 + C)
    check_project(rng.normal(0, 0.05, (R, C)).astype(np.float32), br, bc, rate, tag="gauss", f64_too=True)
    check_project(rng.integers(-3, 4, (R, C)).astype(np.float32), br, bc, rate, tag="ties")   # many equal sums, zeros


def test_project_special_values_and_in_place():
    rng = np.random.default_rng(5)
    W = rng.normal(0, 1, (64, 96)).astype(np.float32)
    W[3, 7] = np.nan
    W[10, 40] = np.inf
    W[20, :] = 0.0
    W[:, 50] = -0.0
    check_project(W, 16, 32, 4.0, tag="nan-inf-zero")
    # in place, strided rows
    big = torch.from_numpy(rng.normal(0, 1, (64, 128)).astype(np.float32)).cuda()
    view = big[:, :96]
    ref = oracle.csb_project(view.cpu().numpy().copy(), 16, 32, 9.0)
    tail = big[:, 96:].clone()
    project(view, 16, 32, 9.0, out=view)
    torch.cuda.synchronize()
    assert np.array_equal(view.cpu().numpy().view(np.uint32), ref.view(np.uint32))
    assert torch.equal(big[:, 96:], tail)


def test_project_then_pack_then_spmv():
    """The projection's output is what csb_pack expects: the density lands near 1/rate (a
    little above it: ColumnPrune prefers columns in blocks that RowPrune already thinned), the
    encoding matches the oracle's, and the mat-vec of the packed matrix matches the oracle's."""
    rng = np.random.default_rng(11)
    W = rng.normal(0, 0.05, (512, 640)).astype(np.float32)
    Z = check_project(W, 32, 32, 10.0, tag="pipeline", f64_too=True)
    assert abs(np.count_nonzero(Z) / Z.size - 0.1) < 0.02
    M = CsbMatrix(Z, 32, 32)
    enc = oracle.csb_encode(Z, 32, 32)
    v = M.view()
    for k in ("nrows", "ncols", "rowidx", "colidx"):
        assert np.array_equal(v[k], getattr(enc, k))
    M.plan()
    M.upload()
    x = csb_inputs.make_vectors(3, 640, 1)
    y = M.spmv(torch.from_numpy(x.reshape(-1)).cuda())
    torch.cuda.synchronize()
    assert rel_max_err(y.cpu().numpy().astype(np.float64), oracle.matvec(Z, x.reshape(-1))) <= 1e-5


def test_project_full_size():
    """8192 x 8192, block 32, 12x: the stress matrix's shape, as bench.py runs it."""
    rng = np.random.default_rng(0)
    W = rng.normal(0, 0.05, (8192, 8192)).astype(np.float32)
    Z = check_project(W, 32, 32, 12.0, tag="8192", f64_too=True)
    assert abs(np.count_nonzero(Z) / Z.size - 1 / 12.0) < 0.02

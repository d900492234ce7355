"""Parity of csb_spmm (fp32 MFMA, through the C ABI) against the oracle's float64 product on
the decompressed matrix.  Same tolerances as the mat-vec: norm-wise 1e-5 and the element-wise
bound 2 k_i 2^-24 sum_j |a_ij x_jk| (any summation order of a float32 dot product)."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix
from helpers import rel_max_err

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_spmm(A, br, bc, X, tag="", rows=None):
    say(f"[spmm] {tag} shape={A.shape} block={br}x{bc} batch={X.shape[1]}")
    D = oracle.csb_decode(oracle.csb_encode(A, br, bc)) if rows is None else A
    M = CsbMatrix(A, br, bc)
    M.plan()
    if rows is None:
        M.validate()
    M.upload()
    Xd = torch.from_numpy(X).cuda()
    Y = M.spmm(Xd)
    torch.cuda.synchronize()
    got = Y.cpu().numpy().astype(np.float64)
    assert got.shape == (A.shape[0], X.shape[1]) and np.all(np.isfinite(got))
    if rows is None:
        ref = oracle.matmat(D, X)
        sel = np.arange(A.shape[0])
    else:
        sel = np.asarray(rows)
        ref = oracle.matmat_rows(D, sel, X)
        got = got[sel]
    assert rel_max_err(got, ref) <= 1e-5, rel_max_err(got, ref)
    k = np.count_nonzero(D[sel], axis=1)[:, None]
    scale = np.abs(D[sel].astype(np.float64)) @ np.abs(X.astype(np.float64))
    assert np.all(np.abs(got - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * scale + 1e-30)
    Y2 = M.spmm(Xd)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)                       # bitwise reproducible
    return M, Y


@pytest.mark.parametrize("R,C,br,bc,rate", [
    (4, 8, 4, 4, 2.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0), (130, 257, 32, 32, 5.0),
    (96, 96, 32, 16, 4.0), (70, 300, 16, 64, 4.0), (300, 40, 128, 8, 3.0), (513, 100, 256, 256, 2.0),
    (64, 64, 64, 64, 1.0)])
@pytest.mark.parametrize("batch", [1, 5, 16, 33, 64])
def test_spmm_small_shapes(R, C, br, bc, rate, batch):
    m = csb_inputs.small_matrix(R * 3 + C, R, C, br, bc, rate=rate)
    X = csb_inputs.make_vectors(R + C, C, max(batch, 2))[:, :batch].copy()
    check_spmm(m.A, br, bc, X, tag="small")


def test_spmm_degenerate_and_column_consistency():
    X = csb_inputs.make_vectors(1, 48, 8)
    check_spmm(np.zeros((40, 48), np.float32), 16, 16, X, tag="all-zero")
    I = np.eye(48, dtype=np.float32)
    _, Y = check_spmm(I, 16, 16, X, tag="identity")
    assert np.array_equal(Y.cpu().numpy(), X)
    m = csb_inputs.small_matrix(7, 160, 200, 32, 32, rate=5.0, law="beta")
    Xb = csb_inputs.make_vectors(2, 200, 20)
    M, Y = check_spmm(m.A, 32, 32, Xb, tag="beta")
    # column k of the batched product is the mat-vec with right-hand side k
    for kcol in (0, 7, 19):
        y = M.spmv(torch.from_numpy(np.ascontiguousarray(Xb[:, kcol])).cuda())
        torch.cuda.synchronize()
        assert rel_max_err(Y[:, kcol].cpu().numpy(), y.cpu().numpy()) <= 1e-5
    # leading dimensions larger than the batch
    Xw = torch.from_numpy(csb_inputs.make_vectors(3, 200, 40)).cuda()
    Yw = torch.zeros((160, 50), dtype=torch.float32, device="cuda")
    M.spmm(Xw[:, :20], Yw[:, :20])
    torch.cuda.synchronize()
    ref = oracle.matmat(m.A, Xw[:, :20].cpu().numpy().copy())
    assert rel_max_err(Yw[:, :20].cpu().numpy(), ref) <= 1e-5 and float(Yw[:, 20:].abs().max()) == 0.0


def test_spmm_wide_rows_several_record_segments():
    """Two row tiles of 750 blocks each: a tile's records exceed the kernel's LDS window, so it
    is staged in several segments; and the widest input the 16-bit offsets allow."""
    m = csb_inputs.small_matrix(21, 40, 12000, 32, 16, rate=2.0)
    X = csb_inputs.make_vectors(4, 12000, 24)
    M, _ = check_spmm(m.A, 32, 16, X, tag="wide")
    m = csb_inputs.small_matrix(22, 70, 16383, 32, 64, rate=6.0)
    X = csb_inputs.make_vectors(5, 16383, 8)
    check_spmm(m.A, 32, 64, X, tag="max-cols")


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg4"])
def test_spmm_rnn_matrices(name):
    cfg = csb_inputs.CONFIGS[name]
    m = csb_inputs.make_rnn(cfg, T=1, batch=1).W[0]
    X = csb_inputs.make_vectors(3, m.cols, 64)
    rows = None if m.rows * m.cols * 64 < 3e8 else np.arange(0, m.rows, 16)
    check_spmm(m.A, m.br, m.bc, X, tag=name, rows=rows)


def test_spmm_full_size_stress():
    """8192 x 8192 heavy-tailed, 128 right-hand sides; the oracle checks 256 sampled rows."""
    m = csb_inputs.make_mat(csb_inputs.CONFIGS["cfg5"])
    X = csb_inputs.make_vectors(5, m.cols, 128)
    rows = np.random.default_rng(0).choice(m.rows, 256, replace=False)
    check_spmm(m.A, m.br, m.bc, X, tag="cfg5", rows=np.sort(rows))


@pytest.mark.parametrize("R,C,br,bc,batch", [(8192, 96, 32, 32, 64), (8192, 70, 32, 16, 128), (4100, 130, 16, 32, 52),
                                             (16384, 40, 64, 8, 48), (8192, 96, 32, 32, 60)])
def test_spmm_wide_form(R, C, br, bc, batch):
    """Tall matrices: enough row tiles that a workgroup takes 64 right-hand sides with 16-byte
    loads (batch a multiple of 4; ragged last batch tile; both wavefront counts)."""
    m = csb_inputs.small_matrix(R + C + batch, R, C, br, bc, rate=4.0)
    X = csb_inputs.make_vectors(batch, C, batch)
    check_spmm(m.A, br, bc, X, tag="wide-form")
    # a strided view of a wider array (leading dimension above the batch, still 16-byte rows)
    Xw = csb_inputs.make_vectors(batch + 1, C, batch + 12)
    M = CsbMatrix(m.A, br, bc)
    M.plan()
    M.upload()
    Xd = torch.from_numpy(Xw).cuda()
    Y = M.spmm(Xd[:, 4:4 + batch])
    torch.cuda.synchronize()
    ref = oracle.matmat(m.A, np.ascontiguousarray(Xw[:, 4:4 + batch]))
    assert rel_max_err(Y.cpu().numpy(), ref) <= 1e-5
    # unaligned view: takes the narrow form, same result within tolerance
    Y1 = M.spmm(Xd[:, 1:1 + batch])
    torch.cuda.synchronize()
    ref1 = oracle.matmat(m.A, np.ascontiguousarray(Xw[:, 1:1 + batch]))
    assert rel_max_err(Y1.cpu().numpy(), ref1) <= 1e-5

"""Pins for the oracle's CSB encoder/decoder (Sec. 3.1.1) -- CPU only."""
import itertools

import numpy as np
import pytest

import csb_inputs
import oracle
from helpers import read_golden


def _check_arrays(enc, g, tag):
    assert enc.nrows.tolist() == g["nrows_" + tag]
    assert enc.ncols.tolist() == g["ncols_" + tag]
    assert enc.rowidx.tolist() == g["rowidx_" + tag]
    assert enc.colidx.tolist() == g["colidx_" + tag]
    assert enc.val.tolist() == g["val_" + tag]
    assert enc.val_off.tolist() == g["val_off"]
    assert enc.row_off.tolist() == g["row_off"]
    assert enc.col_off.tolist() == g["col_off"]


def test_hand_worked_two_block_example():
    g = read_golden("two_block_example.txt")
    A = np.array(g["A"], np.float32)
    assert A.shape == (4, 8)
    enc = oracle.csb_encode(A, 4, 4)
    _check_arrays(enc, g, "a")
    assert enc.nnz == 7
    x = np.array(g["x"], np.float32)
    assert oracle.matvec(oracle.csb_decode(enc), x).tolist() == g["y_a"]
    # explicit zero at a cross-point: same indices, Val carries the zero
    A2 = A.copy()
    A2[2, 3] = 0.0
    enc2 = oracle.csb_encode(A2, 4, 4)
    _check_arrays(enc2, g, "b")
    assert oracle.matvec(oracle.csb_decode(enc2), x).tolist() == g["y_b"]


def _python_encode(A, br, bc):
    """The definition again in the most literal Python (sets and comprehensions)."""
    R, C = A.shape
    nrows, ncols, ri, ci, val = [], [], [], [], []
    for r0 in range(0, R, br):
        for c0 in range(0, C, bc):
            blk = A[r0:r0 + br, c0:c0 + bc]
            rows = sorted({i for i, j in zip(*np.nonzero(blk))})
            cols = sorted({j for i, j in zip(*np.nonzero(blk))})
            nrows.append(len(rows)); ncols.append(len(cols))
            ri += rows; ci += cols
            val += [blk[i, j] for i in rows for j in cols]
    return nrows, ncols, ri, ci, val


@pytest.mark.parametrize("R,C,br,bc", [(4, 8, 4, 4), (7, 5, 3, 2), (12, 12, 5, 5), (9, 11, 4, 3),
                                      (1, 1, 1, 1), (6, 6, 6, 6), (10, 3, 1, 3), (5, 12, 2, 5)])
def test_tiny_matrices_against_literal_definition(R, C, br, bc):
    for seed in range(4):
        rng = np.random.default_rng(100 * seed + R * 13 + C)
        A = rng.normal(size=(R, C)).astype(np.float32)
        A[rng.random((R, C)) < 0.6] = 0.0            # unstructured zeros: the encoder must still cope
        if seed == 1:
            A[:br] = 0.0                              # empty block-row
        if seed == 2:
            A = np.abs(A) + np.float32(1.0)           # fully dense blocks
        enc = oracle.csb_encode(A, br, bc)
        nr, nc, ri, ci, val = _python_encode(A, br, bc)
        assert enc.nrows.tolist() == nr and enc.ncols.tolist() == nc
        assert enc.rowidx.tolist() == ri and enc.colidx.tolist() == ci
        assert enc.val.tolist() == [float(v) for v in val]
        assert np.array_equal(oracle.csb_decode(enc), A)


def test_signed_zero_nan_and_empty_block():
    A = np.zeros((4, 4), np.float32)
    A[0, 0] = -0.0
    A[1, 2] = np.nan
    enc = oracle.csb_encode(A, 2, 2)
    # block (0,0) holds only -0.0: empty.  block (0,1) holds the NaN at local (1,0).
    assert enc.nrows.tolist() == [0, 1, 0, 0] and enc.ncols.tolist() == [0, 1, 0, 0]
    assert enc.rowidx.tolist() == [1] and enc.colidx.tolist() == [0]
    assert np.isnan(enc.val[0]) and enc.nnz == 1
    D = oracle.csb_decode(enc)
    assert np.isnan(D[1, 2]) and np.count_nonzero(np.nan_to_num(D)) == 0
    assert not np.signbit(D[0, 0])                   # -0.0 comes back as +0.0


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
def test_generator_invariants_on_workload_shapes(name):
    cfg = csb_inputs.CONFIGS[name]
    wl = csb_inputs.make_rnn(cfg, T=2)
    for m in wl.W:
        enc = oracle.csb_encode(m.A, m.br, m.bc)
        # exact counts: kernel sizes add up to the mask popcount the generator reports
        assert enc.nnz == m.nnz == int(np.count_nonzero(m.A))
        assert np.array_equal(enc.nrows, m.r_b) and np.array_equal(enc.ncols, m.c_b)
        assert enc.rowidx.shape[0] == int(m.r_b.sum()) and enc.colidx.shape[0] == int(m.c_b.sum())
        # the decoded index sets are the generator's chosen sets, block by block
        for b in range(m.nbr * m.nbc):
            rows = np.nonzero(m.row_mask[b])[0]
            cols = np.nonzero(m.col_mask[b])[0]
            assert np.array_equal(enc.rowidx[enc.row_off[b]:enc.row_off[b + 1]], rows)
            assert np.array_equal(enc.colidx[enc.col_off[b]:enc.col_off[b + 1]], cols)
        # strictly ascending inside each block, below the (edge-aware) block size
        for b in range(m.nbr * m.nbc):
            bi, bj = divmod(b, m.nbc)
            h = min(m.br, m.rows - bi * m.br)
            w = min(m.bc, m.cols - bj * m.bc)
            ri = enc.rowidx[enc.row_off[b]:enc.row_off[b + 1]].astype(int)
            ci = enc.colidx[enc.col_off[b]:enc.col_off[b + 1]].astype(int)
            assert np.all(np.diff(ri) > 0) and (ri.size == 0 or ri[-1] < h)
            assert np.all(np.diff(ci) > 0) and (ci.size == 0 or ci[-1] < w)
        assert np.array_equal(oracle.csb_decode(enc).view(np.uint32), m.A.view(np.uint32))
        # achieved pruning rate within 1 % of the target (fraction read of Alg. 1's rate)
        rate = m.rows * m.cols / enc.nnz
        assert abs(rate - cfg.rate) / cfg.rate < 0.0105


def test_normalized_index_overhead_closed_form():
    """NIO = (#indices)/(#weights).  With r = c = B * rate**-0.5 kept per block it is
    2 / (B * rate**-0.5): about 20 % at block 32 and 10x (Sec. 6.2.1)."""
    cfg = csb_inputs.CONFIGS["cfg2"]
    m = csb_inputs.make_rnn(cfg, T=1).W[0]
    enc = oracle.csb_encode(m.A, m.br, m.bc)
    nio = (enc.rowidx.shape[0] + enc.colidx.shape[0]) / enc.nnz
    closed = 2.0 / (32 * 10 ** -0.5)
    assert abs(closed - 0.1976) < 1e-3
    # binomial kept counts make E[r+c]/E[rc] equal the closed form; edge blocks shift it a little
    assert abs(nio - closed) / closed < 0.05

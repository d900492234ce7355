"""16-bit weight formats (csb_set_value_format) through the C ABI: csb_spmv, csb_spmm and
csb_rnn_forward against the float64 oracle computed with the weights the ORACLE rounded
(numpy / bit arithmetic, pinned against torch).  The library gets the unrounded matrix and
rounds it itself, so a different rounding shows up here.  Sums are still binary32: same
tolerances as the 32-bit path (norm-wise 1e-5 plus the element-wise dot-product bound for the
products, 1e-4 absolute on h)."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbRnn, VAL_F16, VAL_BF16, CELL_LSTM, CELL_GRU
from helpers import rel_max_err

pytestmark = pytest.mark.gpu
FORMATS = [(VAL_F16, "f16"), (VAL_BF16, "bf16")]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def packed(A, br, bc, fmt, n_chunks=0, mode=0):
    M = CsbMatrix(A, br, bc)
    M.set_value_format(fmt)
    M.plan(n_chunks, mode)
    M.validate()
    M.upload()
    return M


def check_spmv(A, br, bc, x, fmt, name, n_chunks=0, mode=0, tag=""):
    say(f"[val16] spmv {tag} {name} shape={A.shape} block={br}x{bc} n_chunks={n_chunks} mode={mode}")
    Aq = oracle.round_weights(A, name)
    ref = oracle.matvec(Aq, x)
    scale = oracle.matvec_abs(Aq, x)
    M = packed(A, br, bc, fmt, n_chunks, mode)
    xd = torch.from_numpy(x).cuda()
    y = M.spmv(xd)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert rel_max_err(got, ref) <= 1e-5, rel_max_err(got, ref)
    k = np.count_nonzero(A, axis=1)
    assert np.all(np.abs(got - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * scale + 1e-30)
    assert torch.equal(y, M.spmv(xd))
    return M


@pytest.mark.parametrize("fmt,name", FORMATS)
@pytest.mark.parametrize("R,C,br,bc,rate", [(4, 8, 4, 4, 2.0), (1, 1, 1, 1, 1.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0),
                                            (130, 257, 32, 32, 5.0), (70, 300, 16, 64, 4.0), (513, 100, 256, 256, 2.0)])
def test_spmv_small_shapes(fmt, name, R, C, br, bc, rate):
    m = csb_inputs.small_matrix(R * 3 + C, R, C, br, bc, rate=rate)
    x = csb_inputs.make_vectors(R + C, C, 1)
    for n_chunks in (0, 1, 3):
        check_spmv(m.A, br, bc, x, fmt, name, n_chunks)
        check_spmv(m.A, br, bc, x, fmt, name, n_chunks, mode=2)


@pytest.mark.parametrize("fmt,name", FORMATS)
def test_spmv_long_wave_runs_and_many_chunks(fmt, name):
    """Wide rows in one chunk (more column steps per wavefront than one batch of value
    registers holds) and a matrix of many chunks and tiles."""
    m = csb_inputs.small_matrix(7, 64, 4000, 32, 32, rate=1.5)
    x = csb_inputs.make_vectors(3, 4000, 1)
    check_spmv(m.A, 32, 32, x, fmt, name, n_chunks=1, tag="one-chunk")
    m = csb_inputs.small_matrix(8, 2048, 1500, 32, 32, rate=8.0)
    x = csb_inputs.make_vectors(4, 1500, 1)
    check_spmv(m.A, 32, 32, x, fmt, name, tag="many-chunks")


@pytest.mark.parametrize("fmt,name", FORMATS)
def test_rounding_is_visible(fmt, name):
    """The 16-bit product differs from the 32-bit one by far more than the tolerance, so the
    parity above does test the rounded weights."""
    m = csb_inputs.small_matrix(9, 256, 256, 32, 32, rate=4.0)
    x = csb_inputs.make_vectors(5, 256, 1)
    ref32 = oracle.matvec(m.A, x)
    ref16 = oracle.matvec(oracle.round_weights(m.A, name), x)
    assert rel_max_err(ref16, ref32) > 3e-5


@pytest.mark.parametrize("fmt,name", FORMATS)
@pytest.mark.parametrize("R,C,br,bc,B", [(37, 53, 8, 8, 1), (200, 150, 16, 16, 5), (130, 257, 32, 32, 17), (300, 200, 64, 64, 40),
                                         (1024, 700, 32, 32, 64),
                                         # 256 row tiles and more, 64 right-hand sides per workgroup: the kernel that keeps
                                         # its results in registers (one and two 16-row parts per tile), 16-bit values unpacked
                                         (4200, 300, 16, 16, 64), (8300, 200, 32, 32, 128), (8300, 90, 32, 32, 52)])
def test_spmm(fmt, name, R, C, br, bc, B):
    say(f"[val16] spmm {name} {R}x{C} block {br}x{bc} batch {B}")
    m = csb_inputs.small_matrix(R + C + B, R, C, br, bc, rate=4.0)
    X = csb_inputs.make_vectors(B, C, B).reshape(C, B)
    Aq = oracle.round_weights(m.A, name)
    ref = oracle.matmat(Aq, X)
    M = packed(m.A, br, bc, fmt)
    Y = M.spmm(torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    got = Y.cpu().numpy().astype(np.float64)
    assert rel_max_err(got, ref) <= 1e-5, rel_max_err(got, ref)
    absr = oracle.matmat(np.abs(Aq), np.abs(X))
    k = np.count_nonzero(m.A, axis=1)[:, None]
    assert np.all(np.abs(got - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * absr + 1e-30)


@pytest.mark.parametrize("fmt,name", FORMATS)
@pytest.mark.parametrize("cell,L,I,H,T,B,block", [(csb_inputs.LSTM, 2, 12, 16, 9, 1, 8), (csb_inputs.GRU, 1, 40, 100, 12, 1, 32),
                                                  (csb_inputs.LSTM, 1, 64, 128, 16, 1, 16), (csb_inputs.GRU, 2, 30, 96, 7, 19, 16),
                                                  (csb_inputs.LSTM, 2, 33, 300, 9, 5, 32)])
def test_rnn(fmt, name, cell, L, I, H, T, B, block):
    cfg = csb_inputs.RnnConfig("t", cell, L, I, H, block, 3.0, "binomial", 0.3, B, T, 90 + L + I)
    wl = csb_inputs.make_rnn(cfg)
    Wq = [oracle.round_weights(m.A, name) for m in wl.W]
    rseq, rhT, rcT = oracle.rnn_forward(cell, Wq, wl.bias, wl.x, I, H)
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    xd = torch.from_numpy(wl.x).cuda()
    for resident in (False, True):        # (a batch with the resident layout alone runs as instances of that kernel)
        say(f"[val16] rnn {name} cell={cell} L={L} I={I} H={H} T={T} B={B} resident={resident}")
        Ws = []
        for m in wl.W:
            M = CsbMatrix(m.A, m.br, m.bc)
            M.set_value_format(fmt)                    # before the handle is created over it
            Ws.append(M)
        rnn = CsbRnn(CELL_LSTM if cell == csb_inputs.LSTM else CELL_GRU, I, H, Ws, bias)
        if resident:
            rnn.upload()
        else:
            for M in Ws:
                assert M.value_format() == fmt
                M.validate()
                M.upload()
        hseq, hT, cT = rnn.forward(xd)
        torch.cuda.synchronize()
        e = max(float(np.max(np.abs(hseq.cpu().numpy() - rseq))), float(np.max(np.abs(hT.cpu().numpy() - rhT))))
        if cell == csb_inputs.LSTM:
            e = max(e, float(np.max(np.abs(cT.cpu().numpy() - rcT))))
        say(f"[val16] rnn err {e:.3g}")
        assert e <= 1e-4


@pytest.mark.parametrize("fmt,name", FORMATS)
@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
def test_rnn_batched_many_row_tiles(fmt, name, cell):
    """Two layers of 1024 units in blocks of 16 at batch 64: 256 row tiles per matrix, so the
    layers' products share launches of the kernel that keeps its results in registers, here
    with 16-bit kernel values (one product per launch and two, one and two input sources)."""
    cfg = csb_inputs.RnnConfig("t", cell, 2, 48, 1024, 16, 12.0, "binomial", 0.05, 64, 3, 33)
    wl = csb_inputs.make_rnn(cfg)
    Wq = [oracle.round_weights(m.A, name) for m in wl.W]
    rseq, rhT, rcT = oracle.rnn_forward(cell, Wq, wl.bias, wl.x, cfg.input, cfg.hidden)
    Ws = []
    for m in wl.W:
        M = CsbMatrix(m.A, m.br, m.bc)
        M.set_value_format(fmt)
        Ws.append(M)
    rnn = CsbRnn(CELL_LSTM if cell == csb_inputs.LSTM else CELL_GRU, cfg.input, cfg.hidden, Ws,
                 [torch.from_numpy(b).cuda() for b in wl.bias])
    for M in Ws:
        M.validate()
        M.upload()
    say(f"[val16] batched rnn {name} cell={cell} 2 x 1024, block 16, batch 64")
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda())
    torch.cuda.synchronize()
    e = max(float(np.max(np.abs(hseq.cpu().numpy() - rseq))), float(np.max(np.abs(hT.cpu().numpy() - rhT))))
    if cell == csb_inputs.LSTM:
        e = max(e, float(np.max(np.abs(cT.cpu().numpy() - rcT))))
    assert e <= 1e-4, e


@pytest.mark.parametrize("fmt,name", FORMATS)
def test_spmv_full_size_stress(fmt, name):
    """The 8192 x 8192 heavy-tailed matrix bench.py times, in its launch configuration (default
    plan), every output row against the oracle."""
    m = csb_inputs.make_mat(csb_inputs.CONFIGS["cfg5"])
    x = csb_inputs.make_vectors(5, m.cols, 1)
    check_spmv(m.A, m.br, m.bc, x, fmt, name, tag="cfg5")


BF_SHAPES = [(37, 53, 8, 8, 4, 4.0), (4, 8, 4, 4, 8, 2.0), (1, 1, 1, 1, 4, 1.0), (200, 150, 16, 16, 20, 4.0), (130, 257, 32, 32, 64, 3.0),
             (300, 200, 64, 64, 68, 4.0), (70, 300, 16, 64, 128, 1.0), (1024, 700, 32, 32, 200, 6.0), (513, 100, 64, 32, 12, 2.0),
             (90, 90, 3, 5, 16, 1.5), (64, 2048, 32, 32, 32, 1.0)]


def run16(M, name, Xq_dev32):
    """csb_spmm_bfloat / csb_spmm_half on float32 values that the format holds exactly."""
    if name == "bf16":
        return M.spmm_bfloat(Xq_dev32.to(torch.bfloat16))
    return M.spmm_half(Xq_dev32.to(torch.float16))


@pytest.mark.parametrize("fmt,name", FORMATS)
@pytest.mark.parametrize("R,C,br,bc,B,rate", BF_SHAPES)
def test_spmm_bfloat(fmt, name, R, C, br, bc, B, rate):
    """csb_spmm_bfloat / csb_spmm_half: 16-bit kernel values times 16-bit right-hand sides on the
    16-bit matrix cores, accumulated in binary32.  Against the float64 product of the operands
    as the ORACLE rounds them (the products of two such numbers are exact in binary32, so the
    float32 dot-product bound of csb_spmm holds), blocks with more than 16 and more than 32
    columns, odd column counts, batches that are not a multiple of 64, a strided X."""
    say(f"[val16] spmm 16-bit operands {name} {R}x{C} block {br}x{bc} batch {B} rate {rate}")
    m = csb_inputs.small_matrix(R + C + B, R, C, br, bc, rate=rate)
    X = csb_inputs.make_vectors(B + 1, C, B).reshape(C, B)
    Aq = oracle.round_weights(m.A, name)
    Xq = oracle.round_weights(X, name).astype(np.float32)
    ref = oracle.matmat(Aq, Xq)
    M = packed(m.A, br, bc, fmt)
    dt = torch.bfloat16 if name == "bf16" else torch.float16
    buf = torch.zeros((C, B + 8), dtype=dt, device="cuda")
    buf[:, :B] = torch.from_numpy(Xq).cuda().to(dt)                      # exact: the values are in the format already
    assert torch.equal(buf[:, :B].float().cpu(), torch.from_numpy(Xq))
    call = M.spmm_bfloat if name == "bf16" else M.spmm_half
    Y = call(buf[:, :B])
    torch.cuda.synchronize()
    got = Y.cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape and np.all(np.isfinite(got))
    absr = oracle.matmat(np.abs(Aq), np.abs(Xq))
    k = np.count_nonzero(m.A, axis=1)[:, None]
    assert np.all(np.abs(got - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * absr + 1e-30)
    assert torch.equal(Y, call(buf[:, :B]))                              # run to run the same bits


def test_spmm_bfloat_refusals():
    from paper_2005_05758_amd import CsbError, VAL_F32
    m = csb_inputs.small_matrix(3, 64, 64, 16, 16, rate=2.0)
    X = torch.zeros((64, 8), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(CsbError):                      # the matrix stores binary32 / binary16 values
        packed(m.A, 16, 16, VAL_F32).spmm_bfloat(X)
    with pytest.raises(CsbError):
        packed(m.A, 16, 16, VAL_F16).spmm_bfloat(X)
    M = packed(m.A, 16, 16, VAL_BF16)
    with pytest.raises(CsbError):                      # batch not a multiple of 4
        M.spmm_bfloat(torch.zeros((64, 6), dtype=torch.bfloat16, device="cuda"))
    with pytest.raises(CsbError):                      # rows of X not 8-byte aligned
        M.spmm_bfloat(torch.zeros((64, 10), dtype=torch.bfloat16, device="cuda")[:, :8])
    with pytest.raises(CsbError):                      # a bfloat16 matrix is not a binary16 one
        M.spmm_half(torch.zeros((64, 8), dtype=torch.float16, device="cuda"))


@pytest.mark.parametrize("fmt,name", FORMATS)
def test_spmm_16bit_values_full_size(fmt, name):
    """csb_spmm with 16-bit kernel values and float32 right-hand sides on the 8192 x 8192
    heavy-tailed matrix at batch 128, the launch bench.py times: sampled rows against the oracle."""
    m = csb_inputs.make_mat(csb_inputs.CONFIGS["cfg5"])
    B = 128
    X = csb_inputs.make_vectors(9, m.cols, B).reshape(m.cols, B)
    M = packed(m.A, m.br, m.bc, fmt)
    Y = M.spmm(torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, 64), np.random.default_rng(1).integers(0, m.rows, 400), [m.rows - 1]]))
    Aq = oracle.round_weights(m.A[rows], name)
    ref = oracle.matmat(Aq, X)
    got = Y.cpu().numpy()[rows].astype(np.float64)
    absr = oracle.matmat(np.abs(Aq), np.abs(X))
    k = np.count_nonzero(Aq, axis=1)[:, None]
    assert np.all(np.abs(got - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * absr + 1e-30)


@pytest.mark.parametrize("fmt,name", FORMATS)
def test_spmm_bfloat_full_size(fmt, name):
    """The 8192 x 8192 heavy-tailed matrix at batch 128, the launch bench.py times: sampled rows
    against the oracle."""
    m = csb_inputs.make_mat(csb_inputs.CONFIGS["cfg5"])
    B = 128
    X = csb_inputs.make_vectors(9, m.cols, B).reshape(m.cols, B)
    Xq = oracle.round_weights(X, name).astype(np.float32)
    M = packed(m.A, m.br, m.bc, fmt)
    Y = run16(M, name, torch.from_numpy(Xq).cuda())
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([np.arange(0, 64), np.random.default_rng(0).integers(0, m.rows, 400), [m.rows - 1]]))
    Aq = oracle.round_weights(m.A[rows], name)
    ref = oracle.matmat(Aq, Xq)
    got = Y.cpu().numpy()[rows].astype(np.float64)
    absr = oracle.matmat(np.abs(Aq), np.abs(Xq))
    k = np.count_nonzero(Aq, axis=1)[:, None]
    assert np.all(np.abs(got - ref) <= 2.0 * np.maximum(k, 1) * 2.0 ** -24 * absr + 1e-30)

"""Parity of csb_spmv (HIP, through the C ABI) against the oracle's float64 product on the
decompressed matrix.  Tolerances (float32 path):
  - norm-wise: max|y - y_ref| / max|y_ref| <= 1e-5
  - element-wise: |y_i - y_ref_i| <= 2 k_i 2^-24 sum_j |a_ij x_j|, k_i = kept entries of row
    i (the textbook bound for a float32 dot product in any summation order)."""
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


def check_spmv(A, br, bc, x, n_chunks=0, tag="", mode=0):
    say(f"[spmv] {tag} shape={A.shape} block={br}x{bc} n_chunks={n_chunks} mode={mode}")
    enc = oracle.csb_encode(A, br, bc)
    D = oracle.csb_decode(enc)                      # oracle works on the decompressed matrix
    ref = oracle.matvec(D, x)
    scale = oracle.matvec_abs(D, x)
    M = CsbMatrix(A, br, bc)
    M.plan(n_chunks, mode)
    M.validate()
    M.upload()
    xd = torch.from_numpy(x).cuda()
    y = M.spmv(xd)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got))
    assert rel_max_err(got, ref) <= 1e-5, rel_max_err(got, ref)
    k = np.count_nonzero(D, axis=1)
    bound = 2.0 * np.maximum(k, 1) * 2.0 ** -24 * scale + 1e-30
    assert np.all(np.abs(got - ref) <= bound)
    # run-to-run bitwise reproducibility
    y2 = M.spmv(xd)
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    return M, got


@pytest.mark.parametrize("R,C,br,bc,rate", [
    (4, 8, 4, 4, 2.0), (1, 1, 1, 1, 1.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0),
    (130, 257, 32, 32, 5.0), (96, 96, 32, 16, 4.0), (70, 300, 16, 64, 4.0), (300, 40, 128, 8, 3.0),
    (513, 100, 256, 256, 2.0), (64, 64, 64, 64, 1.0)])
def test_spmv_small_shapes(R, C, br, bc, rate):
    m = csb_inputs.small_matrix(R * 3 + C, R, C, br, bc, rate=rate)
    x = csb_inputs.make_vectors(R + C, C, 1)
    for n_chunks in (0, 1, 3, 7):
        check_spmv(m.A, br, bc, x, n_chunks, tag="small")
        check_spmv(m.A, br, bc, x, n_chunks, tag="small", mode=2)     # equal split with merges


def test_spmv_degenerate_matrices():
    x = csb_inputs.make_vectors(1, 48, 1)
    Z = np.zeros((40, 48), np.float32)
    check_spmv(Z, 16, 16, x, tag="all-zero")                       # every tile empty
    E = Z.copy()
    E[17, 5] = 2.0                                                 # a single survivor
    _, got = check_spmv(E, 16, 16, x, tag="single")
    assert got[17] == 2.0 * float(x[5]) and np.count_nonzero(got) == 1
    Dn = csb_inputs.small_matrix(2, 40, 48, 16, 16, rate=1.0).A    # fully dense blocks
    check_spmv(Dn, 16, 16, x, tag="dense")
    I = np.eye(48, dtype=np.float32)
    _, got = check_spmv(I, 16, 16, x, tag="identity")
    assert np.array_equal(got, x.astype(np.float64))
    P = np.zeros((48, 48), np.float32)
    perm = np.random.default_rng(0).permutation(48)
    P[np.arange(48), perm] = 1.0
    _, got = check_spmv(P, 16, 16, x, n_chunks=5, tag="permutation")
    assert np.array_equal(got, x[perm].astype(np.float64))


def test_spmv_widest_input_and_long_wavefront_runs():
    """16383 columns: the widest input vector the 16-bit byte offsets address (odd width, so the
    element-wise staging path runs); one chunk for a matrix with far more than 32 steps per
    wavefront (the value registers are refilled batch by batch); non-finite inputs stay in the
    rows that use them (padded steps multiply zeros with a zero word, not with the input)."""
    m = csb_inputs.small_matrix(22, 70, 16383, 32, 64, rate=6.0)
    x = csb_inputs.make_vectors(5, 16383, 1)
    check_spmv(m.A, 32, 64, x, tag="max-cols")
    check_spmv(m.A, 32, 64, x, n_chunks=3, tag="max-cols", mode=2)
    m = csb_inputs.small_matrix(23, 256, 2048, 64, 64, rate=2.0)
    x = csb_inputs.make_vectors(6, 2048, 1)
    check_spmv(m.A, 64, 64, x, n_chunks=1, tag="one-chunk")
    # a column nobody uses carries Inf: no row may see it (77 lies inside a block column, 64 is the
    # first column of one: padded steps name a column their block keeps, never a fixed position)
    for dead in (77, 64, 0):
        A = csb_inputs.small_matrix(24, 96, 130, 16, 16, rate=3.0).A.copy()
        A[:, dead] = 0.0
        x = csb_inputs.make_vectors(7, 130, 1).copy()
        x[dead] = np.inf
        for mode in (0, 2):
            M = CsbMatrix(A, 16, 16)
            M.plan(0, mode)
            M.upload()
            y = M.spmv(torch.from_numpy(x.reshape(-1)).cuda())
            torch.cuda.synchronize()
            assert np.all(np.isfinite(y.cpu().numpy())), (dead, mode)


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
def test_spmv_rnn_matrices(name):
    cfg = csb_inputs.CONFIGS[name]
    m = csb_inputs.make_rnn(cfg, T=1).W[0]
    x = csb_inputs.make_vectors(3, m.cols, 1)
    for n_chunks in (0, 16, 100):
        check_spmv(m.A, m.br, m.bc, x, n_chunks, tag=name)
        check_spmv(m.A, m.br, m.bc, x, n_chunks, tag=name, mode=2)


def test_spmv_result_independent_of_partition():
    m = csb_inputs.small_matrix(9, 512, 640, 32, 32, rate=8.0, law="beta")
    x = csb_inputs.make_vectors(9, 640, 1)
    outs = [check_spmv(m.A, 32, 32, x, n, tag="partition", mode=md)[1] for n in (1, 2, 13, 64) for md in (1, 2)]
    for o in outs[1:]:
        assert rel_max_err(o, outs[0]) <= 1e-5


@pytest.mark.parametrize("mode", [0, 2])
@pytest.mark.parametrize("name", ["cfg5", "cfg5_diag"])
def test_spmv_full_size_stress(name, mode):
    """8192 x 8192, heavy-tailed block sizes, in the launch configurations the benchmark
    times: the default plan (row-owned layout) and the tile-based equal split (mode 2).  In
    both the largest wavefront's work must stay within 10 % of the mean (work as the planner
    counts it: column steps plus the fixed cost of every piece).  The oracle handles the full
    product in a few seconds."""
    m = csb_inputs.make_mat(csb_inputs.CONFIGS[name])
    x = csb_inputs.make_vectors(5, m.cols, 1)
    say(f"[spmv] {name} nnz={m.nnz}")
    ref = oracle.matvec(m.A, x)                    # m.A == decode(encode(m.A)) (pinned on the CPU)
    scale = oracle.matvec_abs(m.A, x)
    M = CsbMatrix(m.A, m.br, m.bc)
    st = M.plan(0, mode)
    say(f"[spmv] plan {st}")
    assert st["row_owned"] == (1 if mode == 0 else 0)
    assert st["work_max"] / st["work_mean"] <= 1.10
    M.validate()
    M.upload()
    xd = torch.from_numpy(x).cuda()
    y = M.spmv(xd)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    assert rel_max_err(got, ref) <= 1e-5
    k = np.count_nonzero(m.A, axis=1)
    assert np.all(np.abs(got - ref) <= 2.0 * k * 2.0 ** -24 * scale + 1e-30)
    for _ in range(3):
        assert torch.equal(M.spmv(xd), y)


@pytest.mark.parametrize("R,C,br,bc,rate", [
    (4, 8, 4, 4, 2.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0), (130, 257, 32, 32, 5.0),
    (70, 300, 16, 64, 4.0), (300, 40, 128, 8, 3.0), (513, 100, 256, 256, 2.0), (1030, 96, 32, 32, 3.0)])
def test_spmv_row_owned_plans(R, C, br, bc, rate):
    """csb_plan_rows with workgroup and round counts of the caller's choosing (several rounds make
    a wavefront request its next segment while it multiplies the current one): same bar as the
    default plan, and the same bits whatever the partition of the rows' slots over rounds."""
    m = csb_inputs.small_matrix(R * 3 + C, R, C, br, bc, rate=rate)
    x = csb_inputs.make_vectors(R + C, C, 1)
    ref = oracle.matvec(oracle.csb_decode(oracle.csb_encode(m.A, br, bc)), x)
    xd = torch.from_numpy(x).cuda()
    for n_wg in (0, 1, 3):
        for rounds in (0, 2, 5):
            say(f"[spmv] row-owned shape={m.A.shape} n_wg={n_wg} rounds>={rounds}")
            M = CsbMatrix(m.A, br, bc)
            st = M.plan_rows(n_wg, rounds)
            assert st["row_owned"] == 1
            M.validate()
            M.upload()
            y = M.spmv(xd)
            torch.cuda.synchronize()
            assert rel_max_err(y.cpu().numpy().astype(np.float64), ref) <= 1e-5
            assert torch.equal(M.spmv(xd), y) and torch.equal(M.spmv_static(xd), y)


@pytest.mark.parametrize("shift", [1, 2, 3])
def test_spmv_input_vector_at_any_four_byte_address(shift):
    """An input vector that starts 4, 8 or 12 bytes past a 16-byte boundary (the kernel then
    stages it 4 bytes per lane), default plan and a plan with several rounds: the same bits as
    with the aligned vector."""
    m = csb_inputs.small_matrix(31, 300, 512, 32, 32, rate=4.0)
    x = csb_inputs.make_vectors(8, 512, 1).reshape(-1)
    buf = torch.zeros(512 + 8, dtype=torch.float32, device="cuda")
    assert buf.data_ptr() % 16 == 0
    xs = buf[shift:shift + 512]
    xs.copy_(torch.from_numpy(x))
    xa = torch.from_numpy(x).cuda()
    ref = oracle.matvec(oracle.csb_decode(oracle.csb_encode(m.A, 32, 32)), x)
    for rounds in (0, 3):
        say(f"[spmv] x at byte offset {4 * shift}, rounds>={rounds}")
        M = CsbMatrix(m.A, 32, 32)
        M.plan_rows(0, rounds)
        M.upload()
        ya = M.spmv(xa)
        ys = M.spmv(xs)
        torch.cuda.synchronize()
        assert torch.equal(ya, ys)
        assert rel_max_err(ys.cpu().numpy().astype(np.float64), ref) <= 1e-5


def test_spmv_replays_from_a_captured_graph():
    """csb_spmv on a row-owned plan is one kernel launch: captured into a HIP graph (two products
    in a row, the second reading what the first wrote) and replayed three times with new inputs
    in the captured buffer and eager launches in between."""
    rng = np.random.default_rng(12)
    m = csb_inputs.make_mat(csb_inputs.MatConfig("g", 320, 320, 16, 4.0, "binomial", 0.05, 3))
    D = oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)).astype(np.float64)
    M = CsbMatrix(m.A, m.br, m.bc)
    assert M.plan()["row_owned"] == 1
    M.upload()
    xs = torch.zeros(320, dtype=torch.float32, device="cuda")
    y1 = torch.empty(320, dtype=torch.float32, device="cuda")
    y2 = torch.empty(320, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        M.spmv(xs, y1)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        M.spmv(xs, y1)
        M.spmv(y1, y2)
    torch.cuda.synchronize()
    for rep in range(3):
        x = rng.uniform(-1, 1, 320).astype(np.float32)
        xs.copy_(torch.from_numpy(x))
        graph.replay()
        torch.cuda.synchronize()
        g1, g2 = y1.clone(), y2.clone()
        e1 = M.spmv(xs)
        e2 = M.spmv(e1)
        torch.cuda.synchronize()
        assert torch.equal(g1, e1) and torch.equal(g2, e2)
        ref = D @ x.astype(np.float64)
        assert rel_max_err(g1.cpu().numpy().astype(np.float64), ref) <= 1e-5


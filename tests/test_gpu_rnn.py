"""Parity of csb_rnn_forward (HIP, through the C ABI) against the oracle's float64 LSTM/GRU
on the decompressed masked matrix: max |h_T - ref| <= 1e-4 per layer (also c_T and every
h_t of the sequence)."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbRnn

pytestmark = pytest.mark.gpu
TOL = 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def build_rnn(wl, resident):
    """resident=True: upload the on-chip layout (one launch for the whole sequence, batch 1);
    resident=False: upload the matrices only (one mat-vec launch per step and layer)."""
    cfg = wl.cfg
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, bias)
    if resident:
        assert rnn.stats()["resident"] == 1
        rnn.upload()
    else:
        for w in Ws:
            w.validate()
            w.upload()
    return rnn


def run_case(wl, h0=None, c0=None, tag="", resident=None):
    cfg = wl.cfg
    T, B, _ = wl.x.shape
    if resident is None:                      # both device paths where both apply
        out = run_case(wl, h0, c0, tag, resident=False)
        if B == 1:
            out = run_case(wl, h0, c0, tag, resident=True)
        return out
    say(f"[rnn] {tag} cell={cfg.cell} L={cfg.n_layers} I={cfg.input} H={cfg.hidden} T={T} B={B} resident={resident}")
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden, h0=h0, c0=c0)
    rnn = build_rnn(wl, resident)
    xd = torch.from_numpy(wl.x).cuda()
    h0d = None if h0 is None else torch.from_numpy(h0.astype(np.float32)).cuda()
    c0d = None if c0 is None else torch.from_numpy(c0.astype(np.float32)).cuda()
    hseq, hT, cT = rnn.forward(xd, h0d, c0d)
    torch.cuda.synchronize()
    e_seq = float(np.max(np.abs(hseq.cpu().numpy() - rseq))) if T else 0.0
    e_h = float(np.max(np.abs(hT.cpu().numpy() - rhT)))
    say(f"[rnn] {tag} err hseq={e_seq:.3g} hT={e_h:.3g}")
    assert e_seq <= TOL and e_h <= TOL
    if cfg.cell == csb_inputs.LSTM:
        assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL
    return rnn, (hseq, hT, cT)


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
@pytest.mark.parametrize("L,I,H,T,B,block", [(1, 5, 7, 6, 1, 4), (2, 12, 16, 9, 3, 8), (1, 40, 100, 12, 2, 32),
                                            (3, 8, 8, 4, 2, 8), (1, 33, 50, 5, 1, 16), (2, 30, 300, 7, 1, 32),
                                            (3, 16, 64, 20, 1, 16)])
def test_rnn_small(cell, L, I, H, T, B, block):
    cfg = csb_inputs.RnnConfig("t", cell, L, I, H, block, 3.0, "binomial", 0.3, B, T, 20 + L + I)
    wl = csb_inputs.make_rnn(cfg)
    rng = np.random.default_rng(1)
    h0 = rng.uniform(-0.5, 0.5, (L, B, H)).astype(np.float32).astype(np.float64)
    c0 = rng.uniform(-0.5, 0.5, (L, B, H)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, c0 if cell == csb_inputs.LSTM else None, tag="small")
    run_case(wl, tag="small-zero-state")


@pytest.mark.parametrize("cell,L", [(csb_inputs.GRU, 1), (csb_inputs.GRU, 3), (csb_inputs.LIGRU, 2)])
def test_rnn_cells_computed_where_they_are_consumed(cell, L):
    """GRU and Li-GRU steps on plans the caller makes (plain row ranges; the GRU's keep the row
    split of its step): the launches that consume a cell's output compute it on their way in."""
    cfg = csb_inputs.RnnConfig("t", cell, L, 24, 96, 16, 3.0, "binomial", 0.3, 1, 7, 150 + L)
    wl = csb_inputs.make_rnn(cfg)
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias])
    for w in Ws:
        assert w.plan_stats()["row_owned"] == 2
        assert w.plan()["row_owned"] == 1                      # (csb_plan keeps a GRU matrix's row split)
        w.validate()
        w.upload()
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda())
    torch.cuda.synchronize()
    assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= TOL
    assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL


@pytest.mark.parametrize("L", [1, 2])
@pytest.mark.parametrize("n_wg,rounds", [(0, 3), (2, 2), (5, 4), (1, 1)])
def test_rnn_streaming_on_row_owned_plans_of_the_callers_choosing(L, n_wg, rounds):
    """The per-step launches of the streaming path on matrices re-planned with csb_plan_rows:
    several rounds per wavefront (the kernels compiled for that case, one product per launch and,
    with two layers, two products of a diagonal in one launch), few and many workgroups."""
    cfg = csb_inputs.RnnConfig("t", csb_inputs.LSTM, L, 24, 96, 16, 3.0, "binomial", 0.3, 1, 7, 50 + L)
    wl = csb_inputs.make_rnn(cfg)
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias])
    for w in Ws:
        st = w.plan_rows(n_wg, rounds)
        say(f"[rnn] re-planned: {st['n_chunks']} workgroups, {st['rounds']} rounds")
        assert st["row_owned"] == 1 and st["rounds"] >= rounds
        w.validate()
        w.upload()
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda())
    torch.cuda.synchronize()
    assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= TOL
    assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL
    assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL


@pytest.mark.parametrize("cell,L,I,H,block,rate,T", [
    (csb_inputs.LSTM, 2, 24, 96, 16, 3.0, 7), (csb_inputs.GRU, 3, 33, 100, 32, 3.0, 6), (csb_inputs.LIGRU, 2, 7, 40, 8, 2.0, 9),
    (csb_inputs.LSTM, 5, 16, 64, 16, 4.0, 5),            # more layers on a diagonal than one launch takes
    (csb_inputs.LSTM, 1, 5, 2048, 64, 2.0, 3)])         # a wide layer: wavefronts with several rounds
def test_rnn_streaming_on_plans_whose_workgroups_own_whole_units(cell, L, I, H, block, rate, T):
    """Stacked (and very wide) layers: csb_rnn_create lays the matrices out so that a workgroup owns
    units with all their gate rows, and a step of the streaming path is one launch that finishes
    its cells.  Without biases and without an output sequence as well; and csb_spmv on such a
    matrix (it reads the tile sections) still gives the plain product."""
    cfg = csb_inputs.RnnConfig("t", cell, L, I, H, block, rate, "binomial", 0.3, 1, T, 90 + L)
    wl = csb_inputs.make_rnn(cfg)
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    rng = np.random.default_rng(3)
    h0 = rng.uniform(-0.5, 0.5, (L, 1, H)).astype(np.float32).astype(np.float64)
    c0 = rng.uniform(-0.5, 0.5, (L, 1, H)).astype(np.float32).astype(np.float64) if cell == csb_inputs.LSTM else None
    for with_bias in (True, False):
        bias = wl.bias if with_bias else [np.zeros_like(b) for b in wl.bias]
        rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, bias, wl.x, cfg.input, cfg.hidden, h0=h0, c0=c0)
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias] if with_bias else None)
        for w in Ws:
            st = w.plan_stats()
            say(f"[rnn] whole units: {st['n_chunks']} workgroups, {st['rounds']} rounds, bias {with_bias}")
            assert st["row_owned"] == 2
            w.upload()
        xd = torch.from_numpy(wl.x).cuda()
        h0d = torch.from_numpy(h0.astype(np.float32)).cuda()
        c0d = None if c0 is None else torch.from_numpy(c0.astype(np.float32)).cuda()
        hseq, hT, cT = rnn.forward(xd, h0d, c0d, want_hseq=with_bias)
        torch.cuda.synchronize()
        if with_bias:
            assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= TOL
        assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL
        if cell == csb_inputs.LSTM:
            assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL
        if cell != csb_inputs.GRU:                          # (a GRU's matrix is laid out for its step: rows relabelled)
            x = rng.uniform(-1, 1, W[0].shape[1]).astype(np.float32)
            y = Ws[0].spmv(torch.from_numpy(x).cuda()).cpu().numpy()
            ref = W[0].astype(np.float64) @ x.astype(np.float64)
            # the float32 dot-product bound: k terms in any order, 2 k 2^-24 sum |a_ij x_j|
            k = np.count_nonzero(W[0], axis=1)
            bound = 2.0 * np.maximum(k, 1) * 2.0 ** -24 * (np.abs(W[0]).astype(np.float64) @ np.abs(x).astype(np.float64)) + 1e-30
            assert np.all(np.abs(y - ref) <= bound)
        del rnn


@pytest.mark.parametrize("cell,L,B", [(csb_inputs.LSTM, 1, 1), (csb_inputs.LSTM, 2, 1), (csb_inputs.GRU, 1, 1), (csb_inputs.LIGRU, 3, 1),
                                      (csb_inputs.LSTM, 2, 8), (csb_inputs.GRU, 1, 5)])
def test_rnn_streaming_forward_replays_from_a_captured_graph(cell, L, B):
    """The streaming path on row-owned plans (and the batched path) is kernel launches only, so a
    caller may capture csb_rnn_forward into a HIP graph and replay it: three replays with new
    inputs written into the captured buffers in between, eager work and synchronisation between
    them, each compared with the oracle and with the eager call."""
    cfg = csb_inputs.RnnConfig("t", cell, L, 20, 72, 16, 3.0, "binomial", 0.3, B, 9, 130 + L)
    wl = csb_inputs.make_rnn(cfg)
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias])
    for w in Ws:
        w.upload()
    rng = np.random.default_rng(8)
    xs = torch.from_numpy(wl.x).cuda()                       # the captured input buffer
    h0s = torch.zeros((L, B, cfg.hidden), dtype=torch.float32, device="cuda")
    c0s = torch.zeros_like(h0s) if cell == csb_inputs.LSTM else None
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        rnn.forward(xs, h0s, c0s)                            # (sizes the workspace outside the capture)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        out = rnn.forward(xs, h0s, c0s)
    torch.cuda.synchronize()
    for rep in range(3):
        x = rng.uniform(-1, 1, wl.x.shape).astype(np.float32)
        h0 = rng.uniform(-0.5, 0.5, (L, B, cfg.hidden)).astype(np.float32)
        c0 = rng.uniform(-0.5, 0.5, (L, B, cfg.hidden)).astype(np.float32)
        xs.copy_(torch.from_numpy(x)); h0s.copy_(torch.from_numpy(h0))
        if c0s is not None:
            c0s.copy_(torch.from_numpy(c0))
        rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, x, cfg.input, cfg.hidden, h0=h0.astype(np.float64),
                                            c0=c0.astype(np.float64) if c0s is not None else None)
        graph.replay()
        torch.cuda.synchronize()
        hseq, hT, cT = (o.clone() if o is not None else None for o in out)
        eager = rnn.forward(xs, h0s, c0s)                     # the program's own eager work between the replays
        torch.cuda.synchronize()
        say(f"[rnn] graph replay {rep}: err {float(np.max(np.abs(hseq.cpu().numpy() - rseq))):.3g}")
        assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= TOL
        assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL
        assert torch.equal(hseq, eager[0]) and torch.equal(hT, eager[1])
        if c0s is not None:
            assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL and torch.equal(cT, eager[2])


@pytest.mark.parametrize("cell,L,record", [(csb_inputs.LSTM, 1, True), (csb_inputs.GRU, 2, True), (csb_inputs.LIGRU, 2, True),
                                           (csb_inputs.LSTM, 2, False)])
def test_rnn_streaming_calls_that_repeat_their_arguments(cell, L, record, monkeypatch):
    """A streaming call that repeats its predecessor's arguments records its launches, later ones
    replay them (csb_rnn_forward keeps the graph): six calls on the same buffers with new contents
    each time, a call with other arguments (a shorter sequence) in the middle, a fresh upload of a
    matrix near the end -- every result against the oracle."""
    if not record:
        monkeypatch.setenv("CSB_RNN_GRAPH", "0")               # (read when the handle is created: every call enqueues its launches)
    cfg = csb_inputs.RnnConfig("t", cell, L, 20, 72, 16, 3.0, "binomial", 0.3, 1, 8, 140 + L)
    wl = csb_inputs.make_rnn(cfg)
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias])
    for w in Ws:
        w.upload()
    rng = np.random.default_rng(9)
    xs = torch.zeros((8, 1, 20), dtype=torch.float32, device="cuda")
    h0s = torch.zeros((L, 1, 72), dtype=torch.float32, device="cuda")
    c0s = torch.zeros_like(h0s) if cell == csb_inputs.LSTM else None
    hseq = torch.empty((8, 1, 72), dtype=torch.float32, device="cuda")
    hT = torch.empty((L, 1, 72), dtype=torch.float32, device="cuda")
    cT = torch.empty((L, 1, 72), dtype=torch.float32, device="cuda") if cell == csb_inputs.LSTM else None
    for call in range(7):
        T = 5 if call == 3 else 8
        if call == 5:
            Ws[0].upload()                                      # the same plan into a new buffer
        x = rng.uniform(-1, 1, (8, 1, 20)).astype(np.float32)
        h0 = rng.uniform(-0.5, 0.5, (L, 1, 72)).astype(np.float32)
        c0 = rng.uniform(-0.5, 0.5, (L, 1, 72)).astype(np.float32)
        xs.copy_(torch.from_numpy(x)); h0s.copy_(torch.from_numpy(h0))
        if c0s is not None:
            c0s.copy_(torch.from_numpy(c0))
        rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, x[:T], cfg.input, cfg.hidden, h0=h0.astype(np.float64),
                                            c0=c0.astype(np.float64) if c0s is not None else None)
        rnn.forward_into(xs[:T], h0s, c0s, hseq[:T], hT, cT)
        torch.cuda.synchronize()
        say(f"[rnn] repeated call {call} (T={T}): err {float(np.max(np.abs(hseq[:T].cpu().numpy() - rseq))):.3g}")
        assert float(np.max(np.abs(hseq[:T].cpu().numpy() - rseq))) <= TOL
        assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL
        if cT is not None:
            assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL
    # the final state written over the initial one (the same tensors for both), one step and several
    for T in (1, 6):
        x = rng.uniform(-1, 1, (8, 1, 20)).astype(np.float32)
        h0 = rng.uniform(-0.5, 0.5, (L, 1, 72)).astype(np.float32)
        c0 = rng.uniform(-0.5, 0.5, (L, 1, 72)).astype(np.float32)
        xs.copy_(torch.from_numpy(x)); h0s.copy_(torch.from_numpy(h0))
        if c0s is not None:
            c0s.copy_(torch.from_numpy(c0))
        rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, x[:T], cfg.input, cfg.hidden, h0=h0.astype(np.float64),
                                            c0=c0.astype(np.float64) if c0s is not None else None)
        rnn.forward_into(xs[:T], h0s, c0s, hseq[:T], h0s, c0s)
        torch.cuda.synchronize()
        assert float(np.max(np.abs(hseq[:T].cpu().numpy() - rseq))) <= TOL
        assert float(np.max(np.abs(h0s.cpu().numpy() - rhT))) <= TOL
        if c0s is not None:
            assert float(np.max(np.abs(c0s.cpu().numpy() - rcT))) <= TOL


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
@pytest.mark.parametrize("L", [1, 2])
def test_rnn_streaming_on_tile_layout_plans(cell, L):
    """The streaming path on matrices planned again in the tile layout (equal split, row tiles
    shared between workgroups): its per-step launches then run the tile kernel, the GRU's with
    the row split of its step, stacked layers two products to a launch."""
    cfg = csb_inputs.RnnConfig("t", cell, L, 33, 100, 16, 3.0, "binomial", 0.3, 1, 6, 70 + L)
    wl = csb_inputs.make_rnn(cfg)
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, [torch.from_numpy(b).cuda() for b in wl.bias])
    for w in Ws:
        st = w.plan(5, 2)                                      # (a GRU's matrix keeps its row split)
        assert st["row_owned"] == 0
        w.validate()
        w.upload()
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda())
    torch.cuda.synchronize()
    assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= TOL
    assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL
    if cell == csb_inputs.LSTM:
        assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
def test_rnn_workloads_full_size(name):
    cfg = csb_inputs.CONFIGS[name]
    wl = csb_inputs.make_rnn(cfg)
    run_case(wl, tag=name)


def test_rnn_batched_two_layer_shape():
    """cfg4's shape (2 x LSTM 1024 -> 1024, block 64, 25x, batch 64) on the MFMA path; T is cut
    to 4 so that the float64 oracle finishes in seconds."""
    cfg = csb_inputs.CONFIGS["cfg4"]
    wl = csb_inputs.make_rnn(cfg, T=4)
    run_case(wl, tag="cfg4-T4", resident=False)


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
def test_rnn_batched_many_row_tiles(cell):
    """Small blocks and 1024 hidden units: 192-256 row tiles per matrix, so the upper layer's
    products (both inputs kept as [H][B]) take 64 right-hand sides per workgroup with 16-byte
    loads, in the two-source form; batch 64 and a batch that ends inside a tile of 64."""
    for B in (64, 52):
        cfg = csb_inputs.RnnConfig("t", cell, 2, 48, 1024, 16, 12.0, "binomial", 0.05, B, 3, 31)
        wl = csb_inputs.make_rnn(cfg)
        run_case(wl, tag=f"many-tiles-B{B}", resident=False)


@pytest.mark.parametrize("cell,I,H", [(csb_inputs.LSTM, 1100, 1000), (csb_inputs.GRU, 40, 1500), (csb_inputs.LSTM, 2040, 700)])
def test_rnn_resident_wide_inputs(cell, I, H):
    """Input plus state wider than 2048: a thread of the resident kernel stages three entries
    (and layer 0 reads two input words per thread when the input alone is wider than 1024)."""
    cfg = csb_inputs.RnnConfig("t", cell, 1, I, H, 50, 40.0, "binomial", 0.05, 1, 4, 17)
    wl = csb_inputs.make_rnn(cfg)
    rng = np.random.default_rng(3)
    h0 = rng.uniform(-0.5, 0.5, (1, 1, H)).astype(np.float32).astype(np.float64)
    c0 = rng.uniform(-0.5, 0.5, (1, 1, H)).astype(np.float32).astype(np.float64) if cell == csb_inputs.LSTM else None
    run_case(wl, h0, c0, tag="wide-inputs", resident=True)


def test_rnn_batched_full_size_sampled():
    """cfg4 as bench.py runs it (2 x LSTM 1024 -> 1024, batch 64, T = 256, the MFMA path).  The
    sequences of a batch are independent, so the float64 oracle runs three sampled ones on
    their own and the device results of those batch entries must match to the same bar."""
    cfg = csb_inputs.CONFIGS["cfg4"]
    wl = csb_inputs.make_rnn(cfg)
    T, B, _ = wl.x.shape
    assert (T, B) == (256, 64)
    say(f"[rnn] cfg4 full size T={T} B={B}")
    rnn = build_rnn(wl, resident=False)
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda())
    torch.cuda.synchronize()
    hseq, hT, cT = hseq.cpu().numpy(), hT.cpu().numpy(), cT.cpu().numpy()
    W = [oracle.csb_decode(oracle.csb_encode(m.A, m.br, m.bc)) for m in wl.W]
    for b in (0, 37, 63):
        rseq, rhT, rcT = oracle.rnn_forward(cfg.cell, W, wl.bias, np.ascontiguousarray(wl.x[:, b:b + 1]), cfg.input, cfg.hidden)
        e_seq = float(np.max(np.abs(hseq[:, b] - rseq[:, 0])))
        e_h = float(np.max(np.abs(hT[:, b] - rhT[:, 0])))
        e_c = float(np.max(np.abs(cT[:, b] - rcT[:, 0])))
        say(f"[rnn] cfg4 sequence {b}: err hseq={e_seq:.3g} hT={e_h:.3g} cT={e_c:.3g}")
        assert e_seq <= TOL and e_h <= TOL and e_c <= TOL


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
def test_rnn_batched_ragged(cell):
    cfg = csb_inputs.RnnConfig("t", cell, 2, 37, 70, 16, 4.0, "binomial", 0.3, 19, 6, 3)
    wl = csb_inputs.make_rnn(cfg)
    rng = np.random.default_rng(4)
    h0 = rng.uniform(-0.5, 0.5, (2, 19, 70)).astype(np.float32).astype(np.float64)
    c0 = rng.uniform(-0.5, 0.5, (2, 19, 70)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, c0 if cell == csb_inputs.LSTM else None, tag="batched-ragged", resident=False)


@pytest.mark.parametrize("batch,resident", [(2, False), (1, False), (1, True)])
@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
def test_rnn_resume_and_T0(cell, batch, resident):
    cfg = csb_inputs.RnnConfig("t", cell, 2, 24, 32, 16, 4.0, "binomial", 0.3, batch, 10, 5)
    wl = csb_inputs.make_rnn(cfg)
    rnn, (hseq, hT, cT) = run_case(wl, tag="resume-full", resident=resident)
    xd = torch.from_numpy(wl.x).cuda()
    s1, h1, c1 = rnn.forward(xd[:4].contiguous())
    s2, h2, c2 = rnn.forward(xd[4:].contiguous(), h1, c1)
    torch.cuda.synchronize()
    assert torch.equal(torch.cat([s1, s2]), hseq) and torch.equal(h2, hT)      # bitwise
    if cell == csb_inputs.LSTM:
        assert torch.equal(c2, cT)
    # T = 0 hands the state through
    s0, h0, c0 = rnn.forward(xd[:0].contiguous(), h1, c1)
    torch.cuda.synchronize()
    assert torch.equal(h0, h1)
    if cell == csb_inputs.LSTM:
        assert torch.equal(c0, c1)


@pytest.mark.parametrize("B,resident", [(2, False), (1, False), (1, True)])
def test_rnn_zero_weights_closed_form(B, resident):
    """W = 0, b = 0: LSTM c_T = c_0 / 2^T, h_T = tanh(c_T) / 2; GRU h_T = h_0 / 2^T."""
    I, H, T = 3, 5, 7
    rng = np.random.default_rng(2)
    x = rng.uniform(-1, 1, (T, B, I)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (1, B, H)).astype(np.float32)
    c0 = rng.uniform(-1, 1, (1, B, H)).astype(np.float32)
    for cell, G in ((0, 4), (1, 3)):
        W = CsbMatrix(np.zeros((G * H, I + H), np.float32), 4, 4)
        rnn = CsbRnn(cell, I, H, [W], None)
        if resident:
            rnn.upload()
        else:
            W.upload()
        _, hT, cT = rnn.forward(torch.from_numpy(x).cuda(), torch.from_numpy(h0).cuda(),
                                torch.from_numpy(c0).cuda() if cell == 0 else None)
        torch.cuda.synchronize()
        if cell == 0:
            assert np.allclose(cT.cpu().numpy(), c0 / 2.0 ** T, rtol=1e-6, atol=0)
            assert np.allclose(hT.cpu().numpy(), 0.5 * np.tanh(c0.astype(np.float64) / 2.0 ** T), rtol=1e-5, atol=1e-9)
        else:
            assert np.allclose(hT.cpu().numpy(), h0 / 2.0 ** T, rtol=1e-6, atol=0)


def test_rnn_handles_sharing_one_workspace_with_changing_lengths():
    """Three models take turns on ONE workspace buffer (a resident LSTM, a resident GRU, a
    streaming LSTM whose matrices are cut with shared row tiles, so its mat-vecs merge partial
    sums through tagged words), with sequence lengths going down and up again: the words that
    workgroups hand to each other carry launch tags, and stale words of another model, or of a
    longer earlier call, must never be taken for current ones."""
    T_max = 40
    cfgs = [csb_inputs.RnnConfig("a", csb_inputs.LSTM, 2, 20, 96, 16, 3.0, "binomial", 0.2, 1, T_max, 11),
            csb_inputs.RnnConfig("b", csb_inputs.GRU, 1, 33, 300, 32, 4.0, "binomial", 0.1, 1, T_max, 12),
            csb_inputs.RnnConfig("c", csb_inputs.LSTM, 1, 24, 64, 16, 2.0, "binomial", 0.2, 1, T_max, 13)]
    wls = [csb_inputs.make_rnn(c) for c in cfgs]
    rnns = []
    for k, wl in enumerate(wls):
        cfg = wl.cfg
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        bias = [torch.from_numpy(b).cuda() for b in wl.bias]
        if k == 2:
            for w in Ws:
                w.plan(7, 2)                                   # equal split: row tiles shared between workgroups
                assert w.stats["n_shared_tiles"] > 0
        rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, bias)
        if k < 2:
            assert rnn.stats()["resident"] == 1 and rnn.stats()["n_workgroups"] > 1
            rnn.upload()
        else:
            for w in Ws:
                w.upload()
        rnns.append(rnn)
    need = max(r.workspace_bytes(1, T_max) for r in rnns)
    shared = torch.empty(need // 4 + 64, dtype=torch.float32, device="cuda")
    shared.fill_(float("nan"))                                 # whatever an allocator may hand out
    for r in rnns:
        r._ws = shared
    refs = {}
    for k, T in [(0, 40), (1, 40), (2, 40), (0, 7), (1, 13), (2, 5), (1, 40), (0, 40), (2, 40), (0, 1), (0, 40)]:
        wl, cfg = wls[k], wls[k].cfg
        say(f"[rnn] shared workspace: model {k} T={T}")
        if (k, T) not in refs:
            refs[(k, T)] = oracle.rnn_forward(cfg.cell, [m.A for m in wl.W], wl.bias, wl.x[:T], cfg.input, cfg.hidden)
        rseq, rhT, _ = refs[(k, T)]
        hseq, hT, _ = rnns[k].forward(torch.from_numpy(wl.x[:T]).cuda())
        torch.cuda.synchronize()
        assert rnns[k]._ws is shared
        assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= TOL
        assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= TOL


@pytest.mark.parametrize("slots,rate", [(4, 8.0), (8, 4.0), (12, 1.5), (16, 1.5), (24, 1.5), (32, 1.5), (40, 1.5), (48, 1.5)])
@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
def test_rnn_resident_every_slot_count(cell, slots, rate, monkeypatch):
    """The resident kernel is compiled once per number of weights a lane keeps (4 to 48 in fours); the
    layout normally picks the smallest that fits.  CSB_RNN_S forces each of them in turn on a
    model dense enough to fill the slots (the forms beyond 24 slots gather in batches)."""
    monkeypatch.setenv("CSB_RNN_S", str(slots))
    cfg = csb_inputs.RnnConfig("t", cell, 2, 60, 160, 32, rate, "binomial", 0.08, 1, 12, 21 + slots)
    wl = csb_inputs.make_rnn(cfg)
    rnn, _ = run_case(wl, tag=f"slots-{slots}", resident=True)
    assert rnn.stats()["slots_per_lane"] == slots


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
@pytest.mark.parametrize("B", [3, 1])
@pytest.mark.parametrize("L,T", [(5, 7), (6, 2), (3, 1), (9, 4)])
def test_rnn_deep_stacks_by_diagonals(cell, L, T, B):
    """The streaming (B = 1) and batched paths run stacks by diagonals (layer l at step t with
    l + t constant share a launch, up to four layers per launch): more layers than a launch takes,
    more layers than steps, one step."""
    cfg = csb_inputs.RnnConfig("t", cell, L, 12, 16, 8, 2.0, "binomial", 0.3, B, T, 40 + L)
    wl = csb_inputs.make_rnn(cfg)
    rng = np.random.default_rng(L)
    h0 = rng.uniform(-0.5, 0.5, (L, B, 16)).astype(np.float32)
    c0 = rng.uniform(-0.5, 0.5, (L, B, 16)).astype(np.float32) if cell == csb_inputs.LSTM else None
    run_case(wl, h0, c0, tag=f"deep-{L}x{T}-b{B}", resident=False)


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
def test_rnn_resident_eight_layers(cell):
    """Eight layers is the deepest stack the resident kernel takes (one bias pointer per layer)."""
    cfg = csb_inputs.RnnConfig("t", cell, 8, 10, 24, 8, 2.0, "binomial", 0.3, 1, 6, 77)
    run_case(csb_inputs.make_rnn(cfg), tag="eight-layers", resident=True)

"""Parity of the further cells of Table 1 / Sec. 2.1 against the float64 oracle, through the
C ABI: Li-GRU (csb_rnn_create with CSB_CELL_LIGRU; streaming, resident and batched paths) and
the GRU with the reset gate before the candidate's recurrent product (csb_rnn_create_gru_rb;
streaming, resident and batched paths).  max |h - oracle| <= 1e-4 on every h_t and h_T; the Li-GRU's
state is not bounded by 1 (its candidate is a ReLU), so there the bound is 1e-4 times
max(1, max |h|) and the weights are drawn small enough for the recurrence to stay stable."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbRnn, CsbError, CELL_LIGRU, CELL_GRU_RB

pytestmark = pytest.mark.gpu
TOL = 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def build(wl, resident, replan=False):
    cfg = wl.cfg
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    if cfg.cell == csb_inputs.LIGRU:
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        rnn = CsbRnn(CELL_LIGRU, cfg.input, cfg.hidden, Ws, bias)
        mats = Ws
    else:
        Was, Uns = [], []
        for l, m in enumerate(wl.W):
            Wa, Un = csb_inputs.split_gru_rb(m.A, cfg.input if l == 0 else cfg.hidden, cfg.hidden)
            Was.append(CsbMatrix(Wa, m.br, m.bc))
            Uns.append(CsbMatrix(Un, m.br, m.bc))
        rnn = CsbRnn(CELL_GRU_RB, cfg.input, cfg.hidden, Was, bias, Wp=Uns)
        mats = Was + Uns
    if resident:
        assert rnn.stats()["resident"] == 1
        rnn.upload()
    else:
        for m in mats:
            # plans whose workgroups own whole units (the step's launches finish their cells)
            assert m.plan_stats()["row_owned"] == 2
            if replan:                        # a plan of the caller's: plain row ranges, cells computed where they are consumed
                assert m.plan_rows(0, 0)["row_owned"] == 1
            m.validate()
            m.upload()
    return rnn


def run_case(wl, h0=None, tag="", resident=False, replan=False):
    cfg = wl.cfg
    T, B, _ = wl.x.shape
    L = cfg.n_layers
    say(f"[cells] {tag} cell={cfg.cell} L={L} I={cfg.input} H={cfg.hidden} T={T} B={B} resident={resident}")
    rseq, rhT, _ = oracle.rnn_forward(cfg.cell, [m.A for m in wl.W], wl.bias, wl.x, cfg.input, cfg.hidden, h0=h0)
    rnn = build(wl, resident, replan)
    h0d = None if h0 is None else torch.from_numpy(h0.astype(np.float32)).cuda()
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda(), h0d)
    torch.cuda.synchronize()
    assert cT is None and hseq.shape == (T, B, cfg.hidden) and hT.shape == (L, B, cfg.hidden)
    e_seq = float(np.max(np.abs(hseq.cpu().numpy() - rseq))) if T else 0.0
    e_h = float(np.max(np.abs(hT.cpu().numpy() - rhT)))
    scale = max(1.0, float(np.max(np.abs(rseq))) if T else 1.0)
    say(f"[cells] {tag} err hseq={e_seq:.3g} hT={e_h:.3g} max|h|={scale:.3g}")
    assert scale < 50.0                       # the case itself must be a sane one
    assert e_seq <= TOL * scale and e_h <= TOL * scale
    return rnn


def workload(cell, L, I, H, T, B, block, seed, rate=3.0, sigma=0.3):
    cfg = csb_inputs.RnnConfig("t", cell, L, I, H, block, rate, "binomial", sigma, B, T, seed)
    return csb_inputs.make_rnn(cfg)


SHAPES = [(1, 5, 8, 6, 1, 4), (2, 12, 16, 9, 3, 8), (3, 7, 12, 4, 2, 4), (1, 40, 100, 12, 1, 32),
          (2, 30, 96, 7, 19, 16), (2, 33, 300, 9, 1, 32), (3, 16, 64, 20, 1, 16),
          (5, 9, 16, 6, 1, 8), (6, 9, 16, 3, 4, 8)]


@pytest.mark.parametrize("L,I,H,T,B,block", SHAPES)
def test_ligru_small(L, I, H, T, B, block):
    wl = workload(csb_inputs.LIGRU, L, I, H, T, B, block, seed=60 + L + I, sigma=min(0.3, 1.2 / np.sqrt(I + H)))
    h0 = np.random.default_rng(1).uniform(-0.5, 0.5, (L, B, H)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, tag="ligru")
    run_case(wl, None, tag="ligru-zero-state")
    if B == 1:
        run_case(wl, h0, tag="ligru-resident", resident=True)
        run_case(wl, None, tag="ligru-resident-zero-state", resident=True)


@pytest.mark.parametrize("cell", [csb_inputs.LIGRU, csb_inputs.GRU_RB])
@pytest.mark.parametrize("L,I,H,T,block", [(1, 40, 100, 12, 32), (2, 33, 300, 9, 32), (5, 9, 16, 6, 8)])
def test_cells_on_plans_the_caller_makes(cell, L, I, H, T, block):
    """Matrices planned again by the caller (plain row ranges instead of the whole units
    csb_rnn_create lays out): the streaming step computes a cell where its output is consumed."""
    wl = workload(cell, L, I, H, T, 1, block, seed=60 + L + I, sigma=min(0.3, 1.2 / np.sqrt(I + H)))   # (keeps the unbounded Li-GRU state tame)
    h0 = np.random.default_rng(2).uniform(-0.5, 0.5, (L, 1, H)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, tag="caller-planned", replan=True)


@pytest.mark.parametrize("L,I,H,T,B,block", SHAPES)
def test_gru_rb_small(L, I, H, T, B, block):
    wl = workload(csb_inputs.GRU_RB, L, I, H, T, B, block, seed=80 + L + I)
    h0 = np.random.default_rng(2).uniform(-0.5, 0.5, (L, B, H)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, tag="gru_rb")
    run_case(wl, None, tag="gru_rb-zero-state")
    if B == 1:
        run_case(wl, h0, tag="gru_rb-resident", resident=True)
        run_case(wl, None, tag="gru_rb-resident-zero-state", resident=True)


def test_ligru_speech_model_shape():
    """The SR3 rows of Table 1: two Li-GRU layers, 39 -> 512 -> 512, pruned 7.1x (32 x 32
    blocks here); batch 1, T = 50, on the resident and the streaming path."""
    wl = workload(csb_inputs.LIGRU, 2, 39, 512, 50, 1, 32, seed=0, rate=7.1, sigma=0.05)
    rnn = run_case(wl, tag="sr3-resident", resident=True)
    say(f"[cells] sr3 resident plan {rnn.stats()}")
    run_case(wl, tag="sr3-streaming", resident=False)


def test_gru_rb_speech_model_shape():
    """The SR2 rows of Table 1 (GRU 39 -> 1024 -> 1024, 21.7x) in the reset-before form, batch 1
    and batch 16."""
    wl = workload(csb_inputs.GRU_RB, 2, 39, 1024, 12, 1, 32, seed=0, rate=21.7, sigma=0.05)
    run_case(wl, tag="sr2-rb")
    rnn = run_case(wl, tag="sr2-rb-resident", resident=True)      # the gate stages stage 39 + 2 x 1024 inputs: three per thread
    say(f"[cells] sr2-rb resident plan {rnn.stats()}")
    wl = workload(csb_inputs.GRU_RB, 2, 39, 1024, 6, 16, 32, seed=1, rate=21.7, sigma=0.05)
    run_case(wl, tag="sr2-rb-batch16")


def test_t0_hands_state_through():
    for cell in (csb_inputs.LIGRU, csb_inputs.GRU_RB):
        wl = workload(cell, 2, 6, 8, 0, 2, 4, seed=3)
        h0 = np.random.default_rng(5).uniform(-1, 1, (2, 2, 8)).astype(np.float32)
        rnn = build(wl, False)
        _, hT, _ = rnn.forward(torch.from_numpy(wl.x).cuda(), torch.from_numpy(h0).cuda())
        assert np.array_equal(hT.cpu().numpy(), h0)


def test_gru_rb_rejects_recurrent_entries_in_the_n_rows_of_wa():
    wl = workload(csb_inputs.GRU_RB, 1, 6, 8, 2, 1, 4, seed=4, rate=1.5)
    A = wl.W[0].A
    assert np.any(A[16:, 6:] != 0)
    _, Un = csb_inputs.split_gru_rb(A, 6, 8)
    with pytest.raises(CsbError):
        CsbRnn(CELL_GRU_RB, 6, 8, [CsbMatrix(A, 4, 4)], None, Wp=[CsbMatrix(Un, 4, 4)])
    with pytest.raises(CsbError):                      # wrong shape of Un
        Wa, _ = csb_inputs.split_gru_rb(A, 6, 8)
        CsbRnn(CELL_GRU_RB, 6, 8, [CsbMatrix(Wa, 4, 4)], None, Wp=[CsbMatrix(A[:8, :7].copy(), 4, 4)])


@pytest.mark.parametrize("kind", ["lstm", "gru", "ligru", "gru_rb", "lstmp"])
@pytest.mark.parametrize("resident", [False, True])
def test_final_state_does_not_depend_on_asking_for_the_sequence(kind, resident):
    """Without an output sequence the streaming paths keep h_t in workspace buffers only (with
    one, the last layer's goes straight into it): both must end in the same state, bit for bit."""
    from paper_2005_05758_amd import CELL_LSTM, CELL_GRU, CELL_LSTMP
    L, I, H, P, T, block = 2, 20, 48, 24, 9, 16
    if kind == "lstmp":
        wl = csb_inputs.make_lstmp(5, L, I, H, P, block, 3.0, T, 1, sigma=0.2)
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        Ps = [CsbMatrix(m.A, m.br, m.bc) for m in wl.Wp]
        rnn = CsbRnn(CELL_LSTMP, I, H, Ws, [torch.from_numpy(b).cuda() for b in wl.bias], proj=P, Wp=Ps)
        mats = Ws + Ps
    elif kind == "gru_rb":
        wl = workload(csb_inputs.GRU_RB, L, I, H, T, 1, block, 5, sigma=0.2)
        parts = [csb_inputs.split_gru_rb(m.A, I if l == 0 else H, H) for l, m in enumerate(wl.W)]
        Was = [CsbMatrix(p[0], block, block) for p in parts]
        Uns = [CsbMatrix(p[1], block, block) for p in parts]
        rnn = CsbRnn(CELL_GRU_RB, I, H, Was, [torch.from_numpy(b).cuda() for b in wl.bias], Wp=Uns)
        mats = Was + Uns
    else:
        cell = {"lstm": CELL_LSTM, "gru": CELL_GRU, "ligru": CELL_LIGRU}[kind]
        wl = workload(cell, L, I, H, T, 1, block, 5, sigma=0.2)
        mats = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        rnn = CsbRnn(cell, I, H, mats, [torch.from_numpy(b).cuda() for b in wl.bias])
    if resident:
        rnn.upload()
    else:
        for m in mats:
            m.upload()
    say(f"[cells] with / without sequence: {kind} resident={resident}")
    xd = torch.from_numpy(wl.x).cuda()
    s1, h1, c1 = rnn.forward(xd, want_hseq=True)
    s2, h2, c2 = rnn.forward(xd, want_hseq=False)
    torch.cuda.synchronize()
    assert s2 is None and torch.equal(h1, h2) and torch.equal(s1[-1, 0], h1[-1, 0])
    if c1 is not None:
        assert torch.equal(c1, c2)

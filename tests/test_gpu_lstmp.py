"""Parity of the LSTM with a recurrent projection (csb_rnn_create_lstmp + csb_rnn_forward,
batch 1 on the mat-vec kernel, batch > 1 on the matrix cores) against the float64 oracle:
max |h - oracle| <= 1e-4 on every h_t, h_T and c_T, as for the other cells."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbRnn, CsbError, CELL_LSTMP

pytestmark = pytest.mark.gpu
TOL = 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def build(wl, resident=False, replan=False):
    """resident=True: upload the on-chip layout (one launch for the whole sequence, batch 1);
    else upload the matrices (mat-vec / mat-mat launches per step)."""
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    Ps = [CsbMatrix(m.A, m.br, m.bc) for m in wl.Wp]
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    rnn = CsbRnn(CELL_LSTMP, wl.input, wl.hidden, Ws, bias, proj=wl.proj, Wp=Ps)
    if resident:
        assert rnn.stats()["resident"] == 1
        rnn.upload()
    else:
        for m in Ws + Ps:
            if replan:                        # a plan of the caller's: plain row ranges, the cell computed where it is consumed
                assert m.plan_rows(0, 0)["row_owned"] == 1
            m.validate()
            m.upload()
    return rnn


def run_case(wl, h0=None, c0=None, tag="", resident=None, replan=False):
    T, B, _ = wl.x.shape
    L = len(wl.W)
    if resident is None:                      # both device paths where both apply
        out = run_case(wl, h0, c0, tag, resident=False)
        if B == 1:
            out = run_case(wl, h0, c0, tag, resident=True)
        return out
    say(f"[lstmp] {tag} L={L} I={wl.input} H={wl.hidden} P={wl.proj} T={T} B={B} resident={resident}")
    W = [m.A for m in wl.W]
    Wp = [m.A for m in wl.Wp]
    rseq, rhT, rcT = oracle.lstmp_forward(W, Wp, wl.bias, wl.x, wl.input, wl.hidden, wl.proj, h0=h0, c0=c0)
    rnn = build(wl, resident, replan)
    h0d = None if h0 is None else torch.from_numpy(h0.astype(np.float32)).cuda()
    c0d = None if c0 is None else torch.from_numpy(c0.astype(np.float32)).cuda()
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda(), h0d, c0d)
    torch.cuda.synchronize()
    assert hseq.shape == (T, B, wl.proj) and hT.shape == (L, B, wl.proj) and cT.shape == (L, B, wl.hidden)
    e_seq = float(np.max(np.abs(hseq.cpu().numpy() - rseq))) if T else 0.0
    e_h = float(np.max(np.abs(hT.cpu().numpy() - rhT)))
    e_c = float(np.max(np.abs(cT.cpu().numpy() - rcT)))
    say(f"[lstmp] {tag} err hseq={e_seq:.3g} hT={e_h:.3g} cT={e_c:.3g}")
    assert e_seq <= TOL and e_h <= TOL and e_c <= TOL
    return rnn


@pytest.mark.parametrize("L,I,H,P,T,B,block", [(1, 5, 8, 3, 6, 1, 4), (2, 12, 16, 8, 9, 3, 8), (3, 7, 12, 11, 4, 2, 4),
                                              (1, 40, 100, 37, 12, 1, 32), (2, 30, 96, 48, 7, 19, 16), (2, 9, 8, 16, 5, 2, 8),
                                              (2, 33, 300, 130, 9, 1, 32), (3, 16, 64, 24, 20, 1, 16),
                                              (5, 10, 16, 12, 6, 1, 8), (6, 10, 16, 8, 3, 4, 8)])   # more layers than one launch takes
def test_lstmp_small(L, I, H, P, T, B, block):
    wl = csb_inputs.make_lstmp(40 + L + I, L, I, H, P, block, 3.0, T, B, sigma=0.3)
    rng = np.random.default_rng(1)
    h0 = rng.uniform(-0.5, 0.5, (L, B, P)).astype(np.float32).astype(np.float64)
    c0 = rng.uniform(-0.5, 0.5, (L, B, H)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, c0, tag="small")
    run_case(wl, tag="small-zero-state")


@pytest.mark.parametrize("L,I,H,P,T,block", [(1, 40, 100, 37, 12, 32), (2, 33, 300, 130, 9, 32), (5, 10, 16, 12, 6, 8)])
def test_lstmp_on_plans_the_caller_makes(L, I, H, P, T, block):
    """Matrices planned again by the caller (plain row ranges instead of the whole units
    csb_rnn_create_lstmp lays the gate matrices out in): the projection's launch computes the cell
    on its way in."""
    wl = csb_inputs.make_lstmp(60 + L + I, L, I, H, P, block, 3.0, T, 1, sigma=0.3)
    rng = np.random.default_rng(2)
    h0 = rng.uniform(-0.5, 0.5, (L, 1, P)).astype(np.float32).astype(np.float64)
    c0 = rng.uniform(-0.5, 0.5, (L, 1, H)).astype(np.float32).astype(np.float64)
    run_case(wl, h0, c0, tag="caller-planned", resident=False, replan=True)


def test_lstmp_speech_model_shape_batch1():
    """The paper's SR1 rows of Table 1: two LSTMP layers, 153 -> 1024 and 512 -> 1024 with a
    512-wide projection, pruned 13x in 32 x 32 blocks; batch 1, T = 20."""
    wl = csb_inputs.make_lstmp(0, 2, 153, 1024, 512, 32, 13.0, 20, 1)
    run_case(wl, tag="sr1-shape")
    wl = csb_inputs.make_lstmp(0, 2, 153, 1024, 512, 32, 13.0, 100, 1)
    run_case(wl, tag="sr1-shape-T100", resident=True)


def test_lstmp_speech_model_shape_batched_sampled():
    """Same model at batch 16 on the matrix cores, T = 50; the oracle runs two of the sequences."""
    wl = csb_inputs.make_lstmp(0, 2, 153, 1024, 512, 32, 13.0, 50, 16)
    rnn = build(wl)
    hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda())
    torch.cuda.synchronize()
    hseq, hT, cT = hseq.cpu().numpy(), hT.cpu().numpy(), cT.cpu().numpy()
    W, Wp = [m.A for m in wl.W], [m.A for m in wl.Wp]
    for b in (0, 11):
        rseq, rhT, rcT = oracle.lstmp_forward(W, Wp, wl.bias, np.ascontiguousarray(wl.x[:, b:b + 1]), 153, 1024, 512)
        e = max(float(np.max(np.abs(hseq[:, b] - rseq[:, 0]))), float(np.max(np.abs(hT[:, b] - rhT[:, 0]))),
                float(np.max(np.abs(cT[:, b] - rcT[:, 0]))))
        say(f"[lstmp] sr1 batched sequence {b}: max err {e:.3g}")
        assert e <= TOL


def test_lstmp_T0_and_shape_errors():
    wl = csb_inputs.make_lstmp(3, 1, 6, 8, 4, 4, 2.0, 0, 2, sigma=0.3)
    rnn = build(wl)
    h0 = torch.rand(1, 2, 4, device="cuda")
    c0 = torch.rand(1, 2, 8, device="cuda")
    hseq, hT, cT = rnn.forward(torch.empty(0, 2, 6, device="cuda"), h0, c0)
    torch.cuda.synchronize()
    assert torch.equal(hT, h0) and torch.equal(cT, c0)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    bad = [CsbMatrix(np.zeros((5, 8), np.float32), 4, 4)]            # projection must be proj x hidden
    with pytest.raises(CsbError):
        CsbRnn(CELL_LSTMP, 6, 8, Ws, None, proj=4, Wp=bad)

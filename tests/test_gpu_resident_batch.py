"""A batch on the resident kernel (csb_rnn_forward with batch > 1 on a handle whose resident
layout is uploaded): the sequences of a batch are independent (Sec. 2.1: every cell's state
depends on its own past only), so they run as instances of the one-sequence kernel side by side.
Against the float64 oracle to 1e-4 like every other path, and bit for bit against the same
handle run one sequence at a time; several rounds, ragged last rounds, all cells, models that
span one and several XCDs, calls of different T, batch and path in turn on one workspace."""
import os
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
import paper_2005_05758_amd as P
from paper_2005_05758_amd import CsbMatrix, CsbRnn

pytestmark = pytest.mark.gpu
TOL = 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def make(kind, L, I, H, proj, block, rate, T, B, seed, sigma=None):
    """(handle, matrices, reference function) of a seeded model."""
    sigma = sigma if sigma is not None else min(0.3, 1.2 / np.sqrt(I + H))
    if kind == "lstmp":
        wl = csb_inputs.make_lstmp(seed, L, I, H, proj, block, rate, T, B, sigma=sigma)
        bias = [torch.from_numpy(b).cuda() for b in wl.bias]
        Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        Ps = [CsbMatrix(m.A, m.br, m.bc) for m in wl.Wp]
        rnn, mats = CsbRnn(P.CELL_LSTMP, I, H, Ws, bias, proj=proj, Wp=Ps), Ws + Ps

        def ref(x, h0, c0):
            return oracle.lstmp_forward([m.A for m in wl.W], [m.A for m in wl.Wp], wl.bias, x, I, H, proj, h0=h0, c0=c0)
        return wl, rnn, mats, ref
    cell = {"lstm": P.CELL_LSTM, "gru": P.CELL_GRU, "ligru": P.CELL_LIGRU, "gru_rb": P.CELL_GRU_RB}[kind]
    wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", cell, L, I, H, block, rate, "binomial", sigma, B, T, seed))
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    if kind == "gru_rb":
        parts = [csb_inputs.split_gru_rb(m.A, I if l == 0 else H, H) for l, m in enumerate(wl.W)]
        Was = [CsbMatrix(p[0], block, block) for p in parts]
        Uns = [CsbMatrix(p[1], block, block) for p in parts]
        rnn, mats = CsbRnn(P.CELL_GRU_RB, I, H, Was, bias, Wp=Uns), Was + Uns
    else:
        mats = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
        rnn = CsbRnn(cell, I, H, mats, bias)

    def ref(x, h0, c0):
        return oracle.rnn_forward(cell, [m.A for m in wl.W], wl.bias, x, I, H, h0=h0, c0=c0)
    return wl, rnn, mats, ref


def states(kind, L, B, H, proj, seed):
    rng = np.random.default_rng(seed)
    hs = proj if kind == "lstmp" else H
    h0 = rng.uniform(-0.5, 0.5, size=(L, B, hs)).astype(np.float32)
    c0 = rng.uniform(-0.5, 0.5, size=(L, B, H)).astype(np.float32) if kind in ("lstm", "lstmp") else None
    return h0, c0


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check(got, want, what):
    hseq, hT, cT = got
    rseq, rhT, rcT = want
    scale = max(1.0, float(np.max(np.abs(rseq))) if rseq.size else 1.0)
    assert scale < 50.0
    e1 = float(np.max(np.abs(hseq.cpu().numpy() - rseq))) if rseq.size else 0.0
    e2 = float(np.max(np.abs(hT.cpu().numpy() - rhT)))
    say(f"[resident batch] {what}: err hseq={e1:.3g} hT={e2:.3g}")
    assert e1 <= TOL * scale and e2 <= TOL * scale
    if cT is not None:
        assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= TOL * max(scale, float(np.max(np.abs(rcT))))


CASES = [  # kind, L, I, H, proj, block, rate, T, B
    ("lstm", 2, 20, 64, 0, 16, 3.0, 7, 2),
    ("lstm", 1, 33, 100, 0, 4, 2.0, 12, 9),
    ("lstm", 1, 10, 24, 0, 4, 2.0, 6, 250),          # a one-workgroup model: many instances per XCD, two rounds
    ("gru", 2, 33, 160, 0, 8, 2.0, 5, 40),
    ("gru", 2, 16, 48, 0, 8, 3.0, 9, 5),
    ("gru", 3, 12, 40, 0, 8, 2.0, 1, 19),
    ("ligru", 2, 24, 64, 0, 16, 4.0, 10, 8),
    ("gru_rb", 2, 16, 48, 0, 8, 3.0, 8, 11),
    ("lstmp", 2, 20, 64, 24, 8, 3.0, 6, 10),
    ("lstm", 2, 153, 1024, 0, 32, 16.0, 5, 6),        # several XCDs per instance: fewer of them side by side
    ("lstmp", 1, 40, 768, 256, 32, 8.0, 4, 3),
]


@pytest.mark.parametrize("kind,L,I,H,proj,block,rate,T,B", CASES)
def test_against_oracle_and_one_sequence_at_a_time(kind, L, I, H, proj, block, rate, T, B):
    wl, rnn, mats, ref = make(kind, L, I, H, proj, block, rate, T, B, seed=300 + L + I)
    st = rnn.stats()
    say(f"[resident batch] {kind} L={L} I={I} H={H} proj={proj} T={T} B={B} plan {st}")
    assert st["resident"] == 1
    rnn.upload()                                      # the matrices are not uploaded: only the resident kernel can run it
    for with_state in (False, True):
        h0, c0 = states(kind, L, B, H, proj, 7) if with_state else (None, None)
        got = rnn.forward(dev(wl.x), dev(h0), dev(c0))
        torch.cuda.synchronize()
        check(got, ref(wl.x, h0, c0), f"{kind} state={with_state}")
        # the same kernel, the same arithmetic: sequence b alone gives the same bits
        for b in sorted({0, B // 2, B - 1}):
            one = rnn.forward(dev(wl.x[:, b:b + 1]), dev(None if h0 is None else h0[:, b:b + 1]),
                              dev(None if c0 is None else c0[:, b:b + 1]))
            torch.cuda.synchronize()
            assert torch.equal(one[0][:, 0], got[0][:, b]) and torch.equal(one[1][:, 0], got[1][:, b])
            if got[2] is not None:
                assert torch.equal(one[2][:, 0], got[2][:, b])
    s2, h2, c2 = rnn.forward(dev(wl.x), want_hseq=False)
    s1, h1, c1 = rnn.forward(dev(wl.x))
    torch.cuda.synchronize()
    assert s2 is None and torch.equal(h1, h2)


def test_both_batch_paths_agree_and_share_a_workspace():
    """With the matrices uploaded too the library picks a path by its cost estimate;
    CSB_RNN_BATCH_PATH names one.  Calls of different T, batch and path follow each other on one
    handle (one workspace): every one must still match the oracle."""
    kind, L, I, H, block = "lstm", 2, 40, 96, 16
    wl, rnn, mats, ref = make(kind, L, I, H, 0, block, 3.0, 40, 8, seed=5)
    rnn.upload()
    for m in mats:
        m.upload()
    old = os.environ.get("CSB_RNN_BATCH_PATH")
    try:
        plan = [("resident", 40, 8), ("batched", 40, 8), ("resident", 5, 8), ("resident", 40, 8), (None, 40, 1),
                ("resident", 17, 3), ("batched", 17, 3), ("resident", 40, 8), (None, 9, 1), (None, 40, 8)]
        for path, T, B in plan:
            if path is None:
                os.environ.pop("CSB_RNN_BATCH_PATH", None)
            else:
                os.environ["CSB_RNN_BATCH_PATH"] = path
            x = np.ascontiguousarray(wl.x[:T, :B])
            h0, c0 = states(kind, L, B, H, 0, T + B)
            got = rnn.forward(dev(x), dev(h0), dev(c0))
            torch.cuda.synchronize()
            check(got, ref(x, h0, c0), f"path={path} T={T} B={B}")
    finally:
        if old is None:
            os.environ.pop("CSB_RNN_BATCH_PATH", None)
        else:
            os.environ["CSB_RNN_BATCH_PATH"] = old


def test_headline_model_batch_of_eight():
    """The model the headline figure is quoted on (LSTM 153 -> 512, pruned 10x, 32 x 32 blocks):
    eight sequences at once on the resident kernel."""
    cfg = csb_inputs.CONFIGS["cfg2"]
    wl = csb_inputs.make_rnn(cfg, T=20, batch=8)
    mats = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(P.CELL_LSTM, cfg.input, cfg.hidden, mats, [torch.from_numpy(b).cuda() for b in wl.bias])
    rnn.upload()
    say(f"[resident batch] headline model, batch 8: plan {rnn.stats()}")
    got = rnn.forward(dev(wl.x))
    torch.cuda.synchronize()
    check(got, oracle.rnn_forward(cfg.cell, [m.A for m in wl.W], wl.bias, wl.x, cfg.input, cfg.hidden), "cfg2 x 8")


PLANNED = [  # kind, L, I, H, proj, block, rate, T, B
    ("lstm", 1, 153, 512, 0, 32, 10.0, 9, 40),        # the headline model's shape
    ("gru", 2, 64, 256, 0, 16, 8.0, 7, 64),
    ("ligru", 2, 39, 512, 0, 32, 7.1, 5, 24),
    ("gru_rb", 2, 24, 128, 0, 8, 4.0, 6, 33),
    ("lstmp", 2, 40, 256, 96, 16, 6.0, 6, 20),
    ("lstm", 2, 20, 64, 0, 16, 3.0, 7, 300),
]


@pytest.mark.parametrize("kind,L,I,H,proj,block,rate,T,B", PLANNED)
def test_layout_planned_for_the_batch(kind, L, I, H, proj, block, rate, T, B):
    """csb_rnn_plan_resident(batch): another slot count per lane, smaller instances, more of them
    per launch -- the same results to the same bar, for one sequence on that layout too."""
    wl, rnn, mats, ref = make(kind, L, I, H, proj, block, rate, T, B, seed=500 + L + I, sigma=0.05 if H >= 256 else None)
    before = rnn.stats()
    rnn.plan_resident(B)
    after = rnn.stats()
    say(f"[resident batch] planned for {B}: {kind} L={L} H={H}: {before['n_workgroups']} workgroups x {before['slots_per_lane']} slots"
        f" -> {after['n_workgroups']} x {after['slots_per_lane']}")
    rnn.upload()
    h0, c0 = states(kind, L, B, H, proj, 11)
    got = rnn.forward(dev(wl.x), dev(h0), dev(c0))
    torch.cuda.synchronize()
    check(got, ref(wl.x, h0, c0), f"{kind} planned for {B}")
    one = rnn.forward(dev(wl.x[:, 3:4]), dev(h0[:, 3:4]), dev(None if c0 is None else c0[:, 3:4]))
    torch.cuda.synchronize()
    assert torch.equal(one[0][:, 0], got[0][:, 3]) and torch.equal(one[1][:, 0], got[1][:, 3])
    rnn.plan_resident(1)                              # and back: the handle must be uploaded again
    with pytest.raises(P.CsbError):
        rnn.forward(dev(wl.x))
    rnn.upload()
    assert rnn.stats() == before
    got = rnn.forward(dev(wl.x), dev(h0), dev(c0))
    torch.cuda.synchronize()
    check(got, ref(wl.x, h0, c0), f"{kind} back on the one-sequence layout")

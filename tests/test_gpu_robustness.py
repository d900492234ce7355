"""Failure handling on the device side, forced from the host so that every kernel still exits
normally: a wait of the resident kernel that gives up (bounded polls) must be visible to the
host (csb_rnn_status), and a weight matrix planned again in another row layout after
csb_rnn_create must be refused by csb_rnn_forward instead of being misread."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbRnn
from paper_2005_05758_amd.binding import CsbError, CELL_GRU

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def test_resident_wait_that_gives_up_is_reported():
    cfg = csb_inputs.CONFIGS["cfg2"]                 # 20 workgroups that wait for each other's h_t every step
    wl = csb_inputs.make_rnn(cfg, T=40)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, bias)
    assert rnn.stats()["resident"] == 1 and rnn.stats()["n_workgroups"] > 1
    rnn.upload()
    xd = torch.from_numpy(wl.x).cuda()
    say("[robust] normal run")
    hseq, hT, cT = rnn.forward(xd)
    torch.cuda.synchronize()
    assert rnn.status() == 0 and bool(torch.isfinite(hT).all())
    good = hT.clone()
    say("[robust] poll limit 0: a word must be there at the first look")
    rnn.set_poll_limit(0)
    hseq, hT, cT = rnn.forward(xd)
    torch.cuda.synchronize()                          # the launch ends by itself
    st = rnn.status()
    say(f"[robust] status {st}, finite {bool(torch.isfinite(hT).all())}")
    # either every word happened to be there (then the result is the good one) or the status says so
    assert st != 0 or torch.equal(hT, good)
    if st != 0:
        assert not bool(torch.isfinite(hseq).all())   # the NaNs are where the wait gave up, and the host knows
    assert rnn.status() == 0                          # reading clears it
    say("[robust] default limit again")
    rnn.set_poll_limit(1 << 24)
    hseq, hT, cT = rnn.forward(xd)
    torch.cuda.synchronize()
    assert rnn.status() == 0 and torch.equal(hT, good)


def test_forward_refuses_a_gru_matrix_planned_in_another_layout():
    cfg = csb_inputs.CONFIGS["cfg3"]
    wl = csb_inputs.make_rnn(cfg, T=3)
    M = CsbMatrix(wl.W[0].A, wl.W[0].br, wl.W[0].bc)
    bias = [torch.from_numpy(b).cuda() for b in wl.bias]
    rnn = CsbRnn(CELL_GRU, cfg.input, cfg.hidden, [M], bias)
    xd = torch.from_numpy(wl.x).cuda()
    M.upload()
    hseq, hT, _ = rnn.forward(xd)                     # streaming path, the layout csb_rnn_create planned
    torch.cuda.synchronize()
    W = [oracle.csb_decode(oracle.csb_encode(wl.W[0].A, wl.W[0].br, wl.W[0].bc))]
    _, rhT, _ = oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
    assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= 1e-4
    M.plan(0, 1)                                      # planned again: same row layout, other mode
    M.upload()
    hseq, hT2, _ = rnn.forward(xd)
    torch.cuda.synchronize()
    assert float(np.max(np.abs(hT2.cpu().numpy() - rhT))) <= 1e-4
    M.plan_rows()                                     # the plain row layout: 3H output rows, not what the step kernels index
    M.upload()
    with pytest.raises(CsbError) as ei:
        rnn.forward(xd)
    assert ei.value.code == -5

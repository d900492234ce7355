"""Pins for the oracle's LSTM / GRU (Sec. 2.1) -- library special case + closed forms."""
import numpy as np
import pytest
import torch

import csb_inputs
import oracle


def _torch_ref(cell, W, bias, x, I, H, h0=None, c0=None):
    """torch.nn.LSTM / torch.nn.GRU, CPU, float64: weight_ih|weight_hh = W split at the input
    width, bias_ih = b, bias_hh = 0 (so the GRU's hidden-side n bias vanishes)."""
    L = len(W)
    T, B, _ = x.shape
    mod = (torch.nn.LSTM if cell == 0 else torch.nn.GRU)(I, H, num_layers=L, bias=True).double()
    with torch.no_grad():
        for l in range(L):
            n_in = I if l == 0 else H
            getattr(mod, f"weight_ih_l{l}").copy_(torch.from_numpy(W[l][:, :n_in].astype(np.float64)))
            getattr(mod, f"weight_hh_l{l}").copy_(torch.from_numpy(W[l][:, n_in:].astype(np.float64)))
            getattr(mod, f"bias_ih_l{l}").copy_(torch.from_numpy(bias[l].astype(np.float64)))
            getattr(mod, f"bias_hh_l{l}").zero_()
        xt = torch.from_numpy(x.astype(np.float64))
        h0t = torch.zeros(L, B, H, dtype=torch.float64) if h0 is None else torch.from_numpy(h0)
        if cell == 0:
            c0t = torch.zeros(L, B, H, dtype=torch.float64) if c0 is None else torch.from_numpy(c0)
            out, (hT, cT) = mod(xt, (h0t, c0t))
            return out.numpy(), hT.numpy(), cT.numpy()
        out, hT = mod(xt, h0t)
        return out.numpy(), hT.numpy(), None


def _small(cell, L, I, H, T, B, seed, block=8, rate=3.0):
    cfg = csb_inputs.RnnConfig("t", cell, L, I, H, block, rate, "binomial", 0.3, B, T, seed)
    return csb_inputs.make_rnn(cfg)


@pytest.mark.parametrize("cell", [csb_inputs.LSTM, csb_inputs.GRU])
@pytest.mark.parametrize("L,I,H,T,B", [(1, 5, 7, 6, 1), (2, 12, 16, 9, 3), (3, 8, 8, 4, 2)])
def test_against_torch_float64(cell, L, I, H, T, B):
    wl = _small(cell, L, I, H, T, B, seed=11 + L)
    W = [m.A for m in wl.W]
    rng = np.random.default_rng(1)
    h0 = rng.uniform(-0.5, 0.5, (L, B, H))
    c0 = rng.uniform(-0.5, 0.5, (L, B, H))
    hseq, hT, cT = oracle.rnn_forward(cell, W, wl.bias, wl.x, I, H, h0=h0, c0=c0)
    rseq, rhT, rcT = _torch_ref(cell, W, wl.bias, wl.x, I, H, h0, c0)
    assert np.allclose(hseq, rseq, rtol=0, atol=1e-12)
    assert np.allclose(hT, rhT, rtol=0, atol=1e-12)
    if cell == 0:
        assert np.allclose(cT, rcT, rtol=0, atol=1e-12)


def test_cfg1_shape_against_torch():
    cfg = csb_inputs.CONFIGS["cfg1"]
    wl = csb_inputs.make_rnn(cfg)
    W = [m.A for m in wl.W]
    hseq, hT, cT = oracle.rnn_forward(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
    rseq, rhT, rcT = _torch_ref(cfg.cell, W, wl.bias, wl.x, cfg.input, cfg.hidden)
    assert np.allclose(hseq, rseq, rtol=0, atol=1e-12) and np.allclose(cT, rcT, rtol=0, atol=1e-12)


def test_zero_weights_closed_forms():
    I, H, T, B = 3, 5, 7, 2
    rng = np.random.default_rng(2)
    x = rng.uniform(-1, 1, (T, B, I)).astype(np.float32)
    h0 = rng.uniform(-1, 1, (1, B, H))
    c0 = rng.uniform(-1, 1, (1, B, H))
    # LSTM, W = 0, b = 0: every sigmoid is 1/2 and g = 0, so c_T = c_0 / 2^T, h_T = tanh(c_T)/2
    W = [np.zeros((4 * H, I + H), np.float32)]
    hseq, hT, cT = oracle.rnn_forward(0, W, None, x, I, H, h0=h0, c0=c0)
    assert np.allclose(cT, c0 / 2.0 ** T, rtol=1e-15, atol=0)
    assert np.allclose(hT, 0.5 * np.tanh(c0 / 2.0 ** T), rtol=1e-15, atol=0)
    assert np.allclose(hseq[0], 0.5 * np.tanh(c0[0] / 2.0), rtol=1e-15, atol=0)
    # GRU, W = 0, b = 0: z = 1/2, n = 0, so h_T = h_0 / 2^T
    W = [np.zeros((3 * H, I + H), np.float32)]
    _, hT, _ = oracle.rnn_forward(1, W, None, x, I, H, h0=h0)
    assert np.allclose(hT, h0 / 2.0 ** T, rtol=1e-15, atol=0)


def test_bias_only_closed_form():
    """W = 0 with a bias: one LSTM step from zero state gives
    c_1 = sig(b_i) tanh(b_g), h_1 = sig(b_o) tanh(c_1) -- fixes the gate row order."""
    I, H = 2, 3
    b = np.array([0.1, 0.2, 0.3, 5, 5, 5, -0.4, 0.5, 0.6, 1.0, -1.0, 0.0], np.float32)  # i | f | g | o
    x = np.zeros((1, 1, I), np.float32)
    _, hT, cT = oracle.rnn_forward(0, [np.zeros((4 * H, I + H), np.float32)], [b], x, I, H)
    sig = lambda v: 1 / (1 + np.exp(-v))
    bd = b.astype(np.float64)
    c1 = sig(bd[0:3]) * np.tanh(bd[6:9])
    assert np.allclose(cT[0, 0], c1, rtol=1e-15)
    assert np.allclose(hT[0, 0], sig(bd[9:12]) * np.tanh(c1), rtol=1e-15)
    # GRU from zero state: h_1 = (1 - sig(b_z)) tanh(b_n)
    bg = np.array([0.3, -0.2, 0.1, 0.7, 0.0, -0.7, 0.4, 0.5, -0.6], np.float32)       # r | z | n
    _, hT, _ = oracle.rnn_forward(1, [np.zeros((3 * H, I + H), np.float32)], [bg], x, I, H)
    bgd = bg.astype(np.float64)
    assert np.allclose(hT[0, 0], (1 - sig(bgd[3:6])) * np.tanh(bgd[6:9]), rtol=1e-15)


@pytest.mark.parametrize("cell", [0, 1])
def test_single_step_is_matvec_plus_gates(cell):
    wl = _small(cell, 1, 6, 8, 1, 1, seed=5)
    I, H = 6, 8
    A = wl.W[0].A
    rng = np.random.default_rng(3)
    h0 = rng.uniform(-1, 1, (1, 1, H))
    c0 = rng.uniform(-1, 1, (1, 1, H))
    _, hT, cT = oracle.rnn_forward(cell, [A], wl.bias, wl.x, I, H, h0=h0, c0=c0)
    sig = lambda v: 1 / (1 + np.exp(-v))
    b = wl.bias[0].astype(np.float64)
    Ad = A.astype(np.float64)
    xv = wl.x[0, 0].astype(np.float64)
    if cell == 0:
        # h0 is float64 here, so form the product in numpy rather than through matvec (float32 x)
        a = Ad @ np.concatenate([xv, h0[0, 0]]) + b
        c1 = sig(a[H:2 * H]) * c0[0, 0] + sig(a[:H]) * np.tanh(a[2 * H:3 * H])
        assert np.allclose(cT[0, 0], c1, rtol=1e-13)
        assert np.allclose(hT[0, 0], sig(a[3 * H:]) * np.tanh(c1), rtol=1e-13)
    else:
        ax = Ad[:, :I] @ xv
        ah = Ad[:, I:] @ h0[0, 0]
        r = sig(ax[:H] + ah[:H] + b[:H])
        z = sig(ax[H:2 * H] + ah[H:2 * H] + b[H:2 * H])
        n = np.tanh(ax[2 * H:] + b[2 * H:] + r * ah[2 * H:])
        assert np.allclose(hT[0, 0], (1 - z) * n + z * h0[0, 0], rtol=1e-13)


@pytest.mark.parametrize("cell", [0, 1])
def test_resume_and_layer_composition(cell):
    L, I, H, T, B = 2, 6, 8, 10, 2
    wl = _small(cell, L, I, H, T, B, seed=9)
    W = [m.A for m in wl.W]
    hseq, hT, cT = oracle.rnn_forward(cell, W, wl.bias, wl.x, I, H)
    # forward(T) == forward(T1) then forward(T2) from the carried state, bit for bit
    s1, h1, c1 = oracle.rnn_forward(cell, W, wl.bias, wl.x[:4], I, H)
    s2, h2, c2 = oracle.rnn_forward(cell, W, wl.bias, wl.x[4:], I, H, h0=h1, c0=c1)
    assert np.array_equal(np.concatenate([s1, s2]), hseq)
    assert np.array_equal(h2, hT) and np.array_equal(c2, cT)
    # two layers == layer 1 over the whole sequence, then layer 2 over its outputs
    # (float32 hand-over would round, so feed layer 2 through torch-free float64 path:
    # compare against layer-wise runs only to float32 rounding of the hand-over)
    q1, qh1, qc1 = oracle.rnn_forward(cell, W[:1], wl.bias[:1], wl.x, I, H)
    q2, qh2, qc2 = oracle.rnn_forward(cell, W[1:], wl.bias[1:], q1.astype(np.float32), H, H)
    assert np.array_equal(qh1[0], hT[0])
    assert np.allclose(q2, hseq, rtol=0, atol=5e-6)


# ---- LSTM with a recurrent projection (the paper's SR1 cell, Table 1) -----------------------

def _torch_lstmp(W, Wp, bias, x, I, H, P, h0, c0):
    """torch.nn.LSTM with proj_size, CPU, float64: weight_ih|weight_hh = W split at the input
    width, weight_hr = the projection, bias_ih = b, bias_hh = 0."""
    L = len(W)
    mod = torch.nn.LSTM(I, H, num_layers=L, bias=True, proj_size=P).double()
    with torch.no_grad():
        for l in range(L):
            n_in = I if l == 0 else P
            getattr(mod, f"weight_ih_l{l}").copy_(torch.from_numpy(W[l][:, :n_in].astype(np.float64)))
            getattr(mod, f"weight_hh_l{l}").copy_(torch.from_numpy(W[l][:, n_in:].astype(np.float64)))
            getattr(mod, f"weight_hr_l{l}").copy_(torch.from_numpy(Wp[l].astype(np.float64)))
            getattr(mod, f"bias_ih_l{l}").copy_(torch.from_numpy(bias[l].astype(np.float64)))
            getattr(mod, f"bias_hh_l{l}").zero_()
        out, (hT, cT) = mod(torch.from_numpy(x.astype(np.float64)), (torch.from_numpy(h0), torch.from_numpy(c0)))
    return out.numpy(), hT.numpy(), cT.numpy()


@pytest.mark.parametrize("L,I,H,P,T,B", [(1, 5, 8, 3, 6, 1), (2, 12, 16, 8, 9, 3), (3, 7, 12, 11, 4, 2), (2, 9, 16, 4, 5, 2)])
def test_lstmp_against_torch_float64(L, I, H, P, T, B):
    wl = csb_inputs.make_lstmp(31 + L, L, I, H, P, 4, 2.0, T, B, sigma=0.3)
    W, Wp = [m.A for m in wl.W], [m.A for m in wl.Wp]
    rng = np.random.default_rng(2)
    h0 = rng.uniform(-0.5, 0.5, (L, B, P))
    c0 = rng.uniform(-0.5, 0.5, (L, B, H))
    hseq, hT, cT = oracle.lstmp_forward(W, Wp, wl.bias, wl.x, I, H, P, h0=h0, c0=c0)
    rseq, rhT, rcT = _torch_lstmp(W, Wp, wl.bias, wl.x, I, H, P, h0, c0)
    assert np.allclose(hseq, rseq, rtol=0, atol=1e-12)
    assert np.allclose(hT, rhT, rtol=0, atol=1e-12)
    assert np.allclose(cT, rcT, rtol=0, atol=1e-12)


def test_lstmp_with_identity_projection_is_the_lstm():
    """P = H and Wp = I: the projected cell is the plain LSTM the other tests pin."""
    L, I, H, T, B = 2, 6, 8, 7, 2
    wl = _small(csb_inputs.LSTM, L, I, H, T, B, seed=5)
    W = [m.A for m in wl.W]
    eye = [np.eye(H, dtype=np.float32)] * L
    a = oracle.lstmp_forward(W, eye, wl.bias, wl.x, I, H, H)
    b = oracle.rnn_forward(csb_inputs.LSTM, W, wl.bias, wl.x, I, H)
    for u, v in zip(a, b):
        assert np.allclose(u, v, rtol=0, atol=1e-13)      # the two add bias and partial sums in different orders


def test_lstmp_zero_gate_weights_closed_form():
    """W = 0, b = 0: every gate is 1/2, g = 0, so c_t = c_0 / 2^t and r_t = Wp (tanh(c_t) / 2)."""
    I, H, P, T = 3, 5, 4, 6
    rng = np.random.default_rng(3)
    Wp = rng.normal(0, 1, (P, H)).astype(np.float32)
    c0 = rng.uniform(-1, 1, (1, 1, H))
    x = rng.uniform(-1, 1, (T, 1, I)).astype(np.float32)
    hseq, hT, cT = oracle.lstmp_forward([np.zeros((4 * H, I + P), np.float32)], [Wp], None, x, I, H, P, c0=c0)
    for t in range(T):
        ct = c0[0, 0] / 2.0 ** (t + 1)
        assert np.allclose(hseq[t, 0], Wp.astype(np.float64) @ (0.5 * np.tanh(ct)), rtol=0, atol=1e-14)
    assert np.allclose(cT[0, 0], c0[0, 0] / 2.0 ** T, rtol=0, atol=1e-15)

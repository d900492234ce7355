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


# ---------------------------------------------------------------- Li-GRU (cell 3, SR3 rows of Table 1)

def _torch_relu_rnn(Wc, bc, x, I, H, h0):
    """torch.nn.RNN(nonlinearity='relu'), CPU, float64: h' = relu(W_ih x + W_hh h + b)."""
    mod = torch.nn.RNN(I, H, num_layers=1, nonlinearity="relu", bias=True).double()
    with torch.no_grad():
        mod.weight_ih_l0.copy_(torch.from_numpy(Wc[:, :I].astype(np.float64)))
        mod.weight_hh_l0.copy_(torch.from_numpy(Wc[:, I:].astype(np.float64)))
        mod.bias_ih_l0.copy_(torch.from_numpy(bc.astype(np.float64)))
        mod.bias_hh_l0.zero_()
        out, hT = mod(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(h0))
    return out.numpy(), hT.numpy()


def test_ligru_with_closed_update_gate_is_the_relu_rnn():
    """Update gate forced to 0 (bias -800: the sigmoid is exactly 0 in float64): h' is the
    candidate alone, which is torch's ReLU RNN -- pins the candidate rows, their operand
    order, the ReLU and that (1 - z) multiplies the candidate."""
    I, H, T, B = 6, 9, 7, 2
    wl = _small(csb_inputs.LIGRU, 1, I, H, T, B, seed=5)
    W = wl.W[0].A.copy()
    W[:H] = 0.0
    b = wl.bias[0].copy()
    b[:H] = -800.0
    h0 = np.random.default_rng(2).uniform(0.0, 0.5, (1, B, H))
    hseq, hT, _ = oracle.rnn_forward(csb_inputs.LIGRU, [W], [b], wl.x, I, H, h0=h0)
    rseq, rhT = _torch_relu_rnn(W[H:], b[H:], wl.x, I, H, h0)
    assert np.abs(rseq).max() > 0.05                       # the ReLU is not idle
    assert np.allclose(hseq, rseq, rtol=0, atol=1e-13) and np.allclose(hT, rhT, rtol=0, atol=1e-13)


def test_ligru_closed_forms():
    I, H, T = 4, 6, 5
    x = np.random.default_rng(0).uniform(-1, 1, (T, 1, I)).astype(np.float32)
    h0 = np.linspace(-1.0, 1.0, H).reshape(1, 1, H)
    # W = 0, b = 0: z = 1/2, candidate 0 -> h halves every step
    W0 = np.zeros((2 * H, I + H), np.float32)
    _, hT, _ = oracle.rnn_forward(csb_inputs.LIGRU, [W0], None, x, I, H, h0=h0)
    assert np.allclose(hT, h0 / 2.0 ** T, rtol=0, atol=1e-15)
    # update gate open (bias +40: the sigmoid rounds to 1): h stays what it was
    b = np.zeros(2 * H, np.float32); b[:H] = 40.0; b[H:] = 3.0
    _, hT, _ = oracle.rnn_forward(csb_inputs.LIGRU, [W0], [b], x, I, H, h0=h0)
    assert np.array_equal(hT, h0)
    # W = 0, z = 1/2, candidate = relu(b_c): h_T = h0 / 2^T + relu(b_c) (1 - 2^-T); negative b_c: no push
    b = np.zeros(2 * H, np.float32); b[H:] = np.linspace(-1.0, 1.5, H).astype(np.float32)
    _, hT, _ = oracle.rnn_forward(csb_inputs.LIGRU, [W0], [b], x, I, H, h0=h0)
    want = h0 / 2.0 ** T + np.maximum(b[H:].astype(np.float64), 0.0) * (1.0 - 2.0 ** -T)
    assert np.allclose(hT, want, rtol=0, atol=1e-15)


def test_ligru_scalar_unit_by_hand():
    """One unit, one input: the recurrence written out with Python floats."""
    import math
    wzx, wzh, wcx, wch, bz, bc = 0.7, -1.3, 0.9, 0.5, 0.1, -0.2
    W = np.array([[wzx, wzh], [wcx, wch]], np.float32)
    b = np.array([bz, bc], np.float32)
    x = np.array([0.5, -1.0, 2.0, 0.25], np.float32).reshape(4, 1, 1)
    h = 0.3
    hs = []
    for t in range(4):
        xt = float(x[t, 0, 0])
        z = 1.0 / (1.0 + math.exp(-(float(W[0, 0]) * xt + float(W[0, 1]) * h + float(b[0]))))
        cand = max(float(W[1, 0]) * xt + float(W[1, 1]) * h + float(b[1]), 0.0)
        h = z * h + (1.0 - z) * cand
        hs.append(h)
    hseq, hT, _ = oracle.rnn_forward(csb_inputs.LIGRU, [W], [b], x, 1, 1, h0=np.array([[[0.3]]]))
    assert np.allclose(hseq.ravel(), hs, rtol=0, atol=1e-15)


def test_ligru_layers_compose_and_resume():
    wl = _small(csb_inputs.LIGRU, 2, 5, 8, 6, 2, seed=8)
    W = [m.A for m in wl.W]
    hseq, hT, _ = oracle.rnn_forward(csb_inputs.LIGRU, W, wl.bias, wl.x, 5, 8)
    s1, h1, _ = oracle.rnn_forward(csb_inputs.LIGRU, W[:1], wl.bias[:1], wl.x, 5, 8)
    s2, h2, _ = oracle.rnn_forward(csb_inputs.LIGRU, W[1:], wl.bias[1:], s1.astype(np.float32), 8, 8)
    # (the second layer reads float32 inputs through this interface: compare loosely)
    assert np.allclose(hseq, s2, rtol=0, atol=1e-6)
    a, ha, _ = oracle.rnn_forward(csb_inputs.LIGRU, W, wl.bias, wl.x[:4], 5, 8)
    b, hb, _ = oracle.rnn_forward(csb_inputs.LIGRU, W, wl.bias, wl.x[4:], 5, 8, h0=ha)
    assert np.array_equal(np.concatenate([a, b]), hseq) and np.array_equal(hb, hT)


# ---------------------------------------------------------------- GRU, reset gate before the product (cell 4)

def test_gru_rb_with_open_reset_gate_is_torch_gru():
    """Reset gate forced to 1 (bias +40): r * (U h) = U (r * h), so both GRU forms agree and
    torch.nn.GRU pins everything but the place of the reset gate."""
    L, I, H, T, B = 2, 7, 10, 6, 2
    wl = _small(csb_inputs.GRU_RB, L, I, H, T, B, seed=21)
    W = [m.A.copy() for m in wl.W]
    bias = [b.copy() for b in wl.bias]
    for l in range(L):
        W[l][:H] = 0.0
        bias[l][:H] = 40.0
    h0 = np.random.default_rng(3).uniform(-0.5, 0.5, (L, B, H))
    hseq, hT, _ = oracle.rnn_forward(csb_inputs.GRU_RB, W, bias, wl.x, I, H, h0=h0)
    rseq, rhT, _ = _torch_ref(1, W, bias, wl.x, I, H, h0)
    assert np.allclose(hseq, rseq, rtol=0, atol=1e-12) and np.allclose(hT, rhT, rtol=0, atol=1e-12)


def test_gru_rb_one_unit_is_torch_gru():
    """With one hidden unit r (u h) = u (r h): the two forms coincide, reset gate live."""
    I, H, T, B = 3, 1, 8, 2
    rng = np.random.default_rng(4)
    W = rng.normal(0, 1.0, (3, I + 1)).astype(np.float32)
    b = rng.normal(0, 0.5, 3).astype(np.float32)
    x = rng.uniform(-1, 1, (T, B, I)).astype(np.float32)
    h0 = rng.uniform(-0.9, 0.9, (1, B, 1))
    hseq, hT, _ = oracle.rnn_forward(csb_inputs.GRU_RB, [W], [b], x, I, H, h0=h0)
    rseq, rhT, _ = _torch_ref(1, [W], [b], x, I, H, h0)
    assert np.allclose(hseq, rseq, rtol=0, atol=1e-13)


def test_gru_rb_place_of_the_reset_gate_by_brute_force():
    """Tiny case in exact rational-free Python floats, straight from the definition:
    n = tanh(Wn x + Un (r * h) + bn).  Also checks that it is NOT the reset-after result."""
    import math
    I, H, T = 2, 3, 4
    rng = np.random.default_rng(6)
    W = rng.normal(0, 0.8, (3 * H, I + H)).astype(np.float32)
    b = rng.normal(0, 0.3, 3 * H).astype(np.float32)
    x = rng.uniform(-1, 1, (T, 1, I)).astype(np.float32)
    h = [0.4, -0.6, 0.2]
    sig = lambda v: 1.0 / (1.0 + math.exp(-v))
    Wd, bd = W.astype(np.float64), b.astype(np.float64)
    for t in range(T):
        xt = [float(v) for v in x[t, 0]]
        pre = lambda row, hv: sum(Wd[row, j] * xt[j] for j in range(I)) + sum(Wd[row, I + j] * hv[j] for j in range(H)) + bd[row]
        r = [sig(pre(k, h)) for k in range(H)]
        z = [sig(pre(H + k, h)) for k in range(H)]
        q = [r[k] * h[k] for k in range(H)]
        n = [math.tanh(pre(2 * H + k, q)) for k in range(H)]
        h = [(1.0 - z[k]) * n[k] + z[k] * h[k] for k in range(H)]
    h0 = np.array([[[0.4, -0.6, 0.2]]])
    _, hT, _ = oracle.rnn_forward(csb_inputs.GRU_RB, [W], [b], x, I, H, h0=h0)
    assert np.allclose(hT.ravel(), h, rtol=0, atol=1e-14)
    _, hA, _ = oracle.rnn_forward(csb_inputs.GRU, [W], [b], x, I, H, h0=h0)
    assert np.abs(hA - hT).max() > 1e-3


def test_gru_rb_zero_weights_closed_form():
    I, H, T = 3, 5, 6
    x = np.zeros((T, 1, I), np.float32)
    h0 = np.linspace(-1, 1, H).reshape(1, 1, H)
    _, hT, _ = oracle.rnn_forward(csb_inputs.GRU_RB, [np.zeros((3 * H, I + H), np.float32)], None, x, I, H, h0=h0)
    assert np.allclose(hT, h0 / 2.0 ** T, rtol=0, atol=1e-15)

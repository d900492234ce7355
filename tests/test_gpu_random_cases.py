"""Seeded random cases for every device entry point, against the oracle: shapes, block sizes
(powers of two and not, 1 to 256), pruning rates (dense to empty), chunk counts, weight
formats, batch sizes, cells, layer counts and paths are drawn together, so that combinations
no hand-written case lists come up.  Bars as in the per-entry-point tests: the float32
dot-product bound for the products, 1e-4 on the states, bit-exact for the projection."""
import sys

import numpy as np
import pytest
import torch

import csb_inputs
import oracle
import paper_2005_05758_amd as P
from paper_2005_05758_amd import CsbMatrix, CsbRnn
from paper_2005_05758_amd.binding import project

pytestmark = pytest.mark.gpu

BLOCKS = [1, 2, 3, 5, 8, 16, 17, 32, 33, 64, 100, 128, 255, 256]
FORMATS = [(P.VAL_F32, None), (P.VAL_F16, "f16"), (P.VAL_BF16, "bf16")]


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dot_bound(D, scale):
    k = np.count_nonzero(D, axis=1)
    k = k[:, None] if scale.ndim == 2 else k
    return 2.0 * np.maximum(k, 1) * 2.0 ** -24 * scale + 1e-30


@pytest.mark.parametrize("group", range(6))
def test_random_products(group):
    for tr in range(group * 40, group * 40 + 40):
        rng = np.random.default_rng(tr)
        big = rng.random() < 0.15
        rows, cols = (int(rng.integers(1, 2500 if big else 400)) for _ in range(2))
        br, bc = int(rng.choice(BLOCKS)), int(rng.choice(BLOCKS))
        rate = float(rng.choice([1.0, 1.5, 4.0, 10.0, 40.0, 0.0]))
        law = str(rng.choice(["binomial", "beta"]))
        n_chunks = int(rng.choice([0, 0, 1, 2, 3, 7, 64, 300]))
        mode = int(rng.choice([0, 0, 2]))
        fmt, fname = FORMATS[int(rng.choice([0, 0, 1, 2]))]
        batch = int(rng.choice([1, 2, 3, 4, 8, 16, 17, 20, 32, 48, 64, 68, 100, 128]))
        say(f"[random products] case {tr}: {rows}x{cols} block {br}x{bc} rate {rate} {law} chunks {n_chunks} "
            f"mode {mode} format {fmt} batch {batch}")
        if rate == 0.0:                                   # empty, or a handful of lone survivors
            A = np.zeros((rows, cols), np.float32)
            for _ in range(int(rng.integers(0, 4))):
                A[int(rng.integers(0, rows)), int(rng.integers(0, cols))] = float(rng.normal())
        else:
            A = csb_inputs.small_matrix(tr, rows, cols, br, bc, rate=rate, law=law).A
        M = CsbMatrix(A, br, bc)
        if fmt != P.VAL_F32:
            M.set_value_format(fmt)
        M.plan(n_chunks, mode)
        M.validate()
        M.upload()
        D = oracle.csb_decode(oracle.csb_encode(A, br, bc))
        if fname:
            D = oracle.round_weights(D, fname)
        x = csb_inputs.make_vectors(tr, cols, 1)
        y = M.spmv(torch.from_numpy(x).cuda())
        torch.cuda.synchronize()
        ref = oracle.matvec(D, x)
        assert np.all(np.abs(y.cpu().numpy().astype(np.float64) - ref) <= dot_bound(D, oracle.matvec_abs(D, x)))
        X = np.ascontiguousarray(csb_inputs.make_vectors(tr + 1, cols, max(batch, 2))[:, :batch])
        Y = M.spmm(torch.from_numpy(X).cuda())
        torch.cuda.synchronize()
        ref = oracle.matmat(D, X)
        got = Y.cpu().numpy().astype(np.float64)
        assert got.shape == ref.shape
        assert np.all(np.abs(got - ref) <= dot_bound(D, oracle.matmat(np.abs(D), np.abs(X))))
        if fmt == P.VAL_BF16 and batch % 4 == 0:          # bfloat16 right-hand sides too, on the bf16 matrix cores
            Xq = oracle.round_weights(X, "bf16").astype(np.float32)
            try:
                Yb = M.spmm_bfloat(torch.from_numpy(Xq).cuda().to(torch.bfloat16))
            except P.CsbError:
                assert br > 64                             # refused only when the accumulator tiles do not fit
            else:
                torch.cuda.synchronize()
                ref = oracle.matmat(D, Xq)
                assert np.all(np.abs(Yb.cpu().numpy().astype(np.float64) - ref) <= dot_bound(D, oracle.matmat(np.abs(D), np.abs(Xq))))
        M.close()


@pytest.mark.parametrize("group", range(5))
def test_random_recurrent_models(group):
    for tr in range(group * 16, group * 16 + 16):
        rng = np.random.default_rng(10_000 + tr)
        kind = str(rng.choice(["lstm", "gru", "ligru", "gru_rb", "lstmp"]))
        L = int(rng.choice([1, 1, 2, 3]))
        big = rng.random() < 0.2
        I, H = int(rng.integers(1, 600 if big else 120)), int(rng.integers(1, 700 if big else 150))
        block = int(rng.choice([4, 8, 16, 32, 64]))
        rate = float(rng.choice([1.5, 3.0, 8.0, 16.0]))
        T = int(rng.choice([0, 1, 2, 5, 17, 40]))
        B = int(rng.choice([1, 1, 1, 2, 5, 16, 33, 64]))
        want_resident = bool(rng.random() < 0.7)
        with_state = bool(rng.random() < 0.5)
        sigma = min(0.3, 1.2 / np.sqrt(I + H))            # keeps the unbounded Li-GRU state tame
        proj = int(rng.integers(1, H + 1))
        hs = proj if kind == "lstmp" else H
        h0 = rng.uniform(-0.5, 0.5, size=(L, B, hs)).astype(np.float32) if with_state else None
        c0 = (rng.uniform(-0.5, 0.5, size=(L, B, H)).astype(np.float32)
              if with_state and kind in ("lstm", "lstmp") else None)
        fmt, fname = FORMATS[int(rng.integers(0, 3))] if kind in ("lstm", "gru", "ligru") else FORMATS[0]   # (drawn last)
        if kind == "lstmp":
            wl = csb_inputs.make_lstmp(tr, L, I, H, proj, block, rate, T, B, sigma=sigma)
            bias = [torch.from_numpy(b).cuda() for b in wl.bias]
            Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
            Ps = [CsbMatrix(m.A, m.br, m.bc) for m in wl.Wp]
            rnn, mats = CsbRnn(P.CELL_LSTMP, I, H, Ws, bias, proj=proj, Wp=Ps), Ws + Ps
            rseq, rhT, rcT = oracle.lstmp_forward([m.A for m in wl.W], [m.A for m in wl.Wp], wl.bias, wl.x, I, H, proj,
                                                  h0=h0, c0=c0)
        else:
            cell = {"lstm": P.CELL_LSTM, "gru": P.CELL_GRU, "ligru": P.CELL_LIGRU, "gru_rb": P.CELL_GRU_RB}[kind]
            wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", cell, L, I, H, block, rate, "binomial", sigma, B, T, tr))
            bias = [torch.from_numpy(b).cuda() for b in wl.bias]
            if kind == "gru_rb":
                parts = [csb_inputs.split_gru_rb(m.A, I if l == 0 else H, H) for l, m in enumerate(wl.W)]
                Was = [CsbMatrix(p[0], block, block) for p in parts]
                Uns = [CsbMatrix(p[1], block, block) for p in parts]
                rnn, mats = CsbRnn(P.CELL_GRU_RB, I, H, Was, bias, Wp=Uns), Was + Uns
            else:
                mats = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
                for m in mats:
                    if fname:
                        m.set_value_format(fmt)                  # before the handle is created over it
                rnn = CsbRnn(cell, I, H, mats, bias)
            Wref = [oracle.round_weights(m.A, fname) if fname else m.A for m in wl.W]
            rseq, rhT, rcT = oracle.rnn_forward(cell, Wref, wl.bias, wl.x, I, H, h0=h0, c0=c0)
        # (a batch on the resident kernel in every second case that asks for the resident layout)
        resident = (B == 1 or tr % 2 == 0) and want_resident and rnn.stats()["resident"] == 1
        say(f"[random models] case {tr}: {kind} L={L} I={I} H={H} proj={proj if kind == 'lstmp' else 0} block={block} "
            f"rate={rate} T={T} B={B} resident={resident} state={with_state} values={fname or 'f32'}")
        if resident:
            rnn.upload()
        else:
            for m in mats:
                m.validate()
                m.upload()
        hseq, hT, cT = rnn.forward(torch.from_numpy(wl.x).cuda(), None if h0 is None else torch.from_numpy(h0).cuda(),
                                   None if c0 is None else torch.from_numpy(c0).cuda())
        torch.cuda.synchronize()
        scale = max(1.0, float(np.max(np.abs(rseq))) if T else 1.0)
        assert scale < 50.0
        if T:
            assert float(np.max(np.abs(hseq.cpu().numpy() - rseq))) <= 1e-4 * scale
        assert float(np.max(np.abs(hT.cpu().numpy() - rhT))) <= 1e-4 * scale
        if cT is not None:
            assert float(np.max(np.abs(cT.cpu().numpy() - rcT))) <= 1e-4 * max(scale, float(np.max(np.abs(rcT))))
        rnn.close()
        for m in mats:
            m.close()


def test_random_projections():
    for tr in range(200):
        rng = np.random.default_rng(20_000 + tr)
        big = rng.random() < 0.1
        rows, cols = (int(rng.integers(1, 3000 if big else 500)) for _ in range(2))
        br, bc = int(rng.choice(BLOCKS)), int(rng.choice(BLOCKS))
        rate = float(rng.choice([1.0, 1.3, 2.0, 4.0, 10.0, 16.0, 100.0, 1e6]))
        style = str(rng.choice(["normal", "ties", "sparse", "strided"]))
        whole = rng.random() < 0.4                        # whole blocks, rows in eights: the 16-byte forms of the kernels
        if whole:
            cols, rows = max(bc, cols // bc * bc), max(8, rows // 8 * 8)
        pad = 8 if whole and rng.random() < 0.5 else 5    # (a row stride that keeps, or breaks, the alignment)
        say(f"[random projections] case {tr}: {rows}x{cols} block {br}x{bc} rate {rate} {style} pad {pad}")
        W = rng.normal(size=(rows, cols)).astype(np.float32)
        if style == "ties":
            W = np.round(W).astype(np.float32)            # many equal segment sums
        if style == "sparse":
            W[rng.random(W.shape) < 0.8] = 0.0
        ref = oracle.csb_project(W, br, bc, rate).astype(np.float32)
        if style == "strided":
            buf = torch.zeros((rows, cols + pad), dtype=torch.float32, device="cuda")
            buf[:, :cols] = torch.from_numpy(W).cuda()
            got = project(buf[:, :cols], br, bc, rate)
        else:
            got = project(torch.from_numpy(W).cuda(), br, bc, rate)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy().view(np.uint32), ref.view(np.uint32))

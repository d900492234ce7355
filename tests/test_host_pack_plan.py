"""Host logic of the library against the oracle: csb_pack bit-exact, plan self-check,
error returns, exported symbols.  No GPU needed (no compute entry point is called)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import csb_inputs
import oracle
from paper_2005_05758_amd import CsbMatrix, CsbError, binding
from helpers import read_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _same_encoding(M, enc):
    v = M.view()
    for k in ("nrows", "ncols", "rowidx", "colidx", "val_off", "row_off", "col_off"):
        assert np.array_equal(v[k], getattr(enc, k)), k
    assert np.array_equal(v["val"].view(np.uint32), enc.val.view(np.uint32))
    assert v["nnz"] == enc.nnz
    return v


def test_library_exports_every_declared_symbol():
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = sorted(set(re.findall(r"\b(csb_[a-z_]+)\s*\(", hdr)))
    assert declared, "no declarations found"
    L = binding.load_library()
    for name in declared:
        assert hasattr(L, name), name
    assert sorted(binding.SYMBOLS) == declared


def test_pack_hand_worked_example():
    g = read_golden("two_block_example.txt")
    A = np.array(g["A"], np.float32)
    v = CsbMatrix(A, 4, 4).view()
    assert v["nrows"].tolist() == g["nrows_a"] and v["ncols"].tolist() == g["ncols_a"]
    assert v["rowidx"].tolist() == g["rowidx_a"] and v["colidx"].tolist() == g["colidx_a"]
    assert v["val"].tolist() == g["val_a"]
    assert v["val_off"].tolist() == g["val_off"] and v["row_off"].tolist() == g["row_off"]
    assert v["col_off"].tolist() == g["col_off"]


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3"])
def test_pack_bit_exact_on_workloads(name):
    cfg = csb_inputs.CONFIGS[name]
    for m in csb_inputs.make_rnn(cfg, T=1).W:
        M = CsbMatrix(m.A, m.br, m.bc)
        _same_encoding(M, oracle.csb_encode(m.A, m.br, m.bc))
        assert np.array_equal(M.unpack().view(np.uint32), m.A.view(np.uint32))


@pytest.mark.parametrize("R,C,br,bc", [(7, 5, 3, 2), (12, 12, 5, 5), (1, 1, 1, 1), (33, 70, 32, 32),
                                      (300, 17, 256, 16), (64, 64, 64, 64), (5, 300, 2, 256)])
def test_pack_ragged_and_degenerate(R, C, br, bc):
    for seed in range(3):
        rng = np.random.default_rng(seed * 7 + R + C)
        A = rng.normal(size=(R, C)).astype(np.float32)
        A[rng.random((R, C)) < (0.0, 0.7, 1.0)[seed]] = 0.0        # dense, sparse, all zero
        M = CsbMatrix(A, br, bc)
        _same_encoding(M, oracle.csb_encode(A, br, bc))
        assert np.array_equal(M.unpack(), A)
        M.plan()
        M.validate()


def test_pack_special_values_and_leading_dimension():
    A = np.zeros((4, 6), np.float32)
    A[0, 0] = -0.0
    A[1, 2] = np.nan
    A[3, 5] = np.inf
    M = CsbMatrix(A, 2, 2)
    enc = oracle.csb_encode(A, 2, 2)
    v = M.view()
    assert np.array_equal(v["nrows"], enc.nrows) and np.array_equal(v["colidx"], enc.colidx)
    assert np.array_equal(v["val"].view(np.uint32), enc.val.view(np.uint32))
    # ld > cols: pack a window of a wider array
    wide = np.arange(40, dtype=np.float32).reshape(4, 10)
    Mw = CsbMatrix(wide[:, :6].copy(), 2, 4)
    h = C.c_void_p()
    L = binding.lib()
    assert L.csb_pack(wide.ctypes.data, 4, 6, 10, 2, 4, C.byref(h)) == 0
    out = np.empty((4, 6), np.float32)
    assert L.csb_unpack(h, out.ctypes.data, 6) == 0
    assert np.array_equal(out, wide[:, :6]) and np.array_equal(Mw.unpack(), out)
    L.csb_free(h)


def test_error_returns():
    L = binding.lib()
    A = np.ones((4, 4), np.float32)
    h = C.c_void_p()
    assert L.csb_pack(None, 4, 4, 4, 2, 2, C.byref(h)) == -1
    assert L.csb_pack(A.ctypes.data, 4, 4, 4, 2, 2, None) == -1
    assert L.csb_pack(A.ctypes.data, 0, 4, 4, 2, 2, C.byref(h)) == -1
    assert L.csb_pack(A.ctypes.data, 4, -1, 4, 2, 2, C.byref(h)) == -1
    assert L.csb_pack(A.ctypes.data, 4, 4, 3, 2, 2, C.byref(h)) == -1
    assert L.csb_pack(A.ctypes.data, 4, 4, 4, 0, 2, C.byref(h)) == -1
    assert L.csb_pack(A.ctypes.data, 4, 4, 4, 2, 257, C.byref(h)) == -1
    assert b"block size" in L.csb_last_error()
    assert L.csb_pack(A.ctypes.data, 4, 4, 4, 2, 2, C.byref(h)) == 0
    # order of calls: nothing device-side before plan + upload
    assert L.csb_device_bytes(h) == 0
    assert L.csb_plan_validate(h) == -5
    assert L.csb_upload(h, 256, 1 << 20, None) == -5
    assert L.csb_spmv(h, 256, 256, None, None) == -5
    assert L.csb_plan(h, -1, None) == -1
    assert L.csb_plan(h, 0, None) == 0
    assert L.csb_device_bytes(h) > 0
    assert L.csb_upload(h, None, 1 << 20, None) == -1
    assert L.csb_upload(h, 256, 16, None) == -2          # undersized device buffer
    assert L.csb_upload(h, 257, 1 << 20, None) == -1      # misaligned
    assert L.csb_spmv(h, None, 256, None, None) == -1
    assert L.csb_spmv(h, 256, 256, None, None) == -5      # planned but not uploaded
    assert L.csb_view_get(None, None) == -1 and L.csb_unpack(h, None, 4) == -1
    r = C.c_void_p()
    Wp = (C.c_void_p * 1)(h)
    assert L.csb_rnn_create(0, 1, 2, 2, Wp, None, C.byref(r)) == -1      # 4x4 is not (4*2) x (2+2)
    assert L.csb_rnn_create(7, 1, 2, 1, Wp, None, C.byref(r)) == -1      # unknown cell
    assert L.csb_rnn_create(0, 0, 2, 1, Wp, None, C.byref(r)) == -1
    assert L.csb_rnn_create(0, 1, 3, 1, Wp, None, C.byref(r)) == 0       # (4*1) x (3+1)
    assert L.csb_rnn_forward(r, None, None, None, None, None, None, 1, 1, None, None) == -1
    assert L.csb_rnn_forward(r, 256, None, None, None, 256, None, -1, 1, 256, None) == -1
    assert L.csb_rnn_forward(r, 256, None, None, None, 256, None, 1, 0, 256, None) == -1
    assert L.csb_rnn_forward(r, 256, None, None, None, 256, None, 1, 1, 256, None) == -5   # not uploaded
    assert L.csb_rnn_forward(r, 256, None, None, None, 256, None, 1, 1, 264, None) == -1   # misaligned workspace
    assert b"aligned" in L.csb_last_error()
    # the projection checks its arguments before anything touches a device
    assert L.csb_project(256, 8, 8, 8, 2, 2, C.c_double(4.0), 256, 8, 264, None) == -1
    assert b"aligned" in L.csb_last_error()
    assert L.csb_project(256, 8, 8, 4, 2, 2, C.c_double(4.0), 256, 8, 256, None) == -1     # ld below cols
    assert L.csb_project(256, 8, 8, 8, 2, 2, C.c_double(0.5), 256, 8, 256, None) == -1     # rate below 1
    assert L.csb_project(256, 20000, 8, 8, 2, 2, C.c_double(4.0), 256, 8, 256, None) == -4 # more rows than one workgroup ranks
    L.csb_rnn_free(r)
    L.csb_free(h)
    L.csb_free(None)
    L.csb_rnn_free(None)


@pytest.mark.parametrize("name,n_chunks", [("cfg1", 0), ("cfg2", 0), ("cfg2", 37), ("cfg3", 0), ("cfg3", 64)])
def test_plan_partition_invariants(name, n_chunks):
    cfg = csb_inputs.CONFIGS[name]
    m = csb_inputs.make_rnn(cfg, T=1).W[0]
    M = CsbMatrix(m.A, m.br, m.bc)
    st = M.plan(n_chunks)
    M.validate()         # every value referenced exactly once, all offsets in bounds, decodes back
    assert st["n_chunks"] >= max(n_chunks, 1)
    assert st["work_max"] >= st["work_mean"] > 0
    assert 0 < st["lane_fill"] <= 1.0


def test_plan_balance_on_skewed_matrix():
    """The load-balance workload (kept fraction per block Beta-distributed): with shares of
    about 50 steps the largest wavefront share stays within 12 % of the mean (a share ends
    where the rest of it would not cover another group's fixed cost, so shares differ by up
    to that cost), where dealing whole blocks out without splitting is far off (the analogue
    of the no-sharing case of Sec. 6.3.2)."""
    m = csb_inputs.make_rnn(csb_inputs.CONFIGS["cfg3"], T=1).W[0]
    M = CsbMatrix(m.A, m.br, m.bc)
    st = M.plan(4, 2)
    assert st["work_mean"] >= 40
    assert st["work_max"] / st["work_mean"] <= 1.12
    assert st["nosplit_max_over_mean"] > 1.2


def test_plan_validate_sweep_small_shapes():
    """Many small shapes, laws, chunk counts and both cut modes: every image the planner
    emits must pass the host-side walk that mirrors the kernels (bounds, padding, coverage)."""
    shapes = [(48, 48, 16, 16), (160, 200, 32, 32), (70, 130, 8, 64), (300, 257, 64, 16), (33, 1000, 32, 128)]
    for seed in range(6):
        for (r, c, br, bc) in shapes:
            for law, rate in (("beta", 5.0), ("heavy", 10.0), ("binomial", 3.0)):
                m = csb_inputs.small_matrix(seed, r, c, br, bc, rate=rate, law=law)
                M = CsbMatrix(m.A, br, bc)
                for nch in (0, 1, 7, 50):
                    for mode in (0, 2):
                        M.plan(nch, mode)
                        M.validate()
    M = CsbMatrix(np.eye(48, dtype=np.float32), 16, 16)
    M.plan(0)
    M.validate()


def test_plan_rejects_inputs_wider_than_the_offset_lists():
    """Input offsets are 16-bit byte offsets into the staged vector (plus a zero word behind
    it): 16383 columns plan, 16384 do not."""
    A = np.zeros((8, 16384), np.float32)
    A[3, 100] = 1.0
    A[5, 16383] = 2.0
    M = CsbMatrix(A, 8, 64)
    with pytest.raises(CsbError) as e:
        M.plan(0)
    assert e.value.code == -4 and "columns" in str(e.value)
    M = CsbMatrix(np.ascontiguousarray(A[:, :16383]), 8, 64)
    M.plan(0)
    M.validate()


# ---------------------------------------------------------------- 16-bit value formats (host side)

@pytest.mark.parametrize("fmt,name", [(binding.VAL_F16, "f16"), (binding.VAL_BF16, "bf16")])
def test_value_format_rounds_like_the_oracle_bit_for_bit(fmt, name):
    rng = np.random.default_rng(0)
    pm = csb_inputs.small_matrix(3, 70, 90, 16, 16, rate=3.0)
    A = pm.A.copy()
    nz = np.flatnonzero(A)
    # spread the magnitudes: ties, subnormals of binary16, overflow
    A.flat[nz[:40]] = np.float32(1.0) + np.arange(40, dtype=np.float32) * np.float32(2.0 ** -12)
    A.flat[nz[40:60]] = rng.uniform(-1e-7, 1e-7, 20).astype(np.float32)
    A.flat[nz[60:64]] = np.array([65519.0, 65520.0, -1e5, 3.4e38], np.float32)
    M = CsbMatrix(A, 16, 16)
    enc = oracle.csb_encode(A, 16, 16)
    assert M.value_format() == binding.VAL_F32
    M.set_value_format(fmt)
    assert M.value_format() == fmt
    v = M.view()
    want = oracle.round_weights(enc.val, name)
    assert np.array_equal(v["val"].view(np.uint32), want.view(np.uint32))
    for k in ("nrows", "ncols", "rowidx", "colidx"):                 # the pattern is untouched (zeros stay stored)
        assert np.array_equal(v[k], getattr(enc, k))
    assert np.array_equal(M.unpack().view(np.uint32) & 0x7FFFFFFF, oracle.round_weights(A, name).view(np.uint32) & 0x7FFFFFFF)
    M.set_value_format(fmt)                                          # idempotent
    assert np.array_equal(M.view()["val"].view(np.uint32), want.view(np.uint32))


def test_value_format_halves_the_value_stream_and_validates():
    pm = csb_inputs.small_matrix(5, 300, 500, 32, 32, rate=4.0)
    M = CsbMatrix(pm.A, 32, 32)
    M.plan()
    M.validate()
    n32 = M.device_bytes()
    nnz = int(M.view()["nnz"])
    for fmt in (binding.VAL_F16, binding.VAL_BF16):
        M.set_value_format(fmt)
        with pytest.raises(CsbError):
            M.validate()                                             # the old plan is gone
        M.plan()
        M.validate()
        assert n32 - M.device_bytes() >= 2 * nnz * 0.9               # 2 of 4 bytes per stored value
    M.set_value_format(binding.VAL_F32)
    M.plan()
    M.validate()
    assert M.device_bytes() == n32
    with pytest.raises(CsbError):
        M.set_value_format(7)


def test_value_format_plan_sweep():
    for seed, (R, Cc, br, bc) in enumerate([(5, 7, 4, 4), (64, 64, 8, 16), (100, 130, 32, 32), (257, 63, 64, 16), (40, 600, 16, 32)]):
        pm = csb_inputs.small_matrix(seed, R, Cc, br, bc, rate=2.5)
        for fmt in (binding.VAL_F16, binding.VAL_BF16):
            M = CsbMatrix(pm.A, br, bc)
            M.set_value_format(fmt)
            for n_chunks in (0, 1, 3):
                M.plan(n_chunks)
                M.validate()


def test_resident_layout_limits():
    """csb_rnn_create is host work: a model whose stage inputs are wider than a workgroup can
    stage gets no resident layout (and still has the streaming paths); a small one gets it."""
    from paper_2005_05758_amd import CsbRnn, CELL_LSTM, CELL_GRU_RB
    wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", csb_inputs.LSTM, 1, 2100, 1000, 50, 40.0, "binomial", 0.05, 1, 1, 0))
    rnn = CsbRnn(CELL_LSTM, 2100, 1000, [CsbMatrix(wl.W[0].A, 50, 50)], None)       # 2100 + 1000 > 3072
    assert rnn.stats()["resident"] == 0 and rnn.device_bytes() == 0
    wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", csb_inputs.LSTM, 1, 1500, 1500, 50, 40.0, "binomial", 0.05, 1, 1, 0))
    rnn = CsbRnn(CELL_LSTM, 1500, 1500, [CsbMatrix(wl.W[0].A, 50, 50)], None)       # 3000: three entries per thread
    assert rnn.stats()["resident"] == 1
    wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", csb_inputs.GRU_RB, 2, 24, 64, 8, 4.0, "binomial", 0.1, 1, 1, 0))
    Was, Uns = [], []
    for l, m in enumerate(wl.W):
        Wa, Un = csb_inputs.split_gru_rb(m.A, 24 if l == 0 else 64, 64)
        Was.append(CsbMatrix(Wa, 8, 8)); Uns.append(CsbMatrix(Un, 8, 8))
    rnn = CsbRnn(CELL_GRU_RB, 24, 64, Was, None, Wp=Uns)
    st = rnn.stats()
    assert st["resident"] == 1 and st["n_workgroups"] >= 4                      # two stages per layer
    # the resident kernel takes the bias pointers of at most 8 layers: a deeper stack streams
    for L, want in ((8, 1), (9, 0)):
        wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", csb_inputs.LSTM, L, 6, 8, 4, 2.0, "binomial", 0.1, 1, 1, 0))
        rnn = CsbRnn(CELL_LSTM, 6, 8, [CsbMatrix(m.A, 4, 4) for m in wl.W], None)
        assert rnn.stats()["resident"] == want


def test_resident_layout_for_batches():
    """csb_rnn_plan_resident is host work: for a batch it trades slots per lane for smaller
    instances (the headline model: 20 workgroups at 8 slots fill an XCD alone; laid out for a
    batch of 64 several instances share one), batch 1 gives the layout of create back, and a
    model without a resident layout is refused."""
    from paper_2005_05758_amd import CsbRnn, CsbError, CELL_LSTM
    cfg = csb_inputs.CONFIGS["cfg2"]
    wl = csb_inputs.make_rnn(cfg, T=1)
    rnn = CsbRnn(CELL_LSTM, cfg.input, cfg.hidden, [CsbMatrix(m.A, m.br, m.bc) for m in wl.W], None)
    one = rnn.stats()
    bytes_one = rnn.device_bytes()
    rnn.plan_resident(64)
    many = rnn.stats()
    assert many["resident"] == 1 and many["slots_per_lane"] > one["slots_per_lane"]
    assert many["n_workgroups"] <= 14 < one["n_workgroups"]
    assert rnn.device_bytes() > 0
    rnn.plan_resident(1)
    assert rnn.stats() == one and rnn.device_bytes() == bytes_one
    with pytest.raises(CsbError):
        rnn.plan_resident(0)
    wl = csb_inputs.make_rnn(csb_inputs.RnnConfig("t", csb_inputs.LSTM, 1, 2100, 1000, 50, 40.0, "binomial", 0.05, 1, 1, 0))
    big = CsbRnn(CELL_LSTM, 2100, 1000, [CsbMatrix(wl.W[0].A, 50, 50)], None)
    with pytest.raises(CsbError):
        big.plan_resident(8)


def test_gru_matrix_keeps_its_row_layout_when_planned_again():
    """A matrix planned by csb_rnn_create for a GRU keeps the layout in which the n rows'
    input-side and recurrent-side sums stay apart when csb_plan / csb_plan_ex plan it again,
    also after csb_set_value_format; csb_rnn_create keeps the workgroup count and mode of an
    earlier plan of the caller's.  (No device needed: csb_spmv refuses such a matrix before it
    touches anything.)"""
    import ctypes as C
    from paper_2005_05758_amd.binding import CsbError, CsbRnn, CELL_GRU, lib
    cfg = csb_inputs.CONFIGS["cfg3"]
    wl = csb_inputs.make_rnn(cfg, T=2)
    m = wl.W[0]
    M = CsbMatrix(m.A, m.br, m.bc)
    M.plan(7, 2)                                  # the caller's choice: 7 workgroups, equal split
    rnn = CsbRnn(CELL_GRU, cfg.input, cfg.hidden, [M], None)
    st = M.plan_stats()                           # csb_rnn_create planned again, for the GRU, with the caller's parameters

    def refused_as_gru():
        rc = lib().csb_spmv(M.handle, C.c_void_p(256), C.c_void_p(256), None, None)
        return rc == -5 and b"GRU" in lib().csb_last_error()

    assert refused_as_gru()
    assert M.plan(7, 2) == st                     # the same request on the GRU layout gives the same plan
    st_default = M.plan()
    assert st_default["n_chunks"] != st["n_chunks"] and refused_as_gru()     # other count, same row layout
    M.validate()
    M.set_value_format(binding.VAL_BF16)          # invalidates the plan
    M.plan()
    assert refused_as_gru()
    M.validate()
    del rnn


@pytest.mark.parametrize("name,limit", [("cfg5", 1.10), ("cfg5_diag", 1.10)])
def test_default_plan_balances_the_stress_matrices(name, limit):
    """The plan csb_spmv runs by default (row-owned layout): largest wavefront work over the mean
    stays within 10 % on the 8192^2 heavy-tailed matrices, and the bytes one launch reads stay
    within 15 % of the algorithmic bytes."""
    m = csb_inputs.make_mat(csb_inputs.CONFIGS[name])
    M = CsbMatrix(m.A, m.br, m.bc)
    st = M.plan()
    assert st["row_owned"] == 1 and st["n_chunks"] == 256
    assert st["work_max"] / st["work_mean"] <= limit, (st["work_max"], st["work_mean"])
    v = M.view()
    alg = 4 * int(v["nnz"]) + len(v["rowidx"]) + len(v["colidx"]) + 2 * int(v["nbr"]) * int(v["nbc"]) + 4 * int(v["cols"]) + 4 * int(v["rows"])
    assert st["matvec_bytes"] <= 1.15 * alg
    M.validate()


def test_small_matrix_plans_trade_balance_for_short_wavefronts():
    """On the RNN matrices a wavefront holds one or two groups, and a group costs a fixed amount
    whatever its width, so the ratio largest / mean cannot be small AND the wavefronts short; the
    default takes short wavefronts (more workgroups).  With half as many workgroups the same
    matrix balances within 10 %, and the largest wavefront's work is then at least as large."""
    m = csb_inputs.make_rnn(csb_inputs.CONFIGS["cfg3"], T=1).W[0]
    M = CsbMatrix(m.A, m.br, m.bc)
    st = M.plan()
    assert st["row_owned"] == 1
    M2 = CsbMatrix(m.A, m.br, m.bc)
    st2 = M2.plan_rows(max(1, (3 * st["n_chunks"]) // 4), 0)
    assert st2["work_max"] / st2["work_mean"] <= 1.10
    assert st2["work_max"] >= st["work_max"]
    M.validate(); M2.validate()


def test_plan_rows_sweep():
    """csb_plan_rows on small shapes: every workgroup count and round count asked for gives a
    section the validator decodes back to the matrix, in all three value formats; the statistics
    describe that section; a workgroup never owns more than 256 rows."""
    shapes = [(4, 8, 4, 4, 2.0), (1, 1, 1, 1, 1.0), (37, 53, 8, 8, 3.0), (200, 150, 16, 16, 6.0), (130, 257, 32, 32, 5.0),
              (70, 300, 16, 64, 4.0), (300, 40, 128, 8, 3.0), (513, 100, 256, 256, 2.0), (64, 64, 64, 64, 1.0), (1030, 96, 32, 32, 3.0)]
    for (R, C, br, bc, rate) in shapes:
        A = csb_inputs.small_matrix(R * 3 + C, R, C, br, bc, rate=rate).A
        for fmt in (binding.VAL_F32, binding.VAL_F16, binding.VAL_BF16):
            for n_wg in (0, 1, 3):
                for rounds in (0, 2, 5):
                    M = CsbMatrix(A, br, bc)
                    if fmt != binding.VAL_F32:
                        M.set_value_format(fmt)
                    st = M.plan_rows(n_wg, rounds)
                    assert st["row_owned"] == 1 and st["rounds"] >= max(1, rounds)
                    assert st["n_chunks"] >= max(1, -(-R // 256)) and st["n_chunks"] >= min(max(n_wg, 1), R) or n_wg == 0
                    assert st["work_max"] >= st["work_mean"] > 0 or int(M.view()["nnz"]) == 0
                    assert st["matvec_bytes"] > 0 and st == M.plan_stats()
                    M.validate()
    Z = CsbMatrix(np.zeros((40, 48), np.float32), 16, 16)
    assert Z.plan_rows(0, 0)["row_owned"] == 1
    Z.validate()


@pytest.mark.parametrize("I,H,block,layers", [(40, 100, 32, 1), (5, 7, 4, 2), (33, 50, 16, 2), (64, 96, 32, 1), (30, 300, 32, 2)])
def test_gru_step_matrices_get_the_row_owned_layout(I, H, block, layers):
    """A GRU handle plans its matrices with the row split of its step (the candidate's rows once
    over the input columns and once, H rows further down, over the recurrent ones).  The
    row-owned section holds that split as well -- also where the split column falls inside a
    block column -- and decodes to the relabelled matrix (csb_plan_validate)."""
    from paper_2005_05758_amd import CsbRnn
    cfg = csb_inputs.RnnConfig("t", csb_inputs.GRU, layers, I, H, block, 3.0, "binomial", 0.3, 1, 2, 11)
    wl = csb_inputs.make_rnn(cfg)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, None)
    for w in Ws:
        st = w.plan_stats()
        assert st["row_owned"] == 2, st                             # workgroups own whole units
        w.validate()
    del rnn


@pytest.mark.parametrize("cell,I,H,block,layers", [
    (csb_inputs.LSTM, 20, 48, 16, 2), (csb_inputs.GRU, 33, 64, 32, 3), (csb_inputs.LIGRU, 7, 40, 8, 2),
    (csb_inputs.LSTM, 5, 2048, 64, 1), (csb_inputs.LSTM, 64, 300, 16, 2), (csb_inputs.GRU, 12, 96, 32, 1)])
def test_rnn_handles_get_plans_whose_workgroups_own_whole_units(cell, I, H, block, layers):
    """csb_rnn_create lays its matrices out so that a workgroup
    owns units with all their gate rows (the streaming step then finishes its cells in the
    product's launch): the section decodes to the matrix (csb_plan_validate walks it with the
    unit-to-row mapping), and a plan the caller makes afterwards owns plain row ranges again."""
    from paper_2005_05758_amd import CsbRnn
    cfg = csb_inputs.RnnConfig("t", cell, layers, I, H, block, 4.0, "binomial", 0.3, 1, 2, 5)
    wl = csb_inputs.make_rnn(cfg)
    Ws = [CsbMatrix(m.A, m.br, m.bc) for m in wl.W]
    rnn = CsbRnn(cfg.cell, cfg.input, cfg.hidden, Ws, None)
    for w in Ws:
        st = w.plan_stats()
        assert st["row_owned"] == 2, st
        w.validate()
    if cell != csb_inputs.GRU:              # (a GRU's matrices keep their row split, and with it the handle's layout rules)
        st = Ws[0].plan()
        assert st["row_owned"] == 1
        Ws[0].validate()
    del rnn

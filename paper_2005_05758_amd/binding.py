"""ctypes binding with the same names as include/csbrnn.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

CELL_LSTM = 0
CELL_GRU = 1
CELL_LSTMP = 2
CELL_LIGRU = 3
CELL_GRU_RB = 4
VAL_F32, VAL_F16, VAL_BF16 = 0, 1, 2

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libcsbrnn.so")
_lib = None

# every symbol include/csbrnn.h declares
SYMBOLS = ["csb_last_error", "csb_pack", "csb_view_get", "csb_unpack", "csb_set_value_format", "csb_value_format", "csb_sharing_model", "csb_plan", "csb_plan_ex", "csb_plan_rows", "csb_plan_stats_get", "csb_plan_validate", "csb_status",
           "csb_device_bytes", "csb_upload", "csb_workspace_bytes", "csb_spmv", "csb_spmv_static_limit", "csb_spmv_static", "csb_spmm", "csb_spmm_bfloat", "csb_spmm_half",
           "csb_debug_stamp_count", "csb_debug_spmv_stamps",
           "csb_debug_stream_read_out_floats", "csb_debug_stream_read",
           "csb_project_workspace_bytes", "csb_project", "csb_rnn_create_lstmp", "csb_rnn_create_gru_rb",
           "csb_rnn_create", "csb_rnn_device_bytes", "csb_rnn_upload", "csb_rnn_plan_resident", "csb_rnn_stats",
           "csb_rnn_set_poll_limit", "csb_rnn_status", "csb_rnn_workspace_bytes", "csb_rnn_forward", "csb_free", "csb_rnn_free"]


class csb_sharing_stats(C.Structure):
    _fields_ = [("work", C.c_int64), ("iterations", C.c_int64), ("cycles_none", C.c_int64),
                ("cycles_horizontal", C.c_int64), ("cycles_vertical", C.c_int64), ("cycles_2d", C.c_int64),
                ("eff_none", C.c_double), ("eff_horizontal", C.c_double), ("eff_vertical", C.c_double),
                ("eff_2d", C.c_double), ("exact_2d", C.c_int32), ("reserved", C.c_int32)]


class CsbError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"csb error {code}: {msg}")
        self.code = code


class csb_view(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64),
                ("br", C.c_int32), ("bc", C.c_int32), ("nbr", C.c_int32), ("nbc", C.c_int32),
                ("nnz", C.c_int64), ("n_rowidx", C.c_int64), ("n_colidx", C.c_int64),
                ("nrows", C.POINTER(C.c_int32)), ("ncols", C.POINTER(C.c_int32)),
                ("rowidx", C.POINTER(C.c_uint16)), ("colidx", C.POINTER(C.c_uint16)),
                ("val", C.POINTER(C.c_float)),
                ("val_off", C.POINTER(C.c_int64)), ("row_off", C.POINTER(C.c_int64)),
                ("col_off", C.POINTER(C.c_int64))]


class csb_rnn_plan_stats(C.Structure):
    _fields_ = [("resident", C.c_int32), ("n_workgroups", C.c_int32), ("slots_per_lane", C.c_int32),
                ("reserved", C.c_int32), ("slot_fill", C.c_double), ("lanes_max_over_mean", C.c_double)]


class csb_plan_stats(C.Structure):
    _fields_ = [("n_chunks", C.c_int32), ("waves_per_chunk", C.c_int32), ("n_groups", C.c_int32),
                ("n_shared_tiles", C.c_int32), ("work_max", C.c_double), ("work_mean", C.c_double),
                ("lane_fill", C.c_double), ("nosplit_max_over_mean", C.c_double),
                ("chunk_max_over_mean", C.c_double), ("whole_tiles", C.c_int32), ("row_owned", C.c_int32),
                ("rounds", C.c_int32), ("reserved", C.c_int32), ("matvec_bytes", C.c_int64)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libcsbrnn.so; fails loudly if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2005_05758_amd.build` "
                          "(there is no CPU fallback)")
    L = C.CDLL(_LIB_PATH)
    L.csb_last_error.restype = C.c_char_p
    L.csb_pack.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
    L.csb_view_get.argtypes = [C.c_void_p, C.POINTER(csb_view)]
    L.csb_unpack.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
    L.csb_sharing_model.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(csb_sharing_stats)]
    L.csb_set_value_format.argtypes = [C.c_void_p, C.c_int32]
    L.csb_value_format.argtypes = [C.c_void_p]
    L.csb_plan.argtypes = [C.c_void_p, C.c_int32, C.POINTER(csb_plan_stats)]
    L.csb_plan_ex.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(csb_plan_stats)]
    L.csb_plan_rows.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(csb_plan_stats)]
    L.csb_plan_stats_get.argtypes = [C.c_void_p, C.POINTER(csb_plan_stats)]
    L.csb_status.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
    L.csb_rnn_set_poll_limit.argtypes = [C.c_void_p, C.c_uint32]
    L.csb_rnn_status.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32)]
    L.csb_plan_validate.argtypes = [C.c_void_p]
    L.csb_device_bytes.argtypes = [C.c_void_p]
    L.csb_device_bytes.restype = C.c_size_t
    L.csb_upload.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.csb_workspace_bytes.argtypes = [C.c_void_p, C.c_int32]
    L.csb_workspace_bytes.restype = C.c_size_t
    L.csb_spmv.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.csb_spmv_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    L.csb_spmv_static_limit.argtypes = []
    L.csb_spmv_static_limit.restype = C.c_size_t
    L.csb_debug_stamp_count.argtypes = [C.c_void_p]
    L.csb_debug_stamp_count.restype = C.c_size_t
    L.csb_debug_spmv_stamps.argtypes = [C.c_void_p] * 6
    L.csb_debug_stream_read_out_floats.argtypes = []
    L.csb_debug_stream_read_out_floats.restype = C.c_size_t
    L.csb_debug_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    L.csb_project_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int32, C.c_int32]
    L.csb_project_workspace_bytes.restype = C.c_size_t
    L.csb_project.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_double,
                              C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
    L.csb_spmm.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    L.csb_spmm_bfloat.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p]
    L.csb_spmm_half.argtypes = L.csb_spmm_bfloat.argtypes
    L.csb_rnn_create.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                 C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
    L.csb_rnn_create_lstmp.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                       C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
    L.csb_rnn_create_gru_rb.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_void_p),
                                        C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
    L.csb_rnn_device_bytes.argtypes = [C.c_void_p]
    L.csb_rnn_device_bytes.restype = C.c_size_t
    L.csb_rnn_upload.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.csb_rnn_plan_resident.argtypes = [C.c_void_p, C.c_int32]
    L.csb_rnn_stats.argtypes = [C.c_void_p, C.POINTER(csb_rnn_plan_stats)]
    L.csb_rnn_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    L.csb_rnn_workspace_bytes.restype = C.c_size_t
    L.csb_rnn_forward.argtypes = [C.c_void_p] + [C.c_void_p] * 6 + [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    L.csb_free.argtypes = [C.c_void_p]
    L.csb_free.restype = None
    L.csb_rnn_free.argtypes = [C.c_void_p]
    L.csb_rnn_free.restype = None
    for name in SYMBOLS:
        fn = getattr(L, name)
        if fn.restype is C.c_int and name not in ("csb_free", "csb_rnn_free"):
            fn.restype = C.c_int
    _lib = L
    return L


def lib():
    return load_library()


def _check(rc: int):
    if rc != 0:
        raise CsbError(rc, lib().csb_last_error().decode())


def _f32():
    import torch
    return torch.float32


def _dptr(t, dtype=None) -> Optional[int]:
    """Device pointer of a contiguous torch tensor (or None); `dtype`: what the callee reads it as."""
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    if dtype is not None:
        assert t.dtype == dtype, f"expected a {dtype} tensor, got {t.dtype}"
    return t.data_ptr()


def _stream_ptr(stream=None) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def stream_read(buf, out=None, stream=None):
    """csb_debug_stream_read on a device tensor (any dtype, size a multiple of 16 bytes)."""
    import torch
    n = int(lib().csb_debug_stream_read_out_floats())
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=buf.device)
    assert out.numel() >= n and buf.is_contiguous()
    _check(lib().csb_debug_stream_read(_dptr(buf), buf.numel() * buf.element_size(), _dptr(out), _stream_ptr(stream)))
    return out


def project(W, br: int, bc: int, rate: float, out=None, stream=None):
    """csb_project on a device tensor W [rows][cols] (float32, rows may be strided): returns the
    pruned matrix (a new tensor, or `out`, which may be W itself)."""
    import torch
    assert W.dim() == 2 and W.dtype == torch.float32 and W.stride(1) == 1
    rows, cols = W.shape
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=W.device)
    assert out.shape == W.shape and out.dtype == torch.float32 and out.stride(1) == 1
    nb = int(lib().csb_project_workspace_bytes(rows, cols, br, bc))
    ws = torch.empty(max(nb, 256), dtype=torch.uint8, device=W.device)
    _check(lib().csb_project(W.data_ptr(), rows, cols, W.stride(0), br, bc, float(rate), out.data_ptr(), out.stride(0),
                             _dptr(ws), _stream_ptr(stream)))
    return out


class CsbMatrix:
    """Owns one csb_matrix handle and (optionally) the torch buffer holding its device image."""

    def __init__(self, dense: np.ndarray, br: int, bc: int, ld: Optional[int] = None):
        dense = np.ascontiguousarray(dense, dtype=np.float32)
        rows, cols = dense.shape
        self._h = C.c_void_p()
        _check(lib().csb_pack(dense.ctypes.data, rows, cols, cols if ld is None else ld, br, bc, C.byref(self._h)))
        self.rows, self.cols, self.br, self.bc = rows, cols, br, bc
        self.d_buf = None
        self.d_ws = None
        self.stats = None

    @property
    def handle(self):
        return self._h

    def view(self):
        v = csb_view()
        _check(lib().csb_view_get(self._h, C.byref(v)))
        nb = v.nbr * v.nbc

        def arr(p, n, dt):
            return np.ctypeslib.as_array(p, shape=(n,)).astype(dt, copy=True) if n else np.zeros(0, dt)
        return dict(rows=v.rows, cols=v.cols, br=v.br, bc=v.bc, nbr=v.nbr, nbc=v.nbc, nnz=v.nnz,
                    nrows=arr(v.nrows, nb, np.int32), ncols=arr(v.ncols, nb, np.int32),
                    rowidx=arr(v.rowidx, v.n_rowidx, np.uint16), colidx=arr(v.colidx, v.n_colidx, np.uint16),
                    val=arr(v.val, v.nnz, np.float32),
                    val_off=arr(v.val_off, nb + 1, np.int64), row_off=arr(v.row_off, nb + 1, np.int64),
                    col_off=arr(v.col_off, nb + 1, np.int64))

    def unpack(self) -> np.ndarray:
        out = np.empty((self.rows, self.cols), np.float32)
        _check(lib().csb_unpack(self._h, out.ctypes.data, self.cols))
        return out

    def sharing_model(self, P: int = 4, Q: int = 4, K: int = 4, L: int = 4) -> dict:
        """csb_sharing_model: PE utilisation of the paper's own engine schedule on this matrix."""
        st = csb_sharing_stats()
        _check(lib().csb_sharing_model(self._h, P, Q, K, L, C.byref(st)))
        return {k: getattr(st, k) for k, _ in csb_sharing_stats._fields_}

    def set_value_format(self, fmt: int):
        """csb_set_value_format: VAL_F32 / VAL_F16 / VAL_BF16; plan and upload again afterwards."""
        _check(lib().csb_set_value_format(self._h, fmt))
        self.d_buf = None
        return self

    def value_format(self) -> int:
        return int(lib().csb_value_format(self._h))

    def plan(self, n_chunks: int = 0, mode: int = 0):
        st = csb_plan_stats()
        _check(lib().csb_plan_ex(self._h, n_chunks, mode, C.byref(st)))
        self.stats = {k: getattr(st, k) for k, _ in csb_plan_stats._fields_}
        return self.stats

    def plan_rows(self, n_workgroups: int = 0, min_rounds: int = 0):
        """csb_plan_rows: the row-owned mat-vec layout with its parameters spelled out."""
        st = csb_plan_stats()
        _check(lib().csb_plan_rows(self._h, n_workgroups, min_rounds, C.byref(st)))
        self.stats = {k: getattr(st, k) for k, _ in csb_plan_stats._fields_}
        self.d_buf = None
        return self.stats

    def plan_stats(self):
        """csb_plan_stats_get: the statistics of the current plan."""
        st = csb_plan_stats()
        _check(lib().csb_plan_stats_get(self._h, C.byref(st)))
        return {k: getattr(st, k) for k, _ in csb_plan_stats._fields_}

    def status(self, stream=None) -> int:
        """csb_status: non-zero if a merge of shared row tiles gave up since the last check."""
        v = C.c_int32(0)
        _check(lib().csb_status(self._h, _stream_ptr(stream), C.byref(v)))
        return int(v.value)

    def validate(self):
        _check(lib().csb_plan_validate(self._h))

    def device_bytes(self) -> int:
        return int(lib().csb_device_bytes(self._h))

    def workspace_bytes(self, batch: int = 1) -> int:
        return int(lib().csb_workspace_bytes(self._h, batch))

    def upload(self, device="cuda", stream=None):
        """Allocate the image buffer with torch and copy the planned image into it."""
        import torch
        n = self.device_bytes()
        self.d_buf = torch.empty(n + 256, dtype=torch.uint8, device=device)
        base = self.d_buf.data_ptr()
        self._d_ptr = (base + 255) // 256 * 256
        _check(lib().csb_upload(self._h, self._d_ptr, n, _stream_ptr(stream)))
        return self

    def spmv(self, x, y=None, stream=None):
        import torch
        if y is None:
            y = torch.empty(self.rows, dtype=torch.float32, device=x.device)
        ws = self._workspace(1, x.device)
        _check(lib().csb_spmv(self._h, _dptr(x, _f32()), _dptr(y, _f32()), _dptr(ws), _stream_ptr(stream)))
        return y

    def spmv_static(self, x, y=None, stream=None):
        """csb_spmv_static: csb_spmv with the library's built-in buffer in place of a workspace."""
        import torch
        if y is None:
            y = torch.empty(self.rows, dtype=torch.float32, device=x.device)
        _check(lib().csb_spmv_static(self._h, _dptr(x, _f32()), _dptr(y, _f32()), _stream_ptr(stream)))
        return y

    def spmv_stamps(self, x, y=None, stream=None):
        """csb_debug_spmv_stamps: returns (y, stamps).  Row-owned layout: int64 [n_workgroups, 16, 8]
        (per wavefront: start, vector staged, first unit landed, same, groups done, after the
        barrier, end; 100 MHz clock).  Tile-based layout: [n_chunks, 8 + 3*16] shader clocks."""
        import torch
        if y is None:
            y = torch.empty(self.rows, dtype=torch.float32, device=x.device)
        n = int(lib().csb_debug_stamp_count(self._h))
        st = torch.zeros(n, dtype=torch.int64, device=x.device)
        ws = self._workspace(1, x.device)
        _check(lib().csb_debug_spmv_stamps(self._h, _dptr(x, _f32()), _dptr(y, _f32()), _dptr(ws), _dptr(st), _stream_ptr(stream)))
        if getattr(self, "stats", None) and self.stats.get("row_owned") == 1:
            return y, st.view(-1, 16, 8)
        return y, st.view(-1, 8 + 3 * 16)

    def spmm(self, X, Y=None, stream=None):
        import torch
        cols, batch = X.shape
        if Y is None:
            Y = torch.empty((self.rows, batch), dtype=torch.float32, device=X.device)
        ws = self._workspace(batch, X.device)
        # rows may be strided views ([cols][ldx], [rows][ldy]); the batch index must be contiguous
        assert X.is_cuda and Y.is_cuda and X.stride(1) == 1 and Y.stride(1) == 1
        assert X.dtype == torch.float32 and Y.dtype == torch.float32
        _check(lib().csb_spmm(self._h, X.data_ptr(), X.stride(0), Y.data_ptr(), Y.stride(0), batch, _dptr(ws),
                              _stream_ptr(stream)))
        return Y

    def spmm_bfloat(self, Xb, Y=None, stream=None):
        """Xb: [cols, batch] torch.bfloat16 cuda (rows may be strided, the batch contiguous)."""
        import torch
        cols, batch = Xb.shape
        if Y is None:
            Y = torch.empty((self.rows, batch), dtype=torch.float32, device=Xb.device)
        assert Xb.is_cuda and Y.is_cuda and Xb.dtype == torch.bfloat16 and Xb.stride(1) == 1 and Y.stride(1) == 1
        _check(lib().csb_spmm_bfloat(self._h, Xb.data_ptr(), Xb.stride(0), Y.data_ptr(), Y.stride(0), batch,
                                   _stream_ptr(stream)))
        return Y

    def spmm_half(self, Xh, Y=None, stream=None):
        """Xh: [cols, batch] torch.float16 cuda (rows may be strided, the batch contiguous)."""
        import torch
        cols, batch = Xh.shape
        if Y is None:
            Y = torch.empty((self.rows, batch), dtype=torch.float32, device=Xh.device)
        assert Xh.is_cuda and Y.is_cuda and Xh.dtype == torch.float16 and Xh.stride(1) == 1 and Y.stride(1) == 1
        _check(lib().csb_spmm_half(self._h, Xh.data_ptr(), Xh.stride(0), Y.data_ptr(), Y.stride(0), batch,
                                   _stream_ptr(stream)))
        return Y

    def _workspace(self, batch, device):
        import torch
        need = self.workspace_bytes(batch)
        if need == 0:
            return None
        if self.d_ws is None or self.d_ws.numel() * 4 < need:
            self.d_ws = torch.empty((need + 3) // 4, dtype=torch.float32, device=device)
        return self.d_ws

    def close(self):
        if self._h:
            lib().csb_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class CsbRnn:
    """csb_rnn handle; keeps its matrices and bias tensors alive."""

    def __init__(self, cell: int, input: int, hidden: int, W: Sequence[CsbMatrix], bias=None,
                 proj: int = 0, Wp: Optional[Sequence[CsbMatrix]] = None):
        """cell CELL_LSTM / CELL_GRU / CELL_LIGRU: csb_rnn_create.  cell CELL_LSTMP:
        csb_rnn_create_lstmp with the projection width `proj` and the projection matrices `Wp`.
        cell CELL_GRU_RB: csb_rnn_create_gru_rb, `W` = the Wa matrices, `Wp` = the Un matrices."""
        self.cell, self.input, self.hidden, self.W = cell, input, hidden, list(W)
        self.proj, self.Wp = proj, (list(Wp) if Wp is not None else [])
        self.bias = list(bias) if bias is not None else None
        L = len(self.W)
        Wv = (C.c_void_p * L)(*[w.handle for w in self.W])
        Bp = None
        if self.bias is not None:
            Bp = (C.c_void_p * L)(*[_dptr(b, _f32()) for b in self.bias])
        self._h = C.c_void_p()
        if cell == CELL_LSTMP:
            assert proj > 0 and len(self.Wp) == L
            Pv = (C.c_void_p * L)(*[w.handle for w in self.Wp])
            _check(lib().csb_rnn_create_lstmp(L, input, hidden, proj, Wv, Pv, Bp, C.byref(self._h)))
        elif cell == CELL_GRU_RB:
            assert len(self.Wp) == L
            Pv = (C.c_void_p * L)(*[w.handle for w in self.Wp])
            _check(lib().csb_rnn_create_gru_rb(L, input, hidden, Wv, Pv, Bp, C.byref(self._h)))
        else:
            _check(lib().csb_rnn_create(cell, L, input, hidden, Wv, Bp, C.byref(self._h)))
        self.n_layers = L
        self._ws = None

    def workspace_bytes(self, batch: int, T: int) -> int:
        return int(lib().csb_rnn_workspace_bytes(self._h, batch, T))

    def stats(self):
        st = csb_rnn_plan_stats()
        _check(lib().csb_rnn_stats(self._h, C.byref(st)))
        return {k: getattr(st, k) for k, _ in csb_rnn_plan_stats._fields_ if k != "reserved"}

    def device_bytes(self) -> int:
        return int(lib().csb_rnn_device_bytes(self._h))

    def set_poll_limit(self, polls: int):
        _check(lib().csb_rnn_set_poll_limit(self._h, polls))
        return self

    def status(self, stream=None) -> int:
        """csb_rnn_status: non-zero if a wait inside the resident kernel gave up since the last check."""
        v = C.c_int32(0)
        _check(lib().csb_rnn_status(self._h, _stream_ptr(stream), C.byref(v)))
        return int(v.value)

    def plan_resident(self, batch: int):
        """Lay the resident kernel out for batches of this size (1: one sequence, as created);
        upload() afterwards."""
        _check(lib().csb_rnn_plan_resident(self._h, batch))
        self._d_img = None
        return self

    def upload(self, device="cuda", stream=None):
        """Upload the resident layout; without it forward() streams the matrices."""
        import torch
        n = self.device_bytes()
        if n == 0:
            raise CsbError(-4, "model has no resident layout")
        self._d_img = torch.empty(n + 256, dtype=torch.uint8, device=device)
        ptr = (self._d_img.data_ptr() + 255) // 256 * 256
        _check(lib().csb_rnn_upload(self._h, ptr, n, _stream_ptr(stream)))
        return self

    def forward(self, x, h0=None, c0=None, want_hseq=True, stream=None):
        """x: [T, B, I] float32 cuda.  Returns (hseq or None, hT, cT or None)."""
        import torch
        T, B, I = x.shape
        dev = x.device
        need = self.workspace_bytes(B, T)
        if self._ws is None or self._ws.numel() * 4 < need:
            self._ws = torch.empty((need + 3) // 4 + 64, dtype=torch.float32, device=dev)
        hs = self.proj if self.cell == CELL_LSTMP else self.hidden        # width of the state h
        hseq = torch.empty((T, B, hs), dtype=torch.float32, device=dev) if want_hseq else None
        hT = torch.empty((self.n_layers, B, hs), dtype=torch.float32, device=dev)
        cT = (torch.empty((self.n_layers, B, self.hidden), dtype=torch.float32, device=dev)
              if self.cell in (CELL_LSTM, CELL_LSTMP) else None)
        _check(lib().csb_rnn_forward(self._h, _dptr(x, _f32()), _dptr(h0, _f32()), _dptr(c0, _f32()), _dptr(hseq, _f32()), _dptr(hT, _f32()), _dptr(cT, _f32()),
                                     T, B, _dptr(self._ws), _stream_ptr(stream)))
        return hseq, hT, cT

    def forward_into(self, x, h0, c0, hseq, hT, cT, stream=None):
        """csb_rnn_forward into the caller's output tensors (hseq, cT may be None)."""
        import torch
        T, B, I = x.shape
        need = self.workspace_bytes(B, T)
        if self._ws is None or self._ws.numel() * 4 < need:
            self._ws = torch.empty((need + 3) // 4 + 64, dtype=torch.float32, device=x.device)
        _check(lib().csb_rnn_forward(self._h, _dptr(x, _f32()), _dptr(h0, _f32()), _dptr(c0, _f32()), _dptr(hseq, _f32()), _dptr(hT, _f32()),
                                     _dptr(cT, _f32()), T, B, _dptr(self._ws), _stream_ptr(stream)))

    def close(self):
        if self._h:
            lib().csb_rnn_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

"""ctypes front end of the CPU oracle (oracle/csb_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by the smoke check and by the benchmark's
cpu_baseline leg; never by the product package.  The method's arithmetic (encode, decode,
products, cell updates, projection) is in the C file and this module marshals numpy arrays
for it.  Two things are computed here in numpy instead, each marked where it stands: the
PE-array utilisation model of Sec. 5 (`eff_1d`, `eff_2d`, integer counts only) and the
rounding of operands to 16-bit storage formats used by the reduced-precision parity cases.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csb_oracle.c")
_LIB = os.path.join(_HERE, "libcsb_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over output rows).  With
    CSB_ORACLE_SANITIZE=<path of a clang> in the environment it is compiled by that clang with
    AddressSanitizer and UndefinedBehaviorSanitizer instead (single-threaded, a library of its
    own name), for runs of the CPU test suite under the sanitizer runtime."""
    san = os.environ.get("CSB_ORACLE_SANITIZE")
    if san:
        lib = os.path.join(_HERE, "libcsb_oracle_sanitize.so")
        if force or not os.path.exists(lib) or os.path.getmtime(lib) < os.path.getmtime(_SRC):
            tmp = lib + f".tmp{os.getpid()}"
            subprocess.check_call([san, "-O1", "-g", "-std=c99", "-fPIC", "-shared", "-fsanitize=address,undefined",
                                   "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-shared-libsan",
                                   "-Wno-unknown-pragmas", "-o", tmp, _SRC, "-lm"])
            os.replace(tmp, lib)
        return lib
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
        _lib.orc_csb_encode.restype = C.c_int
        _lib.orc_csb_decode.restype = C.c_int
        _lib.orc_rnn_forward.restype = C.c_int
        _lib.orc_csb_project.restype = C.c_int
        _lib.orc_csb_project_f64.restype = C.c_int
        _lib.orc_lstmp_forward.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(_load().orc_num_threads())


def set_threads(n: int) -> None:
    _load().orc_set_threads(C.c_int(n))


class CsbArrays:
    """The five CSB arrays of Sec. 3.1.1 plus the derived exclusive prefix sums."""

    def __init__(self, rows, cols, br, bc, nrows, ncols, rowidx, colidx, val):
        self.rows, self.cols, self.br, self.bc = rows, cols, br, bc
        self.nbr, self.nbc = -(-rows // br), -(-cols // bc)
        self.nrows, self.ncols = nrows, ncols
        self.rowidx, self.colidx, self.val = rowidx, colidx, val
        self.nnz = int(val.shape[0])
        self.val_off = np.concatenate(([0], np.cumsum(nrows.astype(np.int64) * ncols.astype(np.int64))))
        self.row_off = np.concatenate(([0], np.cumsum(nrows.astype(np.int64))))
        self.col_off = np.concatenate(([0], np.cumsum(ncols.astype(np.int64))))


def csb_encode(A: np.ndarray, br: int, bc: int) -> CsbArrays:
    lib = _load()
    A = np.ascontiguousarray(A, dtype=np.float32)
    R, Cc = A.shape
    nb = (-(-R // br)) * (-(-Cc // bc))
    nrows = np.zeros(nb, np.int32)
    ncols = np.zeros(nb, np.int32)
    tot = (C.c_int64 * 3)()
    rc = lib.orc_csb_encode(_p(A), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), C.c_int32(br),
                            C.c_int32(bc), _p(nrows), _p(ncols), None, C.c_int64(0), None,
                            C.c_int64(0), None, C.c_int64(0), tot)
    if rc != 0:
        raise ValueError("orc_csb_encode(count) failed")
    nv, nr, nc = int(tot[0]), int(tot[1]), int(tot[2])
    rowidx = np.zeros(nr, np.uint16)
    colidx = np.zeros(nc, np.uint16)
    val = np.zeros(nv, np.float32)
    rc = lib.orc_csb_encode(_p(A), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), C.c_int32(br),
                            C.c_int32(bc), _p(nrows), _p(ncols), _p(rowidx), C.c_int64(nr),
                            _p(colidx), C.c_int64(nc), _p(val), C.c_int64(nv), tot)
    if rc != 0:
        raise ValueError("orc_csb_encode(fill) failed")
    return CsbArrays(R, Cc, br, bc, nrows, ncols, rowidx, colidx, val)


def csb_decode(m: CsbArrays) -> np.ndarray:
    lib = _load()
    A = np.empty((m.rows, m.cols), np.float32)
    rc = lib.orc_csb_decode(C.c_int64(m.rows), C.c_int64(m.cols), C.c_int32(m.br), C.c_int32(m.bc),
                            _p(m.nrows), _p(m.ncols), _p(m.rowidx), _p(m.colidx), _p(m.val),
                            _p(A), C.c_int64(m.cols))
    if rc != 0:
        raise ValueError("orc_csb_decode failed")
    return A


def matvec(A: np.ndarray, x: np.ndarray) -> np.ndarray:
    lib = _load()
    A = np.ascontiguousarray(A, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    R, Cc = A.shape
    assert x.shape == (Cc,)
    y = np.empty(R, np.float64)
    lib.orc_matvec(_p(A), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), _p(x), _p(y))
    return y


def csb_matvec_f32(m: CsbArrays, x: np.ndarray) -> np.ndarray:
    """CSB-MVM on the encoded arrays in float32 (Sec. 4.3.1): the like-for-like CPU baseline
    that the benchmark times; checked against `matvec`, never used as a parity reference."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.shape == (m.cols,)
    y = np.empty(m.rows, np.float32)
    vo, ro, co = (np.ascontiguousarray(a, dtype=np.int64) for a in (m.val_off, m.row_off, m.col_off))
    lib.orc_csb_matvec_f32(C.c_int64(m.rows), C.c_int64(m.cols), C.c_int32(m.br), C.c_int32(m.bc),
                           _p(m.nrows), _p(m.ncols), _p(m.rowidx), _p(m.colidx), _p(m.val),
                           _p(vo), _p(ro), _p(co), _p(x), _p(y))
    return y


def matvec_abs(A: np.ndarray, x: np.ndarray) -> np.ndarray:
    lib = _load()
    A = np.ascontiguousarray(A, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.float32)
    R, Cc = A.shape
    y = np.empty(R, np.float64)
    lib.orc_matvec_abs(_p(A), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), _p(x), _p(y))
    return y


def matmat(A: np.ndarray, X: np.ndarray) -> np.ndarray:
    """Y = A X with X of shape [C, B]."""
    lib = _load()
    A = np.ascontiguousarray(A, dtype=np.float32)
    X = np.ascontiguousarray(X, dtype=np.float32)
    R, Cc = A.shape
    assert X.shape[0] == Cc
    nb = X.shape[1]
    Y = np.empty((R, nb), np.float64)
    lib.orc_matmat(_p(A), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), _p(X), C.c_int64(nb),
                   _p(Y), C.c_int64(nb), C.c_int64(nb))
    return Y


def matmat_rows(A: np.ndarray, rows: Sequence[int], X: np.ndarray) -> np.ndarray:
    lib = _load()
    A = np.ascontiguousarray(A, dtype=np.float32)
    X = np.ascontiguousarray(X, dtype=np.float32)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    Cc = A.shape[1]
    nb = X.shape[1]
    Y = np.empty((rows.shape[0], nb), np.float64)
    lib.orc_matmat_rows(_p(A), C.c_int64(Cc), C.c_int64(Cc), _p(rows), C.c_int64(rows.shape[0]),
                        _p(X), C.c_int64(nb), _p(Y), C.c_int64(nb), C.c_int64(nb))
    return Y


def rnn_forward(cell: int, W: List[np.ndarray], bias: Optional[List[Optional[np.ndarray]]],
                x: np.ndarray, input: int, hidden: int,
                h0: Optional[np.ndarray] = None, c0: Optional[np.ndarray] = None,
                want_hseq: bool = True) -> Tuple[Optional[np.ndarray], np.ndarray, np.ndarray]:
    """Stacked LSTM (cell 0) / GRU (cell 1) / Li-GRU (cell 3) / GRU with the reset gate applied
    before the recurrent product (cell 4).  W[l]: dense (G*H) x (in_l + H) float32.
    x: [T, B, I] float32.  Returns (hseq [T,B,H] or None, hT [L,B,H], cT [L,B,H]) float64."""
    lib = _load()
    L = len(W)
    G = {0: 4, 1: 3, 3: 2, 4: 3}[cell]
    Ws = []
    for l, w in enumerate(W):
        w = np.ascontiguousarray(w, dtype=np.float32)
        n_in = input if l == 0 else hidden
        assert w.shape == (G * hidden, n_in + hidden), (w.shape, l)
        Ws.append(w)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, B, I = x.shape
    assert I == input
    Wp = (C.c_void_p * L)(*[w.ctypes.data for w in Ws])
    bs = None
    Bp = None
    if bias is not None:
        bs = [None if b is None else np.ascontiguousarray(b, dtype=np.float32) for b in bias]
        Bp = (C.c_void_p * L)(*[None if b is None else b.ctypes.data for b in bs])
    h0 = None if h0 is None else np.ascontiguousarray(h0, dtype=np.float64).reshape(L, B, hidden)
    c0 = None if c0 is None else np.ascontiguousarray(c0, dtype=np.float64).reshape(L, B, hidden)
    hseq = np.empty((T, B, hidden), np.float64) if want_hseq else None
    hT = np.empty((L, B, hidden), np.float64)
    cT = np.empty((L, B, hidden), np.float64)
    rc = lib.orc_rnn_forward(C.c_int(cell), C.c_int32(L), C.c_int64(input), C.c_int64(hidden), Wp, Bp,
                             _p(x), _p(h0), _p(c0), _p(hseq), _p(hT), _p(cT), C.c_int64(T), C.c_int64(B))
    if rc != 0:
        raise ValueError("orc_rnn_forward failed")
    return hseq, hT, cT


def csb_project(W: np.ndarray, br: int, bc: int, rate: float) -> np.ndarray:
    """Projection of dense float32 W onto the CSB pattern (blocks br x bc) at pruning rate
    `rate` x: the RowPrune / ColumnPrune step of Algorithm 1.  Returns the pruned matrix."""
    lib = _load()
    W = np.ascontiguousarray(W, dtype=np.float32)
    R, Cc = W.shape
    Z = np.empty_like(W)
    rc = lib.orc_csb_project(_p(W), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), C.c_int32(br), C.c_int32(bc),
                             C.c_double(rate), _p(Z), C.c_int64(Cc))
    if rc != 0:
        raise ValueError("orc_csb_project: bad argument")
    return Z


def csb_project_f64(W: np.ndarray, br: int, bc: int, rate: float) -> np.ndarray:
    """The projection with the ranking sums in float64 (the plain definition, without the reading
    that the decision is taken in float32).  Returns the pruned matrix."""
    lib = _load()
    W = np.ascontiguousarray(W, dtype=np.float32)
    R, Cc = W.shape
    Z = np.empty_like(W)
    rc = lib.orc_csb_project_f64(_p(W), C.c_int64(R), C.c_int64(Cc), C.c_int64(Cc), C.c_int32(br), C.c_int32(bc),
                                 C.c_double(rate), _p(Z), C.c_int64(Cc))
    if rc != 0:
        raise ValueError("orc_csb_project_f64: bad argument")
    return Z


def lstmp_forward(W: List[np.ndarray], Wp: List[np.ndarray], bias: Optional[List[Optional[np.ndarray]]],
                  x: np.ndarray, input: int, hidden: int, proj: int,
                  h0: Optional[np.ndarray] = None, c0: Optional[np.ndarray] = None,
                  want_hseq: bool = True) -> Tuple[Optional[np.ndarray], np.ndarray, np.ndarray]:
    """Stacked LSTM with recurrent projection.  W[l]: (4H) x (in_l + P), Wp[l]: P x H, dense
    float32.  x: [T, B, I].  Returns (hseq [T,B,P] or None, hT [L,B,P], cT [L,B,H]) float64."""
    lib = _load()
    L = len(W)
    Ws, Ps = [], []
    for l in range(L):
        n_in = input if l == 0 else proj
        w = np.ascontiguousarray(W[l], dtype=np.float32)
        p = np.ascontiguousarray(Wp[l], dtype=np.float32)
        assert w.shape == (4 * hidden, n_in + proj) and p.shape == (proj, hidden), (w.shape, p.shape, l)
        Ws.append(w)
        Ps.append(p)
    x = np.ascontiguousarray(x, dtype=np.float32)
    T, B, I = x.shape
    assert I == input
    Wv = (C.c_void_p * L)(*[w.ctypes.data for w in Ws])
    Pv = (C.c_void_p * L)(*[p.ctypes.data for p in Ps])
    bs, Bv = None, None
    if bias is not None:
        bs = [None if b is None else np.ascontiguousarray(b, dtype=np.float32) for b in bias]
        Bv = (C.c_void_p * L)(*[None if b is None else b.ctypes.data for b in bs])
    h0 = None if h0 is None else np.ascontiguousarray(h0, dtype=np.float64).reshape(L, B, proj)
    c0 = None if c0 is None else np.ascontiguousarray(c0, dtype=np.float64).reshape(L, B, hidden)
    hseq = np.empty((T, B, proj), np.float64) if want_hseq else None
    hT = np.empty((L, B, proj), np.float64)
    cT = np.empty((L, B, hidden), np.float64)
    rc = lib.orc_lstmp_forward(C.c_int32(L), C.c_int64(input), C.c_int64(hidden), C.c_int64(proj), Wv, Pv, Bv,
                               _p(x), _p(h0), _p(c0), _p(hseq), _p(hT), _p(cT), C.c_int64(T), C.c_int64(B))
    if rc != 0:
        raise ValueError("orc_lstmp_forward failed")
    return hseq, hT, cT


def round_weights(a: np.ndarray, fmt: str) -> np.ndarray:
    """The float32 values nearest to `a` that a 16-bit weight format can hold (the paper
    quantises weights to 16 bits, Sec. 6.2.2 / 6.3.1; here the two 16-bit floating-point
    formats of the target), round to nearest, ties to even:
      'f16'  IEEE binary16 (overflow to infinity, gradual underflow) -- numpy's conversion;
      'bf16' the upper 16 bits of binary32 -- done on the bit patterns: add 0x7fff plus the
             lowest kept bit, then cut; NaN stays NaN.
    The 16-bit product is then DEFINED as the float64 product with these weights."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if fmt == "f16":
        with np.errstate(over="ignore"):
            return a.astype(np.float16).astype(np.float32)
    if fmt == "bf16":
        bits = a.view(np.uint32).astype(np.uint64)
        lsb = (bits >> np.uint64(16)) & np.uint64(1)
        r = ((bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)).astype(np.uint32)
        nan = np.isnan(a)
        r[nan] = (a.view(np.uint32)[nan] & np.uint32(0xFFFF0000)) | np.uint32(0x00400000)
        return r.view(np.float32).reshape(a.shape)
    raise ValueError(fmt)


def sharing_model(nrows: np.ndarray, ncols: np.ndarray, P: int, Q: int, K: int, L: int, exact_2d: bool = False) -> dict:
    """Cycle counts of the paper's engine schedule (Sec. 4.3.2, 5.2.2, 6.3.2) by brute force,
    for small inputs.  nrows / ncols: [nbr, nbc] kept rows / columns of every block.  K x L
    blocks per block iteration on K x L PEGroups of P x Q PEs; an a x b part takes
    ceil(a/P) ceil(b/Q) cycles; an iteration lasts as long as its most loaded PEGroup.
    Sharing: PEGroup (k,l) hands dnh columns (multiple of Q, at most n) to (k, l+1 mod L) and
    dmv rows (multiple of P, at most m // 2) to (k+1 mod K, l), in one of the two regular
    shapes of the partition constraints: shape 0 = horizontal part of full height (m x dnh),
    vertical part dmv x (n - dnh); shape 1 = vertical part of full width (dmv x n), horizontal
    part (m - dmv) x dnh; the rest (m - dmv) x (n - dnh) stays.  Every mode takes the schedule
    with the smallest largest load (full enumeration with itertools.product)."""
    import itertools
    nrows = np.asarray(nrows); ncols = np.asarray(ncols)
    nbr, nbc = nrows.shape
    cyc = lambda a, b: 0 if a <= 0 or b <= 0 else -(-a // P) * -(-b // Q)

    def parts(m, n, o):
        dnh, dmv, shape = o
        loc = cyc(m - dmv, n - dnh)
        if shape == 0:
            return loc, cyc(m, dnh), cyc(dmv, n - dnh)
        return loc, cyc(m - dmv, dnh), cyc(dmv, n)

    def best(dims, options):
        """dims: K x L list of (m, n); options[k][l]: allowed (dnh, dmv, shape)."""
        flat = [options[k][l] for k in range(K) for l in range(L)]
        bestT = None
        for choice in itertools.product(*flat):
            T = 0
            for k in range(K):
                for l in range(L):
                    m, n = dims[k][l]
                    loc = parts(m, n, choice[k * L + l])[0]
                    ml, nl = dims[k][(l - 1) % L]
                    mu, nu = dims[(k - 1) % K][l]
                    inh = parts(ml, nl, choice[k * L + (l - 1) % L])[1]
                    inv = parts(mu, nu, choice[((k - 1) % K) * L + l])[2]
                    T = max(T, loc + inh + inv)
            if bestT is None or T < bestT:
                bestT = T
        return bestT

    res = dict(work=0, iterations=0, cycles_none=0, cycles_horizontal=0, cycles_vertical=0, cycles_2d=0)
    for bi in range(-(-nbr // K)):
        for bj in range(-(-nbc // L)):
            dims = [[(int(nrows[bi * K + k, bj * L + l]), int(ncols[bi * K + k, bj * L + l]))
                     if bi * K + k < nbr and bj * L + l < nbc else (0, 0) for l in range(L)] for k in range(K)]
            res["iterations"] += 1
            res["work"] += sum(m * n for row in dims for m, n in row)
            res["cycles_none"] += max(cyc(m, n) for row in dims for m, n in row)
            oh = [[[(s, 0, 0) for s in range(0, n + 1, Q)] for (m, n) in row] for row in dims]
            ov = [[[(0, s, 1) for s in range(0, m // 2 + 1, P)] for (m, n) in row] for row in dims]
            res["cycles_horizontal"] += best(dims, oh)
            res["cycles_vertical"] += best(dims, ov)
            if exact_2d:
                o2 = [[[(a, b, sh) for sh in (0, 1) for a in range(0, n + 1, Q) for b in range(0, m // 2 + 1, P)]
                       for (m, n) in row] for row in dims]
                res["cycles_2d"] += best(dims, o2)
    denom = float(P * Q * K * L)
    for key in ("none", "horizontal", "vertical", "2d"):
        c = res["cycles_" + key]
        res["eff_" + key] = res["work"] / (denom * c) if c else 0.0
    return res

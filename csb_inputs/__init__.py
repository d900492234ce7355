"""Seeded synthetic inputs for CSB-RNN inference (shapes after the paper's Table 1).

This module only draws random numbers and applies row/column masks: it holds none of
the method's arithmetic (no encoding, no mat-vec, no cell math).  The CPU oracle and the
HIP library both consume the arrays produced here and share nothing else.

A workload is a set of block-structured pruned weight matrices: the matrix is tiled in
BR x BC blocks and inside every block whole rows and whole columns are zeroed, so the
survivors sit at the cross-points of the kept rows and kept columns (Sec. 3.1.1).  The
kept counts per block follow one of three laws (``binomial``, ``beta``, ``heavy``); a
per-dimension keep probability of rate**-0.5 gives an overall pruning rate of ``rate``
(the 1 - sqrt(1 - PruneRate) rule of Alg. 1 read as a fraction).

Draw order for one matrix (fixed, so that a seed names one matrix for ever):
  1. W_full ~ N(0, sigma), R x C, float32
  2. per-block kept counts (r_b, c_b) by the law, then +-1 fix-ups on random blocks until
     sum(r_b * c_b) is within 1 % of R*C/rate
  3. one uniform key per (block, local row) and per (block, local column); the r_b (c_b)
     smallest keys of a block are its kept rows (columns)
  4. A = W_full * mask
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

LSTM = 0
GRU = 1
LIGRU = 3          # Li-GRU (SR3 rows of Table 1): update gate and ReLU candidate
GRU_RB = 4         # GRU with the reset gate applied before the recurrent product
GATES = {LSTM: 4, GRU: 3, LIGRU: 2, GRU_RB: 3}


@dataclass(frozen=True)
class RnnConfig:
    name: str
    cell: int                 # LSTM / GRU / LIGRU / GRU_RB
    n_layers: int
    input: int
    hidden: int
    block: int                # square CSB block edge
    rate: float               # overall pruning rate (x)
    law: str                  # "binomial" | "beta"
    sigma: float
    batch: int
    T: int
    seed: int = 0


@dataclass(frozen=True)
class MatConfig:
    name: str
    rows: int
    cols: int
    block: int
    rate: float
    law: str                  # "heavy" | "heavy_diag" | "binomial" | "beta"
    sigma: float
    seed: int = 0


# The five workloads named by the baseline description.
CONFIGS: Dict[str, object] = {
    "cfg1": RnnConfig("cfg1", LSTM, 1, 64, 128, 16, 8.0, "binomial", 0.1, 1, 16, 0),
    "cfg2": RnnConfig("cfg2", LSTM, 1, 153, 512, 32, 10.0, "binomial", 0.05, 1, 100, 0),
    "cfg3": RnnConfig("cfg3", GRU, 1, 256, 1024, 32, 16.0, "beta", 0.05, 1, 200, 0),
    "cfg4": RnnConfig("cfg4", LSTM, 2, 1024, 1024, 64, 25.0, "binomial", 0.05, 64, 256, 0),
    "cfg5": MatConfig("cfg5", 8192, 8192, 32, 12.0, "heavy", 0.05, 0),
    "cfg5_diag": MatConfig("cfg5_diag", 8192, 8192, 32, 12.0, "heavy_diag", 0.05, 0),
}


@dataclass
class PrunedMatrix:
    A: np.ndarray             # [R, C] float32, masked dense
    rows: int
    cols: int
    br: int
    bc: int
    nbr: int
    nbc: int
    r_b: np.ndarray           # [nbr*nbc] int32 kept rows per block (0 if block empty)
    c_b: np.ndarray           # [nbr*nbc] int32 kept cols per block (0 if block empty)
    row_mask: np.ndarray      # [nbr*nbc, br] bool
    col_mask: np.ndarray      # [nbr*nbc, bc] bool
    nnz: int                  # sum r_b * c_b == mask popcount


def _edge_sizes(n: int, b: int) -> np.ndarray:
    nb = -(-n // b)
    e = np.full(nb, b, dtype=np.int64)
    e[-1] = n - (nb - 1) * b
    return e


def _draw_counts(rng, law: str, rate: float, er: np.ndarray, ec: np.ndarray):
    """Kept rows/cols per block.  er/ec: edge-aware block heights/widths, [nbr, nbc]."""
    nbr, nbc = er.shape
    if law == "binomial":
        p = rate ** -0.5
        r = rng.binomial(er, p)
        c = rng.binomial(ec, p)
    elif law == "beta":
        u = rng.beta(2.0, 5.0, size=(nbr, nbc))
        d = u * (1.0 / rate) / u.mean()
        root = np.sqrt(d)
        r = np.rint(er * root).astype(np.int64)
        jitter = rng.integers(-1, 2, size=(nbr, nbc))
        c = np.rint(ec * root).astype(np.int64) + jitter
    elif law in ("heavy", "heavy_diag"):
        # 10 % of blocks at density d_h, 90 % at 1/20, overall 1/rate:
        d_l = 1.0 / 20.0
        d_h = (1.0 / rate - 0.9 * d_l) / 0.1
        if law == "heavy":
            nb = nbr * nbc
            perm = rng.permutation(nb)
            heavy = np.zeros(nb, dtype=bool)
            heavy[perm[: int(round(0.1 * nb))]] = True
            heavy = heavy.reshape(nbr, nbc)
        else:
            bi, bj = np.meshgrid(np.arange(nbr), np.arange(nbc), indexing="ij")
            heavy = np.abs(bi - bj) <= 12
            frac = heavy.mean()
            d_h = (1.0 / rate - (1.0 - frac) * d_l) / frac
        p = np.where(heavy, d_h ** 0.5, d_l ** 0.5)
        r = rng.binomial(er, p)
        c = rng.binomial(ec, p)
    else:
        raise ValueError(f"unknown law {law!r}")
    r = np.clip(r, 0, er).astype(np.int64)
    c = np.clip(c, 0, ec).astype(np.int64)
    return r, c


def _fix_total(rng, r, c, er, ec, target: float):
    """+-1 on the larger kept dimension of random blocks until within 1 % of target."""
    nbr, nbc = r.shape
    total = int((r * c).sum())
    guard = 0
    while abs(total - target) > 0.01 * target and guard < 10_000_000:
        guard += 1
        b = int(rng.integers(0, nbr * nbc))
        i, j = divmod(b, nbc)
        ri, ci = int(r[i, j]), int(c[i, j])
        if total > target:
            if ri >= ci and ri > 0:
                r[i, j] = ri - 1
                total -= ci
            elif ci > 0:
                c[i, j] = ci - 1
                total -= ri
        else:
            if ri >= ci and ri < er[i, j]:
                r[i, j] = ri + 1
                total += ci
            elif ci < ec[i, j]:
                c[i, j] = ci + 1
                total += ri
            elif ri < er[i, j]:
                r[i, j] = ri + 1
                total += ci
    return r, c


def _subset_masks(rng, counts: np.ndarray, edges: np.ndarray, width: int) -> np.ndarray:
    """[nb, width] bool: a uniformly random subset of size counts[b] of range(edges[b])."""
    nb = counts.shape[0]
    keys = rng.random((nb, width))
    pos = np.arange(width)[None, :]
    keys = np.where(pos < edges[:, None], keys, 2.0)       # positions past the edge never win
    rank = np.argsort(np.argsort(keys, axis=1, kind="stable"), axis=1, kind="stable")
    return rank < counts[:, None]


def make_matrix(rng, rows: int, cols: int, br: int, bc: int, rate: float, law: str,
                sigma: float) -> PrunedMatrix:
    nbr, nbc = -(-rows // br), -(-cols // bc)
    W = rng.normal(0.0, sigma, size=(rows, cols)).astype(np.float32)
    er = np.broadcast_to(_edge_sizes(rows, br)[:, None], (nbr, nbc)).copy()
    ec = np.broadcast_to(_edge_sizes(cols, bc)[None, :], (nbr, nbc)).copy()
    r, c = _draw_counts(rng, law, rate, er, ec)
    r, c = _fix_total(rng, r, c, er, ec, rows * cols / rate)
    empty = (r == 0) | (c == 0)                            # nothing survives in such a block
    r = np.where(empty, 0, r)
    c = np.where(empty, 0, c)
    rm = _subset_masks(rng, r.reshape(-1), er.reshape(-1), br)
    cm = _subset_masks(rng, c.reshape(-1), ec.reshape(-1), bc)
    m4 = rm.reshape(nbr, nbc, br)[:, :, :, None] & cm.reshape(nbr, nbc, bc)[:, :, None, :]
    mask = m4.transpose(0, 2, 1, 3).reshape(nbr * br, nbc * bc)[:rows, :cols]
    A = np.where(mask, W, np.float32(0.0)).astype(np.float32)
    # A Gaussian draw is never exactly zero in practice; guard the invariant anyway.
    assert int(np.count_nonzero(A)) == int(mask.sum())
    return PrunedMatrix(A=np.ascontiguousarray(A), rows=rows, cols=cols, br=br, bc=bc,
                        nbr=nbr, nbc=nbc, r_b=r.reshape(-1).astype(np.int32),
                        c_b=c.reshape(-1).astype(np.int32), row_mask=rm, col_mask=cm,
                        nnz=int(mask.sum()))


@dataclass
class RnnWorkload:
    cfg: RnnConfig
    W: List[PrunedMatrix]                 # per layer, (G*H) x (in_l + H)
    bias: List[np.ndarray]                # per layer, [G*H] float32
    x: np.ndarray                         # [T, B, I] float32
    extra: dict = field(default_factory=dict)


def make_rnn(cfg: RnnConfig, T: Optional[int] = None, batch: Optional[int] = None,
             seed: Optional[int] = None) -> RnnWorkload:
    """All layers' matrices first (layer order), then all biases, then x."""
    T = cfg.T if T is None else T
    B = cfg.batch if batch is None else batch
    rng = np.random.Generator(np.random.PCG64(cfg.seed if seed is None else seed))
    G = GATES[cfg.cell]
    Ws = []
    for l in range(cfg.n_layers):
        in_l = cfg.input if l == 0 else cfg.hidden
        Ws.append(make_matrix(rng, G * cfg.hidden, in_l + cfg.hidden, cfg.block, cfg.block,
                              cfg.rate, cfg.law, cfg.sigma))
    bias = [rng.normal(0.0, cfg.sigma, size=G * cfg.hidden).astype(np.float32)
            for _ in range(cfg.n_layers)]
    x = rng.uniform(-1.0, 1.0, size=(T, B, cfg.input)).astype(np.float32)
    return RnnWorkload(cfg=cfg, W=Ws, bias=bias, x=x)


def split_gru_rb(A: np.ndarray, n_in: int, hidden: int):
    """Cuts a (3H) x (n_in + H) GRU matrix (rows r,z,n) into the two operands of the
    reset-before form: Wa = the matrix with the n rows' recurrent-side entries removed,
    Un = those entries as an H x H matrix.  Slicing only."""
    Wa = A.copy()
    Wa[2 * hidden:, n_in:] = 0.0
    Un = np.ascontiguousarray(A[2 * hidden:, n_in:])
    return Wa, Un


@dataclass
class LstmpWorkload:
    input: int
    hidden: int
    proj: int
    W: List[PrunedMatrix]       # (4H) x (in_l + P), in_0 = input, in_l = P
    Wp: List[PrunedMatrix]      # P x H
    bias: List[np.ndarray]      # 4H each
    x: np.ndarray               # [T, B, input]


def make_lstmp(seed: int, n_layers: int, input: int, hidden: int, proj: int, block: int, rate: float,
               T: int, batch: int, law: str = "binomial", sigma: float = 0.05) -> LstmpWorkload:
    """LSTM with a recurrent projection (the cell of the paper's SR1 rows of Table 1: 153 ->
    1024 with a 512-wide projection).  Draw order: per layer the gate matrix then the projection
    matrix, then all biases, then x."""
    rng = np.random.Generator(np.random.PCG64(seed))
    Ws, Ps = [], []
    for l in range(n_layers):
        in_l = input if l == 0 else proj
        Ws.append(make_matrix(rng, 4 * hidden, in_l + proj, block, block, rate, law, sigma))
        Ps.append(make_matrix(rng, proj, hidden, block, block, rate, law, sigma))
    bias = [rng.normal(0.0, sigma, size=4 * hidden).astype(np.float32) for _ in range(n_layers)]
    x = rng.uniform(-1.0, 1.0, size=(T, batch, input)).astype(np.float32)
    return LstmpWorkload(input=input, hidden=hidden, proj=proj, W=Ws, Wp=Ps, bias=bias, x=x)


def make_mat(cfg: MatConfig, seed: Optional[int] = None) -> PrunedMatrix:
    rng = np.random.Generator(np.random.PCG64(cfg.seed if seed is None else seed))
    return make_matrix(rng, cfg.rows, cols=cfg.cols, br=cfg.block, bc=cfg.block,
                       rate=cfg.rate, law=cfg.law, sigma=cfg.sigma)


def make_vectors(seed: int, cols: int, batch: int) -> np.ndarray:
    """x ~ U(-1, 1); [cols] for batch 1, else [cols, batch] (column k = right-hand side k)."""
    rng = np.random.Generator(np.random.PCG64(seed + 7919))
    shape = (cols,) if batch == 1 else (cols, batch)
    return rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)


def small_matrix(seed: int, rows: int, cols: int, br: int, bc: int, rate: float = 4.0,
                 law: str = "binomial", sigma: float = 0.5) -> PrunedMatrix:
    """Free-form matrix for parity cases (ragged edges, rectangular blocks, ...)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return make_matrix(rng, rows, cols, br, bc, rate, law, sigma)

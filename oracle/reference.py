"""Chain drivers over the C oracle (lop_oracle.c): unpartitioned and banded.

TEST INFRASTRUCTURE ONLY. Only tests, the bench's cpu_baseline leg and the
smoke check may import this; the product path never does.

``run_chain`` evaluates every layer on the whole tensor: this is the plain
definition of the result, since local operation parallelism re-orders execution
without changing any value (Sec. IV-B: each operation receives the correct
input and produces the correct output). ``run_chain_banded`` evaluates each band
on its own row slabs, holding only the rows the planner oracle says the band
needs, and concatenates the bands' final rows; padding is applied only at true
image borders, interior slab edges hold real halo rows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional

import numpy as np

from . import planner

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liblop_oracle.so")
_SRC = os.path.join(_HERE, "lop_oracle.c")

ACT = {"none": 0, "relu": 1, "relu6": 2}
DTYPE = {"f32": 0, "bf16": 1}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP over output rows)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", _SO, _SRC, "-lm"])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_round_bf16.restype = ctypes.c_double
        _lib.oracle_round_bf16.argtypes = [ctypes.c_double]
        _lib.oracle_out_size.restype = ctypes.c_int
    return _lib


def _fp(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def round_bf16(v: float) -> float:
    return lib().oracle_round_bf16(float(v))


class Slab:
    """Rows [row0, row0+rows) of an N x C x H x W tensor, stored N x C x rows x W."""

    def __init__(self, data: np.ndarray, row0: int, h_full: int):
        self.data = np.ascontiguousarray(data, dtype=np.float32)
        self.row0 = row0
        self.h_full = h_full

    @property
    def rows(self) -> int:
        return self.data.shape[2]


def run_layer(L, x: Slab, w, b, res: Optional[Slab], dtype: str, y_row0: int, y_rows: int,
              h_out: int, w_out: int) -> Slab:
    """One local operator on output rows [y_row0, y_row0+y_rows)."""
    n, c_in, _, wid = x.data.shape
    y = np.empty((n, L.c_out if L.op != "eltwise" else c_in, y_rows, w_out), np.float32)
    r_row0 = res.row0 if res is not None else 0
    r_rows = res.rows if res is not None else 0
    if L.op in ("conv", "dwconv"):
        rc = lib().oracle_conv2d(
            _fp(x.data), x.row0, x.rows, n, c_in, x.h_full, wid,
            _fp(w), _fp(b), L.c_out, L.groups,
            L.k[0], L.k[1], L.s[0], L.s[1], L.p[0], L.p[1], L.d[0], L.d[1],
            _fp(res.data if res is not None else None), r_row0, r_rows,
            ACT[L.act], DTYPE[dtype], _fp(y), y_row0, y_rows)
    elif L.op == "maxpool":
        assert res is None and L.act == "none"
        rc = lib().oracle_maxpool2d(
            _fp(x.data), x.row0, x.rows, n, c_in, x.h_full, wid,
            L.k[0], L.k[1], L.s[0], L.s[1], L.p[0], L.p[1], _fp(y), y_row0, y_rows)
    elif L.op == "eltwise":
        rc = lib().oracle_eltwise(
            _fp(x.data), x.row0, x.rows, n, c_in, x.h_full, wid, _fp(b),
            _fp(res.data if res is not None else None), r_row0, r_rows,
            ACT[L.act], DTYPE[dtype], _fp(y), y_row0, y_rows)
    else:
        raise ValueError(L.op)
    if rc != 0:
        raise RuntimeError(f"oracle layer {L.op} failed with code {rc} "
                           f"(-1: a needed row is outside the slab)")
    return Slab(y, y_row0, h_out)


def run_chain(chain, t, keep_all: bool = False):
    """Unpartitioned chain. Returns the final N x C x H x W array (or all layers')."""
    shapes = planner.infer_shapes(chain)
    outs: Dict[int, Slab] = {-1: Slab(t.x, 0, chain.in_shape[2])}
    for i, L in enumerate(chain.layers):
        res = outs[L.residual_from] if L.residual_from != -2 else None
        _, _, h, w = shapes[i]
        outs[i] = run_layer(L, outs[L.input_from], t.weights[i], t.biases[i], res,
                            chain.dtype, 0, h, h, w)
    if keep_all:
        return [outs[i].data for i in range(len(chain.layers))]
    return outs[len(chain.layers) - 1].data


def run_band(chain, t, need: Dict[int, Optional[tuple]]) -> Optional[Slab]:
    """One band: every tensor is held as the slab need[t]; returns the final slab."""
    shapes = planner.infer_shapes(chain)
    nl = len(chain.layers)
    if need[nl - 1] is None:
        return None
    lo, hi = need[-1]
    outs: Dict[int, Slab] = {-1: Slab(t.x[:, :, lo:hi, :], lo, chain.in_shape[2])}
    for i, L in enumerate(chain.layers):
        if need[i] is None:
            continue
        res = outs[L.residual_from] if L.residual_from != -2 else None
        lo, hi = need[i]
        _, _, h, w = shapes[i]
        outs[i] = run_layer(L, outs[L.input_from], t.weights[i], t.biases[i], res,
                            chain.dtype, lo, hi - lo, h, w)
    return outs[nl - 1]


def run_chain_banded(chain, t, n_bands: Optional[int] = None) -> np.ndarray:
    """All bands, each on its own slabs, concatenated along H."""
    shapes = planner.infer_shapes(chain)
    n, c, h, w = shapes[-1]
    out = np.full((n, c, h, w), np.nan, np.float32)
    covered = np.zeros(h, np.int32)
    for need in planner.plan(chain, n_bands):
        s = run_band(chain, t, need)
        if s is None:
            continue
        out[:, :, s.row0:s.row0 + s.rows, :] = s.data
        covered[s.row0:s.row0 + s.rows] += 1
    assert np.all(covered == 1), "bands must tile the final rows exactly once"
    return out


def run_chain_reuse(chain, t, n_bands: Optional[int] = None) -> np.ndarray:
    """Bands in order on shared full-height buffers; each band computes only the rows the
    planner oracle marks as not yet computed. Buffers start as NaN, so a row that is read
    before any band produced it poisons the result."""
    shapes = planner.infer_shapes(chain)
    nl = len(chain.layers)
    bufs: Dict[int, Slab] = {-1: Slab(t.x, 0, chain.in_shape[2])}
    for i, (n, c, h, w) in enumerate(shapes):
        bufs[i] = Slab(np.full((n, c, h, w), np.nan, np.float32), 0, h)
    for fresh in planner.plan_reuse(chain, n_bands):
        for i, L in enumerate(chain.layers):
            if fresh[i] is None:
                continue
            lo, hi = fresh[i]
            res = bufs[L.residual_from] if L.residual_from != -2 else None
            _, _, h, w = shapes[i]
            part = run_layer(L, bufs[L.input_from], t.weights[i], t.biases[i], res,
                             chain.dtype, lo, hi - lo, h, w)
            bufs[i].data[:, :, lo:hi, :] = part.data
    return bufs[nl - 1].data


# ---- row-wise local operators (Sec. IV-A, Eq. 1) ----

def rowwise(x: np.ndarray, w: np.ndarray, b, res, act: str, dtype: str,
            y: Optional[np.ndarray] = None, row0: int = 0, rows: Optional[int] = None) -> np.ndarray:
    """Rows [row0, row0 + rows) of act(x W^T + b + res) written into y (m x n); the other rows
    of y are left as they are."""
    m, k = x.shape
    n = w.shape[0]
    assert w.shape == (n, k)
    if y is None:
        y = np.full((m, n), np.nan, np.float32)
    rows = m - row0 if rows is None else rows
    rc = lib().oracle_rowwise(_fp(x), m, k, _fp(w), n, _fp(b), _fp(res), ACT[act], DTYPE[dtype],
                              _fp(y), row0, rows)
    if rc != 0:
        raise RuntimeError(f"oracle_rowwise failed with code {rc}")
    return y


def run_row_chain(chain, t, bands=None) -> np.ndarray:
    """A chain of row-wise operators on the whole matrix (bands=None: the definition), or
    band after band on the given list of (lo, hi) row intervals: every band runs the whole
    chain on its own rows before the next band starts."""
    m = chain.m
    outs = {-1: t.x}
    for i, L in enumerate(chain.layers):
        outs[i] = np.full((m, L.n), np.nan, np.float32)
    for lo, hi in ([(0, m)] if bands is None else bands):
        for i, L in enumerate(chain.layers):
            res = outs[L.residual_from] if L.residual_from != -2 else None
            rowwise(outs[L.input_from], t.weights[i], t.biases[i], res, L.act, chain.dtype,
                    outs[i], lo, hi - lo)
    return outs[len(chain.layers) - 1]

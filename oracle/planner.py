"""Planner oracle: which rows of every layer a band of final output rows needs.

TEST INFRASTRUCTURE ONLY; the product's planner is separate C++ and shares no
code with this file.

Two independent derivations are given and tests require them to agree:

* ``plan_closed_form``: interval arithmetic. A windowed local operator's output
  row ``oh`` reads input rows ``oh*s - p + a*d`` for ``a in [0,k)`` (Sec. IV-A:
  the block of a block-wise operator follows from kernel size, padding and
  dilation), so the output interval ``[lo,hi)`` needs the input interval
  ``[lo*s - p, (hi-1)*s - p + d*(k-1) + 1)`` clamped to the image. Where a
  tensor has several consumers (a shortcut branch, a residual read), its needed
  interval is the hull of the consumers' needs, which keeps it one contiguous
  interval (Sec. IV-C, Computational Efficiency). Overlap between bands is the
  paper's local-operation replication (Sec. IV-C).
* ``plan_brute_force``: set arithmetic only. Mark the band's final rows, walk
  the layers backwards and, for every marked output row, mark every in-image
  input row any of its taps touches; take min and max+1 of each set.

Bands are defined on the last layer's output rows and split with the
``numpy.array_split`` convention (first ``H % B`` bands one row longer; bands
may be empty when ``B > H``); together they must cover every operation exactly
once at the last layer (Sec. IV-C, Data Partitioning).
"""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

Interval = Optional[Tuple[int, int]]     # half-open; None = empty


def out_size(n_in: int, k: int, s: int, p: int, d: int) -> int:
    span = n_in + 2 * p - d * (k - 1) - 1
    return span // s + 1 if span >= 0 else 0


def infer_shapes(chain) -> List[Tuple[int, int, int, int]]:
    """(N, C, H, W) of every layer's output; index -1 is not included."""
    shapes = []
    for L in chain.layers:
        n, c, h, w = chain.in_shape if L.input_from < 0 else shapes[L.input_from]
        assert c == L.c_in, f"channel mismatch {c} != {L.c_in}"
        if L.op == "eltwise":
            shapes.append((n, c, h, w))
        else:
            shapes.append((n, L.c_out,
                           out_size(h, L.k[0], L.s[0], L.p[0], L.d[0]),
                           out_size(w, L.k[1], L.s[1], L.p[1], L.d[1])))
    return shapes


def split_rows(h_out: int, n_bands: int) -> List[Tuple[int, int]]:
    """array_split convention written out: first h%B bands get one more row."""
    base, extra = divmod(h_out, n_bands)
    out, lo = [], 0
    for b in range(n_bands):
        hi = lo + base + (1 if b < extra else 0)
        out.append((lo, hi))
        lo = hi
    return out


def _hull(a: Interval, b: Interval) -> Interval:
    if a is None:
        return b
    if b is None:
        return a
    return (min(a[0], b[0]), max(a[1], b[1]))


def _in_height(chain, shapes, L) -> int:
    return chain.in_shape[2] if L.input_from < 0 else shapes[L.input_from][2]


def plan_closed_form(chain, band_rows: Tuple[int, int]) -> Dict[int, Interval]:
    """need[t] for t = -1 (chain input) .. n_layers-1, for one band."""
    shapes = infer_shapes(chain)
    nl = len(chain.layers)
    need: Dict[int, Interval] = {t: None for t in range(-1, nl)}
    lo, hi = band_rows
    if hi > lo:
        need[nl - 1] = (lo, hi)
    for i in range(nl - 1, -1, -1):
        L = chain.layers[i]
        iv = need[i]
        if iv is None:
            continue
        lo, hi = iv
        if L.op == "eltwise":
            src = (lo, hi)
        else:
            k, s, p, d = L.k[0], L.s[0], L.p[0], L.d[0]
            h_in = _in_height(chain, shapes, L)
            a = max(lo * s - p, 0)
            b = min((hi - 1) * s - p + d * (k - 1) + 1, h_in)
            src = (a, b) if b > a else None
        need[L.input_from] = _hull(need[L.input_from], src)
        if L.residual_from != -2:
            need[L.residual_from] = _hull(need[L.residual_from], (lo, hi))
    return need


def plan_brute_force(chain, band_rows: Tuple[int, int]) -> Dict[int, Interval]:
    """Same table by marking individual rows; no interval formula is used."""
    shapes = infer_shapes(chain)
    nl = len(chain.layers)
    marked: Dict[int, set] = {t: set() for t in range(-1, nl)}
    marked[nl - 1] = set(range(band_rows[0], band_rows[1]))
    for i in range(nl - 1, -1, -1):
        L = chain.layers[i]
        rows = marked[i]
        if rows:
            # contiguity (Sec. IV-C): one launch computes [min, max] of the marked rows
            rows = set(range(min(rows), max(rows) + 1))
            marked[i] = rows
        h_in = _in_height(chain, shapes, L)
        for oh in rows:
            if L.op == "eltwise":
                marked[L.input_from].add(oh)
            else:
                for a in range(L.k[0]):
                    ih = oh * L.s[0] - L.p[0] + a * L.d[0]
                    if 0 <= ih < h_in:
                        marked[L.input_from].add(ih)
            if L.residual_from != -2:
                marked[L.residual_from].add(oh)
    return {t: ((min(r), max(r) + 1) if r else None) for t, r in marked.items()}


def plan(chain, n_bands: Optional[int] = None) -> List[Dict[int, Interval]]:
    """Closed-form table for every band of the chain."""
    shapes = infer_shapes(chain)
    bands = split_rows(shapes[-1][2], chain.n_bands if n_bands is None else n_bands)
    return [plan_closed_form(chain, br) for br in bands]


def plan_reuse(chain, n_bands: Optional[int] = None) -> List[Dict[int, Interval]]:
    """Rows each band computes when bands run in order and share per-layer buffers, so
    that data already on the device is reused instead of recomputed (Sec. IV-B: execution
    is placed where the required input already is). Set arithmetic only: of the rows
    band b needs of a layer (brute-force marking), those that no earlier band has
    computed. The result per layer must be one interval (Sec. IV-C contiguity)."""
    shapes = infer_shapes(chain)
    nl = len(chain.layers)
    bands = split_rows(shapes[-1][2], chain.n_bands if n_bands is None else n_bands)
    have: Dict[int, set] = {t: set() for t in range(nl)}
    out = []
    for br in bands:
        need = plan_brute_force(chain, br)
        fresh: Dict[int, Interval] = {}
        for t in range(nl):
            rows = set() if need[t] is None else set(range(need[t][0], need[t][1]))
            new = rows - have[t]
            if new:
                lo, hi = min(new), max(new) + 1
                assert new == set(range(lo, hi)), "fresh rows must be one interval"
                fresh[t] = (lo, hi)
            else:
                fresh[t] = None
            have[t] |= new
        out.append(fresh)
    return out


def flop_counts_reuse(chain, n_bands: Optional[int] = None) -> Tuple[float, float]:
    shapes = infer_shapes(chain)
    useful = sum(conv_flop(chain, shapes, i, shapes[i][2]) for i in range(len(chain.layers)))
    executed = 0.0
    for fresh in plan_reuse(chain, n_bands):
        for i, iv in fresh.items():
            if iv is not None:
                executed += conv_flop(chain, shapes, i, iv[1] - iv[0])
    return useful, executed


def receptive_field_rows(chain_layers) -> int:
    """RF = 1 + sum_l (k_l-1)*d_l*prod_{i<l} s_i along a straight chain of layers."""
    rf, jump = 1, 1
    for L in chain_layers:
        if L.op == "eltwise":
            continue
        rf += (L.k[0] - 1) * L.d[0] * jump
        jump *= L.s[0]
    return rf


def conv_flop(chain, shapes, i: int, rows: int) -> float:
    """2*N*rows*W_out*C_out*(C_in/groups)*kh*kw; padding taps are counted."""
    L = chain.layers[i]
    n, c, h, w = shapes[i]
    if L.op in ("conv", "dwconv"):
        return 2.0 * n * rows * w * L.c_out * (L.c_in // L.groups) * L.k[0] * L.k[1]
    if L.op == "maxpool":
        return 1.0 * n * rows * w * c * L.k[0] * L.k[1]
    return 1.0 * n * rows * w * c


def flop_counts(chain, n_bands: Optional[int] = None) -> Tuple[float, float]:
    """(useful, executed) operation counts: whole layers vs the sum over bands."""
    shapes = infer_shapes(chain)
    useful = sum(conv_flop(chain, shapes, i, shapes[i][2]) for i in range(len(chain.layers)))
    executed = 0.0
    for need in plan(chain, n_bands):
        for i in range(len(chain.layers)):
            if need[i] is not None:
                executed += conv_flop(chain, shapes, i, need[i][1] - need[i][0])
    return useful, executed

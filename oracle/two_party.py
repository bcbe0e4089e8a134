"""Oracle for the runtime stage of Intra-DP (Sec. IV-D, Alg. 1 client and Alg. 2 server): two
parties execute one schedule and exchange only the rows the other side is missing.

TEST INFRASTRUCTURE ONLY: only tests/ may import this. Plain Python over the C oracle's
per-layer functions (reference.run_layer), written from the paper's description:

* party M (the client) starts with the whole chain input, party R (the server) with nothing;
* for every layer u in chain order each party computes its own operations x_D(u) (one launch,
  operation batching) when that set is not empty;
* then, for every edge (u, v), the rows of Output(u) that x_D(v) reads and D does not hold are
  sent by the peer and combined into D's copy of Output(u) (Send / Receive / combine). The
  chain input is vertex -1 and its edges are served before layer 0; the edge from the last
  layer to the result asks for every row on M (the result stays on the client);
* values are never altered by this: each operation receives the correct input (Sec. IV-B), so
  the result must equal the unpartitioned chain.

Every buffer starts as NaN, so an operation that reads a row its party never computed nor
received poisons the result. Reading where the paper is silent:
a party keeps what it has received, so rows already received for an earlier consumer of the
same tensor are not sent again.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np

from . import planner, reference

Interval = Tuple[int, int]      # half-open; (a, a) is empty
INPUT, NO_RESIDUAL = -1, -2


@dataclass
class Transfer:
    u: int                      # tensor the rows belong to (-1: chain input)
    v: int                      # consumer (n_layers: the result)
    to: str                     # receiving party, "M" or "R"
    rows: Interval
    nbytes: int


@dataclass
class Stats:
    transfers: List[Transfer] = field(default_factory=list)

    def bytes_to(self, party: str) -> int:
        return sum(t.nbytes for t in self.transfers if t.to == party)


def _subtract(need: Interval, held: Sequence[Interval]) -> List[Interval]:
    """need minus the union of `held`, as sorted disjoint intervals."""
    out = [need] if need[1] > need[0] else []
    for h in held:
        nxt = []
        for a, b in out:
            if h[1] <= a or h[0] >= b or h[1] <= h[0]:
                nxt.append((a, b))
                continue
            if a < h[0]:
                nxt.append((a, h[0]))
            if h[1] < b:
                nxt.append((h[1], b))
        out = nxt
    return out


def _reads(chain, shapes, v: int, rows: Interval, u: int, identity: bool) -> Interval:
    """Rows of tensor u the operations `rows` of layer v read through that edge."""
    if rows[1] <= rows[0]:
        return (0, 0)
    L = chain.layers[v]
    if identity or L.op == "eltwise":
        return rows
    h_in = chain.in_shape[2] if u < 0 else shapes[u][2]
    lo = max(rows[0] * L.s[0] - L.p[0], 0)
    hi = min((rows[1] - 1) * L.s[0] - L.p[0] + L.d[0] * (L.k[0] - 1) + 1, h_in)
    return (lo, max(lo, hi))


def run(chain, t, sched: Sequence[Dict[str, Interval]]):
    """sched[v] = {"M": (lo, hi), "R": (lo, hi)} per layer. Returns (result on M, Stats)."""
    shapes = planner.infer_shapes(chain)
    nl = len(chain.layers)
    if len(sched) != nl:
        raise ValueError("one allocation per layer")
    esz = 2 if chain.dtype == "bf16" else 4
    for v, a in enumerate(sched):
        h = shapes[v][2]
        covered = set()
        for D in ("M", "R"):
            lo, hi = a[D]
            if not (0 <= lo <= hi <= h):
                raise ValueError("interval outside OP(v)")
            covered |= set(range(lo, hi))
        if covered != set(range(h)):
            raise ValueError("x_M(v) and x_R(v) do not cover OP(v)")

    def blank(u):
        n, c, h, w = (chain.in_shape if u < 0 else shapes[u])
        return np.full((n, c, h, w), np.nan, np.float32)

    buf = {D: {u: blank(u) for u in range(-1, nl)} for D in ("M", "R")}
    held: Dict[str, Dict[int, List[Interval]]] = {D: {u: [] for u in range(-1, nl)} for D in ("M", "R")}
    buf["M"][INPUT][...] = t.x
    held["M"][INPUT] = [(0, chain.in_shape[2])]
    stats = Stats()

    # edges out of u, in the order of their consumers: (v, identity?)
    def edges(u):
        out = []
        for v, L in enumerate(chain.layers):
            if L.input_from == u:
                out.append((v, False))
            if L.residual_from == u:
                out.append((v, True))
        if u == nl - 1:
            out.append((nl, True))
        return out

    def exchange(u):
        n, c, h, w = (chain.in_shape if u < 0 else shapes[u])
        row_bytes = n * c * w * esz
        for v, identity in edges(u):
            for D, O in (("M", "R"), ("R", "M")):
                if v == nl:
                    need = (0, h) if D == "M" else (0, 0)
                else:
                    need = _reads(chain, shapes, v, sched[v][D], u, identity)
                for piece in _subtract(need, held[D][u]):
                    if _subtract(piece, held[O][u]):
                        raise ValueError(f"rows {piece} of tensor {u} are on neither party")
                    buf[D][u][:, :, piece[0]:piece[1], :] = buf[O][u][:, :, piece[0]:piece[1], :]
                    held[D][u].append(piece)
                    stats.transfers.append(Transfer(u, v, D, piece, (piece[1] - piece[0]) * row_bytes))

    exchange(INPUT)
    for u, L in enumerate(chain.layers):
        _, _, h, w = shapes[u]
        for D in ("M", "R"):
            lo, hi = sched[u][D]
            if hi <= lo:
                continue
            src = L.input_from
            x = reference.Slab(buf[D][src], 0, chain.in_shape[2] if src < 0 else shapes[src][2])
            res = None
            if L.residual_from != NO_RESIDUAL:
                r = L.residual_from
                res = reference.Slab(buf[D][r], 0, chain.in_shape[2] if r < 0 else shapes[r][2])
            part = reference.run_layer(L, x, t.weights[u], t.biases[u], res, chain.dtype,
                                       lo, hi - lo, h, w)
            buf[D][u][:, :, lo:hi, :] = part.data
            held[D][u].append((lo, hi))
        exchange(u)
    return buf["M"][nl - 1], stats


def all_on(chain, party: str) -> List[Dict[str, Interval]]:
    shapes = planner.infer_shapes(chain)
    other = "R" if party == "M" else "M"
    return [{party: (0, s[2]), other: (0, 0)} for s in shapes]

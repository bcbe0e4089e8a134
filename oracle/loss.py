"""Oracle for the local-operation scheduling model of Intra-DP (Sec. IV-C): evaluate a schedule.

TEST INFRASTRUCTURE: only tests/ may import this. Plain Python, float64, written from the
paper's definitions:

* a vertex (layer) v has operations OP(v) = its output rows 0 .. n_v - 1;
* a schedule gives every vertex two contiguous intervals x_M(v), x_R(v) (operation batching
  constraint) whose union is OP(v) (data partitioning constraint); they may overlap (local
  operation replication);
* the chain input is whole on M and absent on R, the final result must be whole on M
  (location constraint);
* computing x_D(v) on device D takes C_D(v) = fixed_D(v) + per_row_D(v) * |x_D(v)| (0 if empty);
* data dependency recurrence (Eq. 3) for every edge (u, v) and device D with peer O: if some
  row of u's output that x_D(v) consumes was not produced on D (x_D(v) - child(x_D(u)) not
  empty) it travels from O after O has finished u, taking latency + rows * row_bytes(u) /
  bandwidth; v starts on D when every parent edge is satisfied;
* T = s_M(output) (Eq. 2);
* transmission-efficiency constraint: edges out of a vertex whose output is larger than the raw
  input must carry nothing.

Readings where the paper is silent: several parent edges of one
vertex combine by max; a device runs its operators one after another in chain order (one launch
per operator), so s_D(v) >= s_D(v - 1) + C_D(v - 1) also when v - 1 is not a parent; transfers
do not queue behind each other on the link (the recurrence has no such term); the volume of an
edge is counted in whole rows of the parent's output.

``evaluate_queued`` is the same model with the link as the runtime stage uses it (Sec. IV-D,
Alg. 1 and 2): after every layer u the parties exchange, edge by edge, the rows the consumers
will read; a message occupies its direction of the link for latency + bytes / bandwidth, so
messages of one direction queue in the order they are issued; a party keeps what it received,
so rows it already holds are not sent again. A consumer waits only for its own messages.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

Interval = Tuple[int, int]          # half-open; (a, a) is empty
INPUT, NO_RESIDUAL = -1, -2


@dataclass
class LossLayer:
    n_ops: int                       # output rows
    input_from: int = INPUT          # parent vertex of the windowed edge
    residual_from: int = NO_RESIDUAL  # parent of an identity edge (same rows), or none
    k: int = 1                       # rows of the parent one output row reads: window, stride,
    s: int = 1                       # padding, dilation of the row axis
    p: int = 0
    d: int = 1
    cm_fixed: float = 0.0
    cm_row: float = 0.0
    cr_fixed: float = 0.0
    cr_row: float = 0.0
    row_bytes: float = 0.0           # bytes of one output row


@dataclass
class Alloc:
    m: Interval
    r: Interval


def _len(iv: Interval) -> int:
    return max(0, iv[1] - iv[0])


def consumed_rows(layer: LossLayer, rows: Interval, parent_rows: int, identity: bool) -> Interval:
    """Rows of the parent's output that the operations `rows` of `layer` read (child^-1)."""
    if _len(rows) == 0:
        return (0, 0)
    if identity:
        return rows
    lo = max(rows[0] * layer.s - layer.p, 0)
    hi = min((rows[1] - 1) * layer.s - layer.p + layer.d * (layer.k - 1) + 1, parent_rows)
    return (lo, max(hi, lo))


def missing_rows(need: Interval, have: Interval) -> int:
    """|need - have| for intervals (rows the device must receive)."""
    if _len(need) == 0:
        return 0
    inter = max(0, min(need[1], have[1]) - max(need[0], have[0])) if _len(have) else 0
    return _len(need) - inter


def check(layers: Sequence[LossLayer], sched: Sequence[Alloc]) -> None:
    if len(layers) != len(sched):
        raise ValueError("one allocation per layer")
    for L, a in zip(layers, sched):
        for iv in (a.m, a.r):
            if not (0 <= iv[0] <= iv[1] <= L.n_ops):
                raise ValueError("interval outside OP(v)")
        m, r = a.m, a.r
        if _len(m) + _len(r) == 0:
            raise ValueError("no operation is executed")
        covered = set(range(*m)) | set(range(*r))
        if covered != set(range(L.n_ops)):
            raise ValueError("x_M(v) and x_R(v) do not cover OP(v)")


def evaluate(layers: Sequence[LossLayer], in_rows: int, in_row_bytes: float, bandwidth: float,
             latency: float, sched: Sequence[Alloc]):
    """Returns (T, s_M, s_R, pi_violations): start times per vertex (index n = output)."""
    check(layers, sched)
    n = len(layers)
    rows_of = lambda u: in_rows if u == INPUT else layers[u].n_ops
    bytes_of = lambda u: in_row_bytes if u == INPUT else layers[u].row_bytes
    x = {"M": lambda u: (0, in_rows) if u == INPUT else sched[u].m,
         "R": lambda u: (0, 0) if u == INPUT else sched[u].r}
    raw_input_bytes = in_rows * in_row_bytes

    def cost(dev: str, u: int) -> float:
        if u == INPUT:
            return 0.0
        L = layers[u]
        rows = _len(x[dev](u))
        if rows == 0:
            return 0.0
        return (L.cm_fixed + L.cm_row * rows) if dev == "M" else (L.cr_fixed + L.cr_row * rows)

    start = {"M": {INPUT: 0.0}, "R": {INPUT: 0.0}}
    violations = 0

    def ready(dev: str, peer: str, edges, prev: Optional[int]) -> float:
        nonlocal violations
        t = 0.0
        if prev is not None:
            t = start[dev][prev] + cost(dev, prev)
        for u, need in edges:
            local = start[dev][u] + cost(dev, u)
            miss = missing_rows(need, x[dev](u))
            if miss:
                arrive = start[peer][u] + cost(peer, u) + latency + miss * bytes_of(u) / bandwidth
                local = max(local, arrive)
                if rows_of(u) * bytes_of(u) > raw_input_bytes:
                    violations += 1
            t = max(t, local)
        return t

    for v, L in enumerate(layers):
        for dev, peer in (("M", "R"), ("R", "M")):
            mine = x[dev](v)
            edges = [(L.input_from, consumed_rows(L, mine, rows_of(L.input_from), False))]
            if L.residual_from != NO_RESIDUAL:
                edges.append((L.residual_from, consumed_rows(L, mine, rows_of(L.residual_from), True)))
            start[dev][v] = ready(dev, peer, edges, v - 1 if v > 0 else None)
    last = n - 1
    t_out = ready("M", "R", [(last, (0, layers[last].n_ops))], last)
    s_m = [start["M"][v] for v in range(n)] + [t_out]
    s_r = [start["R"][v] for v in range(n)]
    return t_out, s_m, s_r, violations


def _minus(need: Interval, held: Sequence[Interval]) -> List[Interval]:
    out = [need] if _len(need) else []
    for h in held:
        if not _len(h):
            continue
        nxt = []
        for a, b in out:
            if h[1] <= a or h[0] >= b:
                nxt.append((a, b))
                continue
            if a < h[0]:
                nxt.append((a, h[0]))
            if h[1] < b:
                nxt.append((h[1], b))
        out = nxt
    return out


def evaluate_queued(layers: Sequence[LossLayer], in_rows: int, in_row_bytes: float, bandwidth: float,
                    latency: float, sched: Sequence[Alloc]):
    """Same returns as evaluate(), with the link shared as the runtime stage shares it."""
    check(layers, sched)
    n = len(layers)
    rows_of = lambda u: in_rows if u == INPUT else layers[u].n_ops
    bytes_of = lambda u: in_row_bytes if u == INPUT else layers[u].row_bytes
    x = {"M": lambda v: sched[v].m, "R": lambda v: sched[v].r}
    raw_input_bytes = in_rows * in_row_bytes
    held = {D: {u: [] for u in range(-1, n)} for D in "MR"}
    held["M"][INPUT] = [(0, in_rows)]
    finish = {D: {INPUT: 0.0} for D in "MR"}        # when D's own rows of u exist
    start = {D: {} for D in "MR"}
    arrive = {D: {v: 0.0 for v in range(n + 1)} for D in "MR"}   # last message for consumer v
    link_free = {"M": 0.0, "R": 0.0}                # direction into that party
    violations = 0

    def exchange(u):
        nonlocal violations
        for v in range(n + 1):
            kinds = []
            if v == n:
                if u == n - 1:
                    kinds.append(True)
            else:
                if layers[v].input_from == u:
                    kinds.append(False)
                if layers[v].residual_from == u:
                    kinds.append(True)
            for identity in kinds:
                for D, O in (("M", "R"), ("R", "M")):
                    if v == n:
                        need = (0, rows_of(u)) if D == "M" else (0, 0)
                    else:
                        need = consumed_rows(layers[v], x[D](v), rows_of(u), identity)
                    for lo, hi in _minus(need, held[D][u]):
                        begin = max(finish[O][u], link_free[D])
                        done = begin + latency + (hi - lo) * bytes_of(u) / bandwidth
                        link_free[D] = done
                        arrive[D][v] = max(arrive[D][v], done)
                        held[D][u].append((lo, hi))
                        if rows_of(u) * bytes_of(u) > raw_input_bytes:
                            violations += 1

    exchange(INPUT)
    for u, L in enumerate(layers):
        for D in "MR":
            s = arrive[D][u]
            if u > 0:
                s = max(s, finish[D][u - 1])
            start[D][u] = s
            rows = _len(x[D](u))
            c = 0.0
            if rows:
                c = (L.cm_fixed + L.cm_row * rows) if D == "M" else (L.cr_fixed + L.cr_row * rows)
                held[D][u].append(x[D](u))
            finish[D][u] = s + c
        exchange(u)
    t_out = max(finish["M"][n - 1], arrive["M"][n])
    s_m = [start["M"][v] for v in range(n)] + [t_out]
    s_r = [start["R"][v] for v in range(n)]
    return t_out, s_m, s_r, violations


def all_on(layers: Sequence[LossLayer], dev: str) -> List[Alloc]:
    return [Alloc((0, L.n_ops), (0, 0)) if dev == "M" else Alloc((0, 0), (0, L.n_ops)) for L in layers]


def brute_force(layers: Sequence[LossLayer], in_rows: int, in_row_bytes: float, bandwidth: float,
                latency: float):
    """Smallest T over every schedule of the form x_M = [0, a), x_R = [b, n) with b <= a
    (M takes leading rows, R trailing rows, overlap = replication) and no violation of the
    transmission-efficiency constraint. Exponential: tiny instances only."""
    choices = []
    for L in layers:
        c = []
        for a in range(L.n_ops + 1):
            for b in range(a + 1):
                if a == 0 and b != 0:
                    continue
                m, r = (0, a), (b, L.n_ops)
                if a == L.n_ops and b == a:
                    r = (0, 0)
                c.append(Alloc(m, r))
        choices.append(c)
    best, best_s = float("inf"), None
    for combo in itertools.product(*choices):
        try:
            t, _, _, viol = evaluate(layers, in_rows, in_row_bytes, bandwidth, latency, combo)
        except ValueError:
            continue
        if viol == 0 and t < best:
            best, best_s = t, list(combo)
    return best, best_s

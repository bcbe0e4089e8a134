"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, its
integer planner agrees bit for bit with the planner oracle, and argument errors come back
as the documented codes. No kernel is launched."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads
from oracle import planner as oplan
from paper_2507_05829_amd import lop

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "lop.h")).read()
    declared = set(re.findall(r"LOP_API\s+[\w\s\*]+?\b(lop_\w+)\s*\(", hdr))
    assert declared == set(lop.EXPORTS)
    lib = ctypes.CDLL(lop.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_covers_codes():
    texts = {lop.lop_strerror(c) for c in range(0, -8, -1)}
    assert len(texts) == 8 and "unknown error" not in texts
    assert lop.lop_strerror(-99) == "unknown error"


@pytest.mark.parametrize("name", list(workloads.CONFIGS))
def test_planner_matches_oracle_bit_exact(name):
    chain = workloads.CONFIGS[name]()
    plan = lop.Plan(chain)                         # plan-only: no GPU needed
    shapes = oplan.infer_shapes(chain)
    assert plan.out_shape() == shapes[-1]
    for l, s in enumerate(shapes):
        assert plan.layer_shape(l) == s
    want = oplan.plan(chain)
    split = oplan.split_rows(shapes[-1][2], chain.n_bands)
    for b in range(chain.n_bands):
        assert plan.band_out_rows(b) == split[b]
        for t in range(-1, len(chain.layers)):
            got = plan.band_layer_rows(b, t)
            exp = want[b][t]
            assert got == ((0, 0) if exp is None else exp), (name, b, t)
        assert plan.band_in_rows(b) == plan.band_layer_rows(b, -1)
    u, e, scratch = plan.stats()
    ou, oe = oplan.flop_counts(chain)
    assert u == ou and e == oe
    assert scratch > 0


def test_planner_matches_oracle_random_chains():
    from test_oracle_planner import _random_chain
    rng = np.random.default_rng(5)
    done = 0
    while done < 100:
        chain = _random_chain(rng)
        if chain is None or any(L.op == "maxpool" and L.p[0] >= L.k[0] for L in chain.layers):
            continue
        done += 1
        plan = lop.Plan(chain)
        want = oplan.plan(chain)
        for b in range(chain.n_bands):
            for t in range(-1, len(chain.layers)):
                exp = want[b][t]
                assert plan.band_layer_rows(b, t) == ((0, 0) if exp is None else exp)


def test_layer_work_counts():
    chain = workloads.tiny_chain()
    plan = lop.Plan(chain)
    # band 1, layer 0: rows (7,17) = 10 rows out, reads rows (6,18) = 12 rows in
    flop, byts = plan.layer_work(1, 0)
    assert flop == 2 * 10 * 32 * 16 * 16 * 9
    assert byts == 4 * (12 * 32 * 16 + 10 * 32 * 16) + 4 * 16 * 16 * 9


def _desc(n=1, c=4, h=8, w=8, dt=lop.LOP_F32):
    return lop.lop_tensor_desc_t(n, c, h, w, dt)


def _layer(op=lop.LOP_CONV2D, c_in=4, c_out=4, k=3, s=1, p=1, d=1, act=0, src=-1, res=-2):
    return lop.lop_layer_t(op, c_in, c_out, k, k, s, s, p, p, d, d, act, src, res, None, None)


def _code(layers, desc=None, n_bands=2, flags=lop.LOP_FLAG_PLAN_ONLY):
    try:
        h = lop.lop_plan(layers, desc or _desc(), n_bands, flags)
    except lop.LopError as e:
        return e.code
    lop.lop_plan_destroy(h)
    return 0


def test_error_codes():
    assert _code([_layer()]) == 0
    assert _code([_layer()], n_bands=0) == lop.LOP_ERR_INVALID_ARG
    assert _code([_layer()], n_bands=65) == lop.LOP_ERR_INVALID_ARG
    assert _code([_layer()], desc=_desc(h=0)) == lop.LOP_ERR_INVALID_ARG
    assert _code([_layer(src=0)]) == lop.LOP_ERR_INVALID_ARG          # forward reference
    assert _code([_layer(s=0)]) == lop.LOP_ERR_INVALID_ARG
    assert _code([_layer(op=9)]) == lop.LOP_ERR_UNSUPPORTED           # e.g. a global operator
    assert _code([_layer()], desc=_desc(dt=5)) == lop.LOP_ERR_UNSUPPORTED
    assert _code([_layer(c_in=3)]) == lop.LOP_ERR_SHAPE               # channel mismatch
    assert _code([_layer(k=11, p=0)]) == lop.LOP_ERR_SHAPE            # window larger than input
    assert _code([_layer(op=lop.LOP_DWCONV2D, c_out=8)]) == lop.LOP_ERR_SHAPE
    assert _code([_layer(s=2), _layer(src=0, res=-1)]) == lop.LOP_ERR_SHAPE   # residual shape
    assert _code([_layer(op=lop.LOP_MAXPOOL2D, act=1)]) == lop.LOP_ERR_INVALID_ARG
    assert _code([_layer(op=lop.LOP_MAXPOOL2D, k=2, p=2)]) == lop.LOP_ERR_UNSUPPORTED
    # a plan that needs weights but has none
    assert _code([_layer()], flags=0) in (lop.LOP_ERR_INVALID_ARG, lop.LOP_ERR_HIP)


def test_band_range_and_not_ready():
    h = lop.lop_plan([_layer()], _desc(), 2, lop.LOP_FLAG_PLAN_ONLY)
    try:
        with pytest.raises(lop.LopError) as e:
            lop.lop_plan_band_out_rows(h, 2)
        assert e.value.code == lop.LOP_ERR_BAND_RANGE
        with pytest.raises(lop.LopError) as e:
            lop.lop_plan_band_layer_rows(h, 0, 1)
        assert e.value.code == lop.LOP_ERR_BAND_RANGE
        with pytest.raises(lop.LopError) as e:
            lop.lop_run_band(h, 0, 16, 16)        # dummy non-null addresses, never touched
        assert e.value.code == lop.LOP_ERR_NOT_READY
        with pytest.raises(lop.LopError) as e:
            lop.lop_run_chain(h, 16, 16)
        assert e.value.code == lop.LOP_ERR_NOT_READY
        with pytest.raises(lop.LopError) as e:
            lop.lop_run_chain(h, None, 16)
        assert e.value.code == lop.LOP_ERR_INVALID_ARG
        # tensors start on a 16-byte boundary
        for call in (lambda: lop.lop_run_band(h, 0, 24, 16), lambda: lop.lop_run_band(h, 0, 16, 16, 8),
                     lambda: lop.lop_run_chain(h, 16, 40), lambda: lop.lop_run_chain(h, 16, 16, 4),
                     lambda: lop.lop_run_chain_static(h, 2, 16)):
            with pytest.raises(lop.LopError) as e:
                call()
            assert e.value.code == lop.LOP_ERR_INVALID_ARG
    finally:
        lop.lop_plan_destroy(h)
    lop.lop_plan_destroy(None)                   # destroying NULL is a no-op


@pytest.mark.parametrize("name", list(workloads.CONFIGS))
def test_reuse_planner_matches_oracle_bit_exact(name):
    chain = workloads.CONFIGS[name]()
    plan = lop.Plan(chain, flags=lop.LOP_FLAG_REUSE)
    want = oplan.plan_reuse(chain)
    need = oplan.plan(chain)
    for b in range(chain.n_bands):
        for l in range(len(chain.layers)):
            exp = want[b][l]
            assert plan.band_compute_rows(b, l) == ((0, 0) if exp is None else exp), (name, b, l)
            n = need[b][l]
            assert plan.band_layer_rows(b, l) == ((0, 0) if n is None else n)
    u, e, _ = plan.stats()
    ou, oe = oplan.flop_counts_reuse(chain)
    assert u == ou and e == oe
    # independent plans compute exactly what they need
    ind = lop.Plan(chain)
    for b in range(chain.n_bands):
        for l in range(len(chain.layers)):
            assert ind.band_compute_rows(b, l) == ind.band_layer_rows(b, l)


def test_reuse_planner_random_chains():
    from test_oracle_planner import _random_chain
    rng = np.random.default_rng(9)
    done = 0
    while done < 100:
        chain = _random_chain(rng)
        if chain is None or any(L.op == "maxpool" and L.p[0] >= L.k[0] for L in chain.layers):
            continue
        if any(L.d[0] > 1 and L.k[0] > 1 for L in chain.layers):
            continue        # with dilation the closed form is a superset (see the planner pins)
        done += 1
        plan = lop.Plan(chain, flags=lop.LOP_FLAG_REUSE)
        try:
            want = oplan.plan_reuse(chain)
        except AssertionError:
            continue        # a chain whose fresh rows are not one interval is not plannable
        for b in range(chain.n_bands):
            for l in range(len(chain.layers)):
                exp = want[b][l]
                assert plan.band_compute_rows(b, l) == ((0, 0) if exp is None else exp), (chain, b, l)


def test_rowwise_plan_rows_and_errors():
    """lop_plan_rowwise: bands are numpy.array_split of the matrix rows, no halo anywhere."""
    chain = workloads.RowChain("c", 1000, 48, "f32", 7)
    chain.add(96, "relu").add(48, "none", residual_from=-1)
    plan = lop.Plan.rowwise(chain)
    assert plan.out_shape() == (1, 48, 1000, 1)
    want = [(int(a[0]), int(a[-1]) + 1) for a in np.array_split(np.arange(1000), 7)]
    for b in range(7):
        assert plan.band_out_rows(b) == want[b]
        assert plan.band_in_rows(b) == want[b]
        for l in range(2):
            assert plan.band_layer_rows(b, l) == want[b]
    u, e, _ = plan.stats()
    assert u == e == 2.0 * 1000 * (48 * 96 + 96 * 48)
    plan.destroy()
    with pytest.raises(lop.LopError) as ei:
        lop.lop_plan_rowwise([], 10, 4, 0, 2, lop.LOP_FLAG_PLAN_ONLY)
    assert ei.value.code == -1
    bad = lop.lop_rowwise_t(5, 8, 0, -1, -2, None, None)          # k does not match the input
    with pytest.raises(lop.LopError) as ei:
        lop.lop_plan_rowwise([bad], 10, 4, 0, 2, lop.LOP_FLAG_PLAN_ONLY)
    assert ei.value.code in (-1, -3)


def test_two_party_schedule_is_checked_on_the_host():
    """The schedule's constraints (two intervals covering OP(v), Sec. IV-C) are checked before
    anything touches the GPU, so a plan-only plan is enough to see the codes."""
    h = lop.lop_plan([_layer(), _layer(src=0)], _desc(), 2, lop.LOP_FLAG_PLAN_ONLY)

    def code(sched, bandwidth=1e9, latency=0.0):
        try:
            lop.lop_run_two_party(h, 16, 16, sched, bandwidth, latency)
        except lop.LopError as e:
            return e.code
        return 0

    try:
        good = [((0, 5), (5, 8)), ((0, 8), (0, 0))]
        assert code(good) == lop.LOP_ERR_NOT_READY                      # valid, but nothing uploaded
        assert code(good[:1]) == lop.LOP_ERR_INVALID_ARG                # one entry per layer
        assert code(good, bandwidth=0.0) == lop.LOP_ERR_INVALID_ARG
        assert code(good, latency=-1.0) == lop.LOP_ERR_INVALID_ARG
        assert code([((0, 4), (5, 8)), ((0, 8), (0, 0))]) == lop.LOP_ERR_BAND_RANGE   # row 4 missing
        assert code([((0, 9), (0, 0)), ((0, 8), (0, 0))]) == lop.LOP_ERR_BAND_RANGE   # outside OP(v)
        assert code([((3, 2), (0, 8)), ((0, 8), (0, 0))]) == lop.LOP_ERR_BAND_RANGE   # lo > hi
        assert code([((2, 6), (0, 3)), ((0, 8), (0, 0))]) == lop.LOP_ERR_BAND_RANGE   # rows 6, 7 missing
        assert code([((2, 8), (0, 3)), ((0, 0), (0, 8))]) == lop.LOP_ERR_NOT_READY    # overlap is fine
    finally:
        lop.lop_plan_destroy(h)


def test_kernel_query_on_a_plan_without_device_state():
    """A plan-only plan has tables but no uploaded weights. Which kernel takes a layer depends
    on the weight packings that exist, so such a plan names no kernel (rather than one that the
    same chain's ready plan would not launch), and its work counts are those of the layers."""
    h = lop.lop_plan([_layer(c_in=4, c_out=64), _layer(c_in=64, c_out=64, src=0)],
                     _desc(c=4, h=32, w=32), 2, lop.LOP_FLAG_PLAN_ONLY)
    try:
        for band in range(2):
            for layer in range(2):
                name, slices = lop.lop_plan_layer_kernel(h, band, layer)
                assert name == "" and slices == 0
                flop, byts = lop.lop_plan_layer_work(h, band, layer)
                lo, hi = lop.lop_plan_band_compute_rows(h, band, layer)
                c_in = 4 if layer == 0 else 64
                assert flop == 2.0 * (hi - lo) * 32 * 64 * c_in * 9 and byts > 0
    finally:
        lop.lop_plan_destroy(h)

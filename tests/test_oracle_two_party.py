"""Pins of the two-party runtime oracle (Sec. IV-D, Alg. 1 and 2) against what the paper and
plain counting fix: the result equals the unpartitioned chain for any schedule that obeys the
partitioning constraint, the rows exchanged equal what marking individual rows says, and the
special schedules reduce to closed forms."""
import numpy as np
import pytest

import workloads
from oracle import planner, two_party


def _heights(chain):
    return [s[2] for s in planner.infer_shapes(chain)]


def test_hand_worked_two_layer_example(oracle):
    """Two 3x3 convolutions (stride 1, padding 1) on 6 rows; M owns rows [0, 3) and R rows
    [3, 6) of both layers. Counting by hand along Alg. 1 / Alg. 2:
    input -> layer 0: R's rows 3..5 read input rows 2..5, all missing on R: 4 rows M->R;
    layer 0 -> layer 1: M's rows 0..2 read rows 0..3, row 3 is R's: 1 row R->M;
                        R's rows 3..5 read rows 2..5, row 2 is M's: 1 row M->R;
    layer 1 -> result: M lacks rows 3..5: 3 rows R->M."""
    c = workloads.Chain("hand", (1, 4, 6, 5), "f32", 1)
    c.add(workloads.CONV, 4, 4, 3, 1, 1, act="relu")
    c.add(workloads.CONV, 4, 4, 3, 1, 1, act="relu")
    t = workloads.make_tensors(c, zero_bias=False, seed=5)
    sched = [{"M": (0, 3), "R": (3, 6)}] * 2
    out, st = two_party.run(c, t, sched)
    np.testing.assert_array_equal(out, oracle.run_chain(c, t))
    got = [(x.u, x.v, x.to, x.rows) for x in st.transfers]
    assert got == [(-1, 0, "R", (2, 6)), (0, 1, "M", (3, 4)), (0, 1, "R", (2, 3)), (1, 2, "M", (3, 6))]
    row = 1 * 4 * 5 * 4
    assert st.bytes_to("R") == 5 * row and st.bytes_to("M") == 4 * row


@pytest.mark.parametrize("party", ["M", "R"])
def test_single_party_schedules(oracle, party):
    """Everything on the client moves nothing; everything on the server moves the input one way
    and the result the other way, once (the layer-partitioning extremes of Sec. II)."""
    c = workloads.resnet18_chain(h=64, w=48)
    t = workloads.make_tensors(c, zero_bias=False)
    out, st = two_party.run(c, t, two_party.all_on(c, party))
    np.testing.assert_array_equal(out, oracle.run_chain(c, t))
    if party == "M":
        assert st.transfers == []
    else:
        shapes = planner.infer_shapes(c)
        assert st.bytes_to("R") == int(np.prod(c.in_shape)) * 4
        assert st.bytes_to("M") == int(np.prod(shapes[-1])) * 4
        assert len(st.transfers) == 2


def _brute_bytes(chain, sched):
    """Bytes per direction by marking single rows, no interval arithmetic."""
    shapes = planner.infer_shapes(chain)
    nl = len(chain.layers)
    esz = 2 if chain.dtype == "bf16" else 4
    held = {D: {u: set() for u in range(-1, nl)} for D in "MR"}
    held["M"][-1] = set(range(chain.in_shape[2]))
    total = {"M": 0, "R": 0}

    def serve(u):
        n, ch, h, w = chain.in_shape if u < 0 else shapes[u]
        for v in range(nl + 1):
            kinds = []
            if v == nl:
                if u == nl - 1:
                    kinds.append("out")
            else:
                L = chain.layers[v]
                if L.input_from == u:
                    kinds.append("win")
                if L.residual_from == u:
                    kinds.append("id")
            for kind in kinds:
                for D in "MR":
                    want = set()
                    if kind == "out":
                        want = set(range(h)) if D == "M" else set()
                    else:
                        L = chain.layers[v]
                        for oh in range(*sched[v][D]):
                            if kind == "id" or L.op == "eltwise":
                                want.add(oh)
                            else:
                                for a in range(L.k[0]):
                                    ih = oh * L.s[0] - L.p[0] + a * L.d[0]
                                    if 0 <= ih < h:
                                        want.add(ih)
                    if want:   # one message carries a contiguous run of rows (strided windows
                        want = set(range(min(want), max(want) + 1))   # leave gaps inside it)
                    new = want - held[D][u]
                    total[D] += len(new) * n * ch * w * esz
                    held[D][u] |= new

    serve(-1)
    for u in range(nl):
        for D in "MR":
            held[D][u] |= set(range(*sched[u][D]))
        serve(u)
    return total


@pytest.mark.parametrize("name,kw", [
    ("tiny", {}),
    ("resnet18", dict(h=64, w=48)),
    ("mbv2", dict(h=48, w=40, n=2)),
    ("detector720p", dict(h=90, w=64)),
])
def test_random_schedules_keep_the_result_and_the_row_count(oracle, name, kw):
    chain = workloads.CONFIGS[name](**kw)
    t = workloads.make_tensors(chain, zero_bias=False)
    full = oracle.run_chain(chain, t)
    for seed in range(3):
        sched = workloads.random_schedule(_heights(chain), seed=100 + seed, overlap=3)
        out, st = two_party.run(chain, t, sched)
        assert not np.isnan(out).any()
        np.testing.assert_array_equal(out, full)
        brute = _brute_bytes(chain, sched)
        assert st.bytes_to("M") == brute["M"] and st.bytes_to("R") == brute["R"]


def test_a_dropped_halo_row_poisons_the_result(oracle, monkeypatch):
    """Plant a mistake in the oracle (the window's last row is not requested): the operation
    then reads a row nobody sent, which is NaN by construction, so the mistake cannot pass."""
    chain = workloads.Chain("plain", (1, 8, 32, 12), "f32", 1)     # no activation: a ReLU
    chain.add(workloads.CONV, 8, 8, 3, 1, 1)                         # would turn NaN into 0
    chain.add(workloads.CONV, 8, 8, 3, 1, 1)
    t = workloads.make_tensors(chain, zero_bias=False)
    good = two_party._reads

    def short(chain_, shapes, v, rows, u, identity):
        lo, hi = good(chain_, shapes, v, rows, u, identity)
        return (lo, max(lo, hi - 1))

    monkeypatch.setattr(two_party, "_reads", short)
    sched = [{"M": (0, 16), "R": (16, 32)}] * 2
    out, _ = two_party.run(chain, t, sched)
    assert np.isnan(out).any()
    monkeypatch.setattr(two_party, "_reads", good)
    out, _ = two_party.run(chain, t, sched)
    np.testing.assert_array_equal(out, oracle.run_chain(chain, t))


def test_schedule_that_does_not_cover_is_refused(oracle):
    chain = workloads.tiny_chain()
    t = workloads.make_tensors(chain)
    with pytest.raises(ValueError):
        two_party.run(chain, t, [{"M": (0, 10), "R": (11, 32)}] * 2)
    with pytest.raises(ValueError):
        two_party.run(chain, t, [{"M": (0, 33), "R": (0, 0)}] * 2)

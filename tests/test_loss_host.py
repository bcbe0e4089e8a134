"""The library's schedule evaluator and solver (host code, no GPU) against the oracle of
the scheduling model (Intra-DP Sec. IV-C)."""
import numpy as np
import pytest

import workloads
from oracle import loss as O
from oracle import planner
from paper_2507_05829_amd import lop


def as_sched(allocs):
    return [(a.m, a.r) for a in allocs]


def unit_chain(k2=1, p2=0):
    return [O.LossLayer(3, -1, cm_row=1, cr_row=1, row_bytes=1),
            O.LossLayer(3, 0, k=k2, p=p2, cm_row=1, cr_row=1, row_bytes=1)]


def test_hand_worked_timelines_through_the_abi():
    sched = [((0, 2), (2, 3)), ((0, 2), (2, 3))]
    assert lop.lop_loss_eval(unit_chain(), 3, 1.0, 1.0, 0.0, sched) == (4.0, [0.0, 2.0, 4.0], [1.0, 2.0], 0)
    assert lop.lop_loss_eval(unit_chain(3, 1), 3, 1.0, 1.0, 0.0, sched) == (5.0, [0.0, 3.0, 5.0], [1.0, 3.0], 0)
    rep = [((0, 2), (1, 3)), ((0, 2), (2, 3))]
    assert lop.lop_loss_eval(unit_chain(3, 1), 3, 1.0, 1.0, 0.0, rep)[0] == 7.0


def random_problem(rng, n_layers):
    layers, rows = [], int(rng.integers(4, 40))
    in_rows = rows
    for v in range(n_layers):
        src = v - 1
        parent_rows = in_rows if src < 0 else layers[src].n_ops
        k = int(rng.choice([1, 2, 3, 5])); s = int(rng.choice([1, 1, 2])); d = int(rng.choice([1, 1, 2]))
        p = int(rng.integers(0, (d * (k - 1)) // 2 + 1))
        n_ops = (parent_rows + 2 * p - d * (k - 1) - 1) // s + 1
        if n_ops < 2:
            k, s, p, d, n_ops = 1, 1, 0, 1, parent_rows
        res = -2
        cands = [u for u in range(-1, v) if (in_rows if u < 0 else layers[u].n_ops) == n_ops]
        if cands and rng.random() < 0.4:
            res = int(rng.choice(cands))
        layers.append(O.LossLayer(n_ops, src, res, k, s, p, d, *(float(x) for x in rng.random(4)),
                                  row_bytes=float(rng.integers(1, 2000))))
    return layers, in_rows, float(rng.integers(1, 3000))


def random_sched(rng, layers):
    out = []
    for L in layers:
        n = L.n_ops
        a = int(rng.integers(0, n + 1)); b = int(rng.integers(0, a + 1))
        m, r = (0, a), (b, n)
        if a == n and rng.random() < 0.5:
            r = (0, 0)
        if rng.random() < 0.3:                       # the roles of the devices swapped
            m, r = r, m
        if m[1] - m[0] <= 0 and r[1] - r[0] <= 0:
            m = (0, n)
        out.append(O.Alloc(m, r))
    return out


def test_evaluator_equals_oracle_on_random_chains():
    rng = np.random.Generator(np.random.PCG64(7))
    for trial in range(300):
        layers, in_rows, in_bytes = random_problem(rng, int(rng.integers(1, 9)))
        sched = random_sched(rng, layers)
        bw, lat = float(rng.uniform(1.0, 1e4)), float(rng.choice([0.0, 0.01]))
        try:
            want = O.evaluate(layers, in_rows, in_bytes, bw, lat, sched)
        except ValueError:
            with pytest.raises(lop.LopError):
                lop.lop_loss_eval(layers, in_rows, in_bytes, bw, lat, as_sched(sched))
            continue
        got = lop.lop_loss_eval(layers, in_rows, in_bytes, bw, lat, as_sched(sched))
        assert got[3] == want[3]
        np.testing.assert_allclose(got[0], want[0], rtol=1e-14)
        np.testing.assert_allclose(got[1], want[1], rtol=1e-14)
        np.testing.assert_allclose(got[2], want[2], rtol=1e-14)


def test_queued_link_evaluator_equals_oracle_on_random_chains():
    """The link model of the runtime stage (messages queue per direction, held rows are not
    resent) through the C ABI against the oracle's."""
    rng = np.random.Generator(np.random.PCG64(17))
    checked = 0
    for trial in range(300):
        layers, in_rows, in_bytes = random_problem(rng, int(rng.integers(1, 9)))
        sched = random_sched(rng, layers)
        bw, lat = float(rng.uniform(1.0, 1e4)), float(rng.choice([0.0, 0.01]))
        try:
            want = O.evaluate_queued(layers, in_rows, in_bytes, bw, lat, sched)
        except ValueError:
            continue
        got = lop.lop_loss_eval(layers, in_rows, in_bytes, bw, lat, as_sched(sched), lop.LOP_LINK_QUEUED)
        assert got[3] == want[3]
        np.testing.assert_allclose(got[0], want[0], rtol=1e-14)
        np.testing.assert_allclose(got[1], want[1], rtol=1e-14)
        np.testing.assert_allclose(got[2], want[2], rtol=1e-14)
        checked += 1
    assert checked > 100
    L = [O.LossLayer(4, -1, cm_row=0.25, cr_row=1, row_bytes=1),
         O.LossLayer(4, 0, residual_from=-1, cm_row=0.25, cr_row=1, row_bytes=1)]
    sched = [((0, 4), (0, 0)), ((0, 0), (0, 4))]
    assert lop.lop_loss_eval(L, 4, 1.0, 1.0, 0.0, sched, lop.LOP_LINK_QUEUED)[0] == 16.0   # hand-worked
    assert lop.lop_loss_eval(L, 4, 1.0, 1.0, 0.0, sched, lop.LOP_LINK_INDEPENDENT)[0] == 13.0
    with pytest.raises(lop.LopError):
        lop.lop_loss_eval(L, 4, 1.0, 1.0, 0.0, sched, 7)


def test_solver_with_the_queued_link_never_loses_to_one_device():
    layers, in_rows, in_bytes = chain_problem(workloads.resnet18_chain())
    for bw_mb in (2, 10, 50):
        bw = bw_mb * 1e6
        t_m = O.evaluate_queued(layers, in_rows, in_bytes, bw, 1e-3, O.all_on(layers, "M"))[0]
        t_r, _, _, v_r = O.evaluate_queued(layers, in_rows, in_bytes, bw, 1e-3, O.all_on(layers, "R"))
        sched, T, viol = lop.lop_loss_solve(layers, in_rows, in_bytes, bw, 1e-3, generations=100, seed=5,
                                            link_model=lop.LOP_LINK_QUEUED)
        assert viol == 0 and T <= t_m * (1 + 1e-12)
        if v_r == 0:
            assert T <= t_r * (1 + 1e-12)
        want = O.evaluate_queued(layers, in_rows, in_bytes, bw, 1e-3, [O.Alloc(m, r) for m, r in sched])
        assert want[0] == pytest.approx(T, rel=1e-14)


def test_errors():
    L = unit_chain()
    with pytest.raises(lop.LopError) as e:
        lop.lop_loss_eval(L, 3, 1.0, 1.0, 0.0, [((0, 1), (2, 3)), ((0, 3), (0, 0))])
    assert e.value.code == -4
    with pytest.raises(lop.LopError) as e:
        lop.lop_loss_eval(L, 3, 1.0, 0.0, 0.0, [((0, 3), (0, 0))] * 2)       # zero bandwidth
    assert e.value.code == -1


def test_solver_finds_the_brute_force_optimum_on_tiny_chains():
    rng = np.random.Generator(np.random.PCG64(3))
    for trial in range(6):
        layers = unit_chain(3, 1) + [O.LossLayer(3, 1, cm_row=1, cr_row=1, row_bytes=1)]
        for L in layers:
            L.cm_row = float(rng.uniform(0.5, 2.0)); L.cr_row = float(rng.uniform(0.05, 0.5))
            L.row_bytes = float(rng.uniform(0.5, 2.0))
        bw = float(rng.uniform(0.5, 8.0))
        best, _ = O.brute_force(layers, 3, 1.0, bw, 0.0)
        sched, T, viol = lop.lop_loss_solve(layers, 3, 1.0, bw, 0.0, population=40, generations=60, seed=trial)
        assert viol == 0
        assert T == pytest.approx(best, rel=1e-12)
        assert lop.lop_loss_eval(layers, 3, 1.0, bw, 0.0, sched)[0] == T
        again = lop.lop_loss_solve(layers, 3, 1.0, bw, 0.0, population=40, generations=60, seed=trial)
        assert again == (sched, T, viol)                                       # deterministic


def chain_problem(chain, flops_m=2e11, flops_r=2e13, launch_m=2e-5, launch_r=8e-6):
    """A workload chain as a scheduling problem: per-row cost from the operator's arithmetic at
    a sustained rate per device plus a launch cost; bytes per row from the tensor shapes."""
    shapes = planner.infer_shapes(chain)
    esz = 2 if chain.dtype == "bf16" else 4
    layers = []
    for i, L in enumerate(chain.layers):
        n, c, h, w = shapes[i]
        flop_row = planner.conv_flop(chain, shapes, i, 1)
        layers.append(O.LossLayer(h, L.input_from, L.residual_from, L.k[0], L.s[0], L.p[0], L.d[0],
                                  launch_m, flop_row / flops_m, launch_r, flop_row / flops_r,
                                  row_bytes=float(n * c * w * esz)))
    n, c, h, w = chain.in_shape
    return layers, h, float(n * c * w * esz)


@pytest.mark.parametrize("bw_mb", [1, 10, 50, 1000])
def test_solver_on_a_backbone_never_loses_to_one_device(bw_mb):
    layers, in_rows, in_bytes = chain_problem(workloads.resnet18_chain())
    bw = bw_mb * 1e6
    t_m = O.evaluate(layers, in_rows, in_bytes, bw, 1e-3, O.all_on(layers, "M"))[0]
    t_r, _, _, v_r = O.evaluate(layers, in_rows, in_bytes, bw, 1e-3, O.all_on(layers, "R"))
    sched, T, viol = lop.lop_loss_solve(layers, in_rows, in_bytes, bw, 1e-3, generations=150, seed=11)
    assert viol == 0
    assert T <= t_m * (1 + 1e-12)
    if v_r == 0:
        assert T <= t_r * (1 + 1e-12)
    want = O.evaluate(layers, in_rows, in_bytes, bw, 1e-3, [O.Alloc(m, r) for m, r in sched])
    assert want[0] == pytest.approx(T, rel=1e-14) and want[3] == 0

"""Pins of the schedule evaluator (Intra-DP Sec. IV-C, Eq. 2 and Eq. 3) against hand-worked
timelines shaped like the paper's workflow figure: two local operators of three operations,
one time unit per operation on either device and one per transmitted row."""
import math

import pytest

from oracle import loss
from oracle.loss import Alloc, LossLayer


def unit_chain(k2=1, p2=0):
    lo1 = LossLayer(3, -1, cm_row=1, cr_row=1, row_bytes=1)
    lo2 = LossLayer(3, 0, k=k2, p=p2, cm_row=1, cr_row=1, row_bytes=1)
    return [lo1, lo2]


def ev(layers, sched, bw=1.0, lat=0.0):
    return loss.evaluate(layers, 3, 1.0, bw, lat, sched)


def test_everything_on_the_device_is_the_sum_of_its_compute_times():
    t, s_m, s_r, viol = ev(unit_chain(), loss.all_on(unit_chain(), "M"))
    assert (t, s_m, viol) == (6.0, [0.0, 3.0, 6.0], 0)


def test_everything_on_the_server_pays_both_transfers_in_sequence():
    # input 3 rows up (3), LO1 (3), LO2 (3), result 3 rows down (3)
    t, s_m, s_r, _ = ev(unit_chain(), loss.all_on(unit_chain(), "R"))
    assert t == 12.0 and s_r == [3.0, 6.0]


def test_split_overlaps_transfer_and_compute():
    # M: rows 0,1 of both operators; R: row 2 of both. Row 2 of the input goes up during M's
    # LO1 (arrives 1, R finishes LO1 at 2, LO2 at 3), its result comes down at 4 = when M ends.
    sched = [Alloc((0, 2), (2, 3)), Alloc((0, 2), (2, 3))]
    t, s_m, s_r, _ = ev(unit_chain(), sched)
    assert (t, s_m, s_r) == (4.0, [0.0, 2.0, 4.0], [1.0, 2.0])


def test_block_wise_operator_needs_the_neighbours_rows():
    # LO2 reads rows r-1..r+1 of LO1: M misses row 2 (arrives 1+1+1 = 3), R misses row 1
    # (arrives 2+1 = 3); M ends at 5, R's row reaches M at 3+1+1 = 5
    sched = [Alloc((0, 2), (2, 3)), Alloc((0, 2), (2, 3))]
    t, s_m, s_r, _ = ev(unit_chain(3, 1), sched)
    assert (t, s_m, s_r) == (5.0, [0.0, 3.0, 5.0], [1.0, 3.0])


def test_replication_removes_the_transfer_of_the_replicated_row():
    # R also computes row 1 of LO1 (two input rows up: starts at 2, ends at 4), so its LO2
    # needs nothing from M; M still waits for row 2 (4 + 1 = 5) and ends at 7
    sched = [Alloc((0, 2), (1, 3)), Alloc((0, 2), (2, 3))]
    t, s_m, s_r, _ = ev(unit_chain(3, 1), sched)
    assert (t, s_m, s_r) == (7.0, [0.0, 5.0, 7.0], [2.0, 4.0])


def test_latency_bandwidth_and_fixed_costs():
    layers = unit_chain()
    layers[0].cr_fixed = 0.5
    sched = [Alloc((0, 2), (2, 3)), Alloc((0, 2), (2, 3))]
    t, _, s_r, _ = ev(layers, sched, bw=2.0, lat=0.25)
    # row 2 up: 0.25 + 1/2 = 0.75; R: LO1 0.75 .. 2.25, LO2 .. 3.25; down: 3.25 + 0.75 = 4.0
    assert s_r == [0.75, 2.25] and t == 4.0
    assert ev(layers, sched, bw=1e-3)[0] > ev(layers, sched, bw=1.0)[0]


def test_residual_edge_and_device_order():
    # v2 adds v0's rows to its own input v1 (identity edge): a device that has v1's rows but not
    # v0's must receive them; and a vertex waits for the previous one on its device
    v0 = LossLayer(4, -1, cm_row=1, cr_row=1, row_bytes=1)
    v1 = LossLayer(4, 0, cm_row=1, cr_row=1, row_bytes=1)
    v2 = LossLayer(4, 1, residual_from=0, cm_row=1, cr_row=1, row_bytes=1)
    sched = [Alloc((0, 4), (0, 0)), Alloc((0, 2), (2, 4)), Alloc((0, 2), (2, 4))]
    t, s_m, s_r, _ = loss.evaluate([v0, v1, v2], 4, 1.0, 1.0, 0.0, sched)
    # M: v0 0..4, v1 4..6, v2 6..8. R: v1 needs v0 rows 2,3 from M: 4 + 2 = 6, runs 6..8;
    # v2 needs v1 rows 2,3 (local, ready 8) and v0 rows 2,3 from M (4 + 2 = 6): starts 8, ends 10;
    # output rows 2,3 reach M at 10 + 2 = 12
    assert (s_m, s_r, t) == ([0.0, 4.0, 6.0, 12.0], [0.0, 6.0, 8.0], 12.0)


def test_constraints():
    layers = unit_chain()
    with pytest.raises(ValueError):
        ev(layers, [Alloc((0, 1), (2, 3)), Alloc((0, 3), (0, 0))])      # row 1 of LO1 nowhere
    with pytest.raises(ValueError):
        ev(layers, [Alloc((0, 4), (0, 0)), Alloc((0, 3), (0, 0))])      # outside OP(v)
    # transmission efficiency: LO1's output (3 rows x 2 bytes) exceeds the raw input (3 bytes),
    # so an edge out of it that carries rows is a violation
    layers[0].row_bytes = 2.0
    _, _, _, viol = ev(layers, [Alloc((0, 3), (0, 0)), Alloc((0, 2), (2, 3))])
    assert viol == 1
    _, _, _, viol = ev(layers, [Alloc((0, 2), (2, 3)), Alloc((0, 2), (2, 3))])
    assert viol == 0


def test_brute_force_optimum_beats_the_two_one_device_schedules():
    layers = unit_chain(3, 1)
    for L in layers:
        L.cr_row = 0.25                                   # the server is four times faster
    best, sched = loss.brute_force(layers, 3, 1.0, 2.0, 0.0)
    t_m = ev(layers, loss.all_on(layers, "M"), bw=2.0)[0]
    t_r = ev(layers, loss.all_on(layers, "R"), bw=2.0)[0]
    assert best <= min(t_m, t_r) and math.isfinite(best)
    assert ev(layers, sched, bw=2.0)[0] == best


# ---- the same model with the link shared as the runtime stage shares it (Sec. IV-D) ----
def test_queued_link_equals_the_recurrence_when_messages_never_meet():
    """On the timelines above no two messages of one direction are in flight together and no
    row is asked for twice, so sharing the link changes nothing."""
    sched = [Alloc((0, 2), (2, 3)), Alloc((0, 2), (2, 3))]
    for layers, s in ((unit_chain(), sched), (unit_chain(3, 1), sched),
                      (unit_chain(), loss.all_on(unit_chain(), "M")),
                      (unit_chain(), loss.all_on(unit_chain(), "R")),
                      (unit_chain(3, 1), [Alloc((0, 2), (1, 3)), Alloc((0, 2), (2, 3))])):
        assert loss.evaluate_queued(layers, 3, 1.0, 1.0, 0.0, s) == loss.evaluate(layers, 3, 1.0, 1.0, 0.0, s)


def test_queued_link_hand_worked_halo_example():
    """Two 3-row-window operators on 6 rows, M rows 0..2 and R rows 3..5 of both; 2 time units
    per row on M, 1 on R, 1 per transmitted row. By hand along Alg. 1 / Alg. 2:
    input rows 2..5 go up (0 -> 4); M's first operator 0 -> 6, R's 4 -> 7; row 3 comes down
    7 -> 8 and row 2 goes up 6 -> 7 (the up link has been free since 4); second operator: M
    8 -> 14, R 7 -> 10; R's three result rows come down 10 -> 13. T = 14."""
    layers = [LossLayer(6, -1, k=3, p=1, cm_row=2, cr_row=1, row_bytes=1),
              LossLayer(6, 0, k=3, p=1, cm_row=2, cr_row=1, row_bytes=1)]
    sched = [Alloc((0, 3), (3, 6))] * 2
    t, s_m, s_r, _ = loss.evaluate_queued(layers, 6, 1.0, 1.0, 0.0, sched)
    assert (t, s_m, s_r) == (14.0, [0.0, 8.0, 14.0], [4.0, 7.0])


def test_queued_link_makes_a_second_message_wait_for_the_first():
    """An element-wise operator on M, then one on R that also adds the chain input. The input's
    four rows go up first (0 -> 4, issued when the input exists); the first operator's rows are
    ready at 1 but the link is busy until 4, so they arrive at 8 (the recurrence as printed
    lets them arrive at 5); R computes 8 -> 12; the result comes down 12 -> 16 (13 as printed)."""
    layers = [LossLayer(4, -1, cm_row=0.25, cr_row=1, row_bytes=1),
              LossLayer(4, 0, residual_from=-1, cm_row=0.25, cr_row=1, row_bytes=1)]
    sched = [Alloc((0, 4), (0, 0)), Alloc((0, 0), (0, 4))]
    assert loss.evaluate_queued(layers, 4, 1.0, 1.0, 0.0, sched)[0] == 16.0
    assert loss.evaluate(layers, 4, 1.0, 1.0, 0.0, sched)[0] == 13.0


def test_queued_link_does_not_send_rows_twice():
    """Both operators on R: the input is sent once although two edges leave it (0 -> 4), R
    computes 4 -> 8 -> 12, the result comes down by 16; with a latency of 10 per message a
    second copy of the input would show."""
    layers = [LossLayer(4, -1, cm_row=0.25, cr_row=1, row_bytes=1),
              LossLayer(4, 0, residual_from=-1, cm_row=0.25, cr_row=1, row_bytes=1)]
    sched = loss.all_on(layers, "R")
    assert loss.evaluate_queued(layers, 4, 1.0, 1.0, 0.0, sched)[0] == 16.0
    assert loss.evaluate_queued(layers, 4, 1.0, 1.0, 10.0, sched)[0] == 36.0

"""Closed-form checks of the timing model of delayed transfers (a performance model:
"parity unpinned" beyond these cases)."""
import pytest

from oracle import schedule as sch
from oracle import transfer_sim as ts


def _sim(k, M, f, b, d, copy=0.0):
    dl = [d] * M
    return ts.simulate(sch.kfkb_order(k, M, 0), k, f, b, dl, dl, dl, dl, copy)


def test_no_delay_means_no_stall():
    for k in (1, 2, 4):
        r = _sim(k, 8, 1.0, 2.0, 0.0)
        assert r["stall"] == pytest.approx(0.0) and r["compute_end"] == pytest.approx(8 * 3.0)


def test_1f1b_exposes_two_delays_per_microbatch():
    """k = 1: B(mb) needs dY_mb, which starts only after Y_mb is sent: each micro-batch waits
    2 delays; the first input adds one more."""
    f, b, d, M = 1.0, 2.0, 0.4, 8
    r = _sim(1, M, f, b, d)
    assert r["compute_end"] == pytest.approx(d + M * (f + b + 2 * d))


def test_group_of_k_hides_delay_behind_the_other_forwards():
    """Per group the exposed wait is max(0, 2 d - (k-1) f) while a transfer is shorter than a
    forward (Section 4.1: the second computation overlaps the transfer of the first)."""
    f, b, M = 1.0, 2.0, 8
    for k in (2, 4):
        for d in (0.2, 0.45):
            r = _sim(k, M, f, b, d)
            groups = M // k
            assert r["compute_end"] == pytest.approx(d + M * (f + b) + groups * max(0.0, 2 * d - (k - 1) * f))
    # paper's analysis setting: B = 2F, transfer = F/2: 2F2B is shorter than 1F1B
    assert _sim(2, M, 1.0, 2.0, 0.5)["total"] < _sim(1, M, 1.0, 2.0, 0.5)["total"]


def test_prefetched_input_absorbs_a_slow_transfer():
    """Section 4.4: an input that already sits in the queue costs nothing even if its own
    transfer was slow."""
    M, k = 8, 4
    order = sch.kfkb_order(k, M, 0)
    zero = [0.0] * M
    slow = list(zero); slow[5] = 2.5            # X_5 is slow but is sent one group ahead
    base = ts.simulate(order, k, 1.0, 2.0, zero, zero, zero, zero)
    r = ts.simulate(order, k, 1.0, 2.0, slow, zero, zero, zero)
    assert r["compute_end"] == pytest.approx(base["compute_end"])


def test_receive_plan_is_a_permutation_feeding_the_order():
    for M in (4, 8, 9):
        for k in (1, 2, 4):
            for w in (0, 1, 2):
                order = sch.kfkb_order(k, M, w)
                d = [0.1] * M
                for ahead in (False, True, None):
                    if ahead is not None:
                        plan = ts.receive_plan(order, ahead)
                        assert sorted(plan) == sorted(order)
                        if not ahead:
                            assert plan == list(order)
                    ts.simulate(order, k, 1.0, 2.0, d, d, d, d, inputs_ahead=ahead)      # never starves


def test_consumption_order_keeps_a_backward_unit_from_waiting_behind_the_next_inputs():
    """Receives of one stream complete one after the other (Section 5.3).  With inputs ahead the k input transfers of
    the next forward unit sit in front of the first upstream gradient of the current backward unit; in consumption
    order they follow it and arrive while the backwards run.  Worked case: k = 2, M = 4, every transfer 3, F = 1, B = 2.
    Consumption order: X0 3, X1 6 | F0 3-4, F1 6-7 | Y0 sent 7, Y1 sent 10 | dY0 10, dY1 13 | B0 10-12, B1 13-15 |
    X2 16, X3 19 (behind dY1) | F2 16-17, F3 19-20 | Y2 sent 20 (the send stream carried dX0 until 15, dX1 until 18;
    Y2 goes 18-21: F2 ended 17) ...  The exact totals are left to the simulator; what the rule fixes is the ORDER of
    arrivals, checked here, and that the first backward starts earlier than with inputs ahead."""
    M, k, d = 4, 2, [3.0] * 4
    order = sch.kfkb_order(k, M, 0)
    cons = ts.simulate(order, k, 1.0, 2.0, d, d, d, d, inputs_ahead=False)
    ahead = ts.simulate(order, k, 1.0, 2.0, d, d, d, d, inputs_ahead=True)
    i_b0 = order.index((sch.B, 0))
    # consumption order: dY0 is the third receive: it starts when Y0 has been sent (F0 3-4, sent at 7) -> arrives 10
    assert cons["start"][i_b0] == pytest.approx(10.0)
    # inputs ahead: X2 and X3 (3 each, from 6 on) come first: dY0 is received 12-15
    assert ahead["start"][i_b0] == pytest.approx(15.0)
    assert cons["total"] < ahead["total"]


def test_default_receive_list_is_inputs_ahead_for_1f1b_only():
    d = [0.7] * 8
    for k, ahead in ((1, True), (2, False), (4, False)):
        order = sch.kfkb_order(k, 8, 0)
        a = ts.simulate(order, k, 1.0, 2.0, d, d, d, d)
        b = ts.simulate(order, k, 1.0, 2.0, d, d, d, d, inputs_ahead=ahead)
        assert a["start"] == b["start"] and a["total"] == b["total"]

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
                plan = ts.receive_plan(order)
                assert sorted(plan) == sorted(order)
                d = [0.1] * M
                ts.simulate(order, k, 1.0, 2.0, d, d, d, d)      # never starves

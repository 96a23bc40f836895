"""Pins of the oracle's cost model / tuner (paper Sections 3.2.2, 4.3, 5.2, 5.4): closed forms and invariants.
It is a heuristic: beyond these cases it is "parity unpinned"."""
import pytest

from oracle import tuner as tu


def test_window_is_a_moving_average_of_the_last_samples():
    w = tu.Window(3)
    assert w.mean() == 0.0
    for v, want in [(3.0, 3.0), (6.0, 4.5), (0.0, 3.0), (9.0, 5.0), (9.0, 6.0)]:
        w.push(v)
        assert w.mean() == pytest.approx(want)              # the first sample has dropped out by the fourth
    with pytest.raises(ValueError):
        tu.Window(0)


def test_estimate_without_communication_is_the_sum_of_the_stage_times():
    comm = {d: 0.0 for d in tu.DIRECTIONS}
    for k in (1, 2, 4, 8):
        assert tu.predict(k, 8, 0, 1.0, 2.0, comm) == pytest.approx(8 * 3.0)


def test_estimate_of_1f1b_exposes_two_transfers_per_microbatch():
    d, M, f, b = 0.4, 8, 1.0, 2.0
    comm = {x: d for x in tu.DIRECTIONS}
    # compute ends at d + M (f + b + 2 d) (Section 2.5); the last dX still has to be sent
    assert tu.predict(1, M, 0, f, b, comm) == pytest.approx(d + M * (f + b + 2 * d) + d)


def test_choice_without_delay_is_the_smallest_candidate_and_grows_with_delay():
    M, f, b = 16, 1.0, 2.0
    prof = {k: (f, b) for k in (1, 2, 4, 8)}
    k, est = tu.choose(prof, M, 0, prof, {d: 0.0 for d in tu.DIRECTIONS})
    assert k == 1 and len(set(round(v, 9) for v in est.values())) == 1      # a tie: least memory wins
    # d = 0.3: 2 d <= (k - 1) f already for k = 2, every k >= 2 hides the transfers completely (Section 4.1):
    # d (first input) + M (f + b) + d (last dX), while 1F1B pays 2 d per micro-batch on top
    d = 0.3
    k_small, est = tu.choose(prof, M, 0, prof, {x: d for x in tu.DIRECTIONS})
    assert k_small == 2
    for kk in (2, 4, 8):
        assert est[kk] == pytest.approx(2 * d + M * (f + b))
    assert est[1] == pytest.approx(2 * d + M * (f + b + 2 * d))
    # transfers about as long as a forward: two forwards no longer hide two transfers, four do better
    k_big, est = tu.choose(prof, M, 0, prof, {x: 0.9 for x in tu.DIRECTIONS})
    assert k_big == 4 and est[1] > est[2] > est[4]
    # a plan whose groups compute more slowly loses even if it hides the transfers as well
    prof_slow = dict(prof); prof_slow[4] = (1.5, 3.0)
    assert tu.choose(prof, M, 0, prof_slow, {x: 0.9 for x in tu.DIRECTIONS})[0] != 4


def test_choice_respects_the_activation_limit():
    M, prof = 16, {k: (1.0, 2.0) for k in (1, 2, 4, 8)}
    comm = {d: 3.0 for d in tu.DIRECTIONS}
    assert tu.choose(prof, M, 0, prof, comm, mem_limit=4 * 10, per_mb_bytes=10)[0] == 4      # k = 8 needs 80
    assert tu.choose(prof, M, 1, prof, comm, mem_limit=4 * 10, per_mb_bytes=10)[0] == 2      # one warm-up group doubles the live set
    with pytest.raises(ValueError):
        tu.choose(prof, M, 0, prof, comm, mem_limit=5, per_mb_bytes=10)


def test_tuner_switches_only_at_its_interval_and_on_the_window_mean():
    M, prof = 8, {k: (1.0, 2.0) for k in (1, 2, 4)}
    t = tu.Tuner([1, 2, 4], M, 0, prof, window=2, interval=3)
    quiet = {d: [0.0] * M for d in tu.DIRECTIONS}
    busy = {d: [1.5] * M for d in tu.DIRECTIONS}
    ks = []
    for it in range(15):
        ks.append(t.next_k())
        t.observe(busy if 3 <= it < 8 else quiet)
    # evaluations happen before iterations 3, 6, 9, 12 on the mean of the last two iterations:
    # (1, 2) quiet -> 1;  (4, 5) busy -> 4;  (7, 8) busy, quiet: mean 0.75 -> still 4;  (10, 11) quiet -> 1
    assert ks == [1] * 6 + [4] * 6 + [1] * 3
    assert t.last_estimates[1] == pytest.approx(M * 3.0)

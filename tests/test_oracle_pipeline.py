"""Pins of the oracle's S-stage pipeline: per-stage plans, dependencies, the invariance of the result
under S and k (Section 1: the plans are mathematically equivalent), the memory gradient over the
stages (Section 3.2.1) and the closed forms of the timing model."""
import numpy as np
import pytest

import kfkb_synth as synth
from oracle import pipeline as pl
from oracle import schedule as sch

F, B = sch.F, sch.B


@pytest.mark.parametrize("S", [1, 2, 3, 4])
def test_list_schedule_is_every_stage_plan_in_a_valid_global_order(S):
    for M in range(1, 9):
        for k in range(1, M + 1):
            order = pl.list_schedule(S, k, M)
            assert len(order) == 2 * M * S and len(set(order)) == len(order)
            for s in range(S):                      # the ops of stage s, in the order they are issued, are its plan
                assert [(op, mb) for st, op, mb in order if st == s] == \
                    sch.kfkb_order(k, M, sch.warmup_groups(S, s, k, M))
            pos = {e: i for i, e in enumerate(order)}
            for s in range(S):
                for mb in range(M):
                    assert pos[(s, F, mb)] < pos[(s, B, mb)]
                    if s > 0:
                        assert pos[(s - 1, F, mb)] < pos[(s, F, mb)]     # activations flow down the pipeline
                        assert pos[(s, B, mb)] < pos[(s - 1, B, mb)]     # gradients flow back up


def test_one_stage_is_the_stage_plan():
    for M in range(1, 7):
        for k in range(1, M + 1):
            assert pl.list_schedule(1, k, M) == [(0, op, mb) for op, mb in sch.kfkb_order(k, M, 0)]


def test_2_stage_1f1b_written_out():
    # two stages, three micro-batches, 1F1B (stage 0 warms up with one forward), forward 1 and backward 2 time
    # units, worked by hand: F0 [0,1) on stage 0; stage 1 F0 [1,2) (tie at 1 goes to the later stage), stage 0 F1
    # [1,2); stage 1 B0 [2,4); at 4 both stage 1 F1 and stage 0 B0 can start, the later stage goes first; ...
    assert pl.list_schedule(2, 1, 3) == [
        (0, F, 0), (1, F, 0), (0, F, 1), (1, B, 0), (1, F, 1), (0, B, 0), (1, B, 1), (0, F, 2), (1, F, 2),
        (0, B, 1), (1, B, 2), (0, B, 2)]
    assert pl.simulate(2, 1, 3, 1, 2) == 12


@pytest.mark.parametrize("S,k", [(1, 2), (2, 1), (2, 2), (3, 1), (3, 2), (3, 6), (6, 3)])
def test_result_does_not_depend_on_stages_or_k(S, k):
    L, H, heads, T, b, M = 6, 16, 2, 6, 2, 6
    blocks = synth.stage_weights(L, H, 4 * H, "f32")
    xs = [synth.microbatch_inputs(mb, b, T, H, "f32") for mb in range(M)]
    dys = [synth.microbatch_upstream_grads(mb, b, T, H, "f32") for mb in range(M)]
    Gr, Yr, dXr, _ = sch.run_iteration(sch.kfkb_order(1, M, 0), blocks, xs, dys, heads)
    G, Y, dX, max_live, order = pl.run_pipeline(S, k, blocks, xs, dys, heads)
    for mb in range(M):                              # same arithmetic in the same order per block: identical bits
        assert np.array_equal(Y[mb], Yr[mb]) and np.array_equal(dX[mb], dXr[mb])
    for l in range(L):
        for n in synth.PARAM_ORDER:
            assert np.array_equal(G[l][n], Gr[l][n]), (l, n)
    # Section 3.2.1: a stage holds (w + 1) k micro-batches at its peak, more towards the front of the pipeline
    for s in range(S):
        w = sch.warmup_groups(S, s, k, M)
        assert max_live[s] == min((w + 1) * k, M)
    assert max_live == sorted(max_live, reverse=True)


def test_timing_closed_forms_without_transfer_time():
    f, b = 1.0, 2.0
    for S in range(1, 6):
        for M in range(S, 13):
            assert pl.simulate(S, 1, M, f, b) == pytest.approx((M + S - 1) * (f + b))      # 1F1B
            assert pl.simulate(S, M, M, f, b) == pytest.approx((M + S - 1) * (f + b))      # GPipe
    for M in range(1, 9):
        for k in range(1, M + 1):
            assert pl.simulate(1, k, M, f, b) == pytest.approx(M * (f + b))                # one stage: no bubble


def test_timing_grows_with_transfer_time_and_groups_absorb_it():
    # Section 3.2.1 / Figure "kFkB": with k forwards in a row a stage has k - 1 micro-batches of work to do while
    # the first one's output and its gradient travel; 1F1B has none and pays every round trip
    S, M, f, b = 2, 8, 1.0, 2.0
    for k in (1, 2, 4):
        ts = [pl.simulate(S, k, M, f, b, c) for c in (0.0, 0.5, 1.0, 2.0)]
        assert ts == sorted(ts)
    c = 1.0
    assert pl.simulate(S, 4, M, f, b, c) < pl.simulate(S, 1, M, f, b, c)
    # the last stage of a two-stage 1F1B pipeline waits one round trip (2 c) per micro-batch once it is the bottleneck
    assert pl.simulate(S, 1, M, f, b, c) >= M * (f + b) + 2 * c

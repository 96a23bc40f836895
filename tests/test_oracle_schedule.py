"""Pins of the oracle's kFkB order and iteration against the identities the paper states."""
import numpy as np
import pytest

import kfkb_synth as synth
from oracle import schedule as sch
from oracle import stage_math as sm

F, B = sch.F, sch.B


def _hand_1f1b_last_stage(M):
    out = []
    for i in range(M):
        out += [(F, i), (B, i)]
    return out


def test_k1_is_1f1b():                       # Section 1: k = 1 is the special case 1F1B
    for M in range(1, 9):
        assert sch.kfkb_order(1, M, 0) == _hand_1f1b_last_stage(M)
        for w in range(0, 4):
            assert sch.kfkb_order(1, M, w) == sch.one_f_one_b_order(M, w)
    # a stage two hops from the end, written out by hand
    assert sch.kfkb_order(1, 4, 2) == [(F, 0), (F, 1), (F, 2), (B, 0), (F, 3), (B, 1), (B, 2), (B, 3)]


def test_k_equals_M_is_gpipe():              # Section 1 / 4.1: k = M degenerates to GPipe
    for M in range(1, 9):
        for w in range(0, 3):
            assert sch.kfkb_order(M, M, w) == [(F, i) for i in range(M)] + [(B, i) for i in range(M)]


def test_2f2b_written_out():
    assert sch.kfkb_order(2, 4, 0) == [(F, 0), (F, 1), (B, 0), (B, 1), (F, 2), (F, 3), (B, 2), (B, 3)]
    assert sch.kfkb_order(3, 7, 0) == [(F, 0), (F, 1), (F, 2), (B, 0), (B, 1), (B, 2),
                                        (F, 3), (F, 4), (F, 5), (B, 3), (B, 4), (B, 5), (F, 6), (B, 6)]


def test_two_definitions_agree():            # Section 5.4: k cross-merged copies of 1F1B
    for M in range(1, 14):
        for k in range(1, M + 1):
            for w in range(0, 5):
                if M % k == 0 or w == 0:
                    assert sch.kfkb_order(k, M, w) == sch.kfkb_order_by_interleave(k, M, w), (k, M, w)


def test_structure_and_live_count():
    for M in range(1, 14):
        for k in range(1, M + 1):
            for w in range(0, 4):
                order = sch.kfkb_order(k, M, w)
                assert len(order) == 2 * M
                pos = {op_mb: i for i, op_mb in enumerate(order)}
                for mb in range(M):
                    assert pos[(F, mb)] < pos[(B, mb)]
                assert [mb for op, mb in order if op == B] == list(range(M))     # accumulation order
                assert [mb for op, mb in order if op == F] == list(range(M))
                G = -(-M // k)
                assert sch.peak_live(order) == min((min(w, G) + 1) * k, M)
                # early backward: once the warm-up is over, a full forward group is followed
                # at once by the oldest pending backward group
                lc = sch.live_counts(order)
                assert min(lc[:-1] + [1]) >= 0 and lc[-1] == 0


def test_memory_grows_with_k():              # Section 3.1: 1F1B is the most memory-efficient
    per = sch.activation_bytes_per_microbatch(6, 4, 1024, 1024, 16, 4096, 2)
    # 16 n elements of bf16 + fp32 statistics, n = b T H
    n = 4 * 1024 * 1024
    assert per == 6 * (16 * n * 2 + (4 * 4096 + 4 * 16 * 1024) * 4)
    # with the LayerNorm outputs and the GELU output recomputed: 10 n elements (Section 2.2: more micro-batches fit)
    rec = sch.activation_bytes_per_microbatch(6, 4, 1024, 1024, 16, 4096, 2, recompute=True)
    assert rec == 6 * (10 * n * 2 + (4 * 4096 + 4 * 16 * 1024) * 4)
    assert sch.largest_admissible_k(16, 0, 4 * per, rec) == 4 and sch.largest_admissible_k(16, 0, 8 * rec, rec) == 8
    assert 8 * rec < 6 * per                 # what held 5 micro-batches now holds 8
    sizes = [sch.plan_activation_bytes(k, 16, 0, 6, 4, 1024, 1024, 16, 4096, 2) for k in (1, 2, 4, 8, 16)]
    assert sizes == sorted(sizes) and sizes[0] == per and sizes[-1] == 16 * per
    assert sch.largest_admissible_k(16, 0, 4 * per, per) == 4
    assert sch.largest_admissible_k(16, 0, 5 * per, per) == 4
    assert sch.largest_admissible_k(16, 0, per - 1, per) == 0
    # first stage of eight (w = 7), 32 micro-batches, room for 20: k = 1 holds 8, k = 2 holds 16, k = 4 all 32
    assert sch.largest_admissible_k(32, 7, 20 * per, per) == 2


@pytest.fixture(scope="module")
def tiny():
    L, b, T, H, heads, Fm, M = 2, 2, 6, 16, 4, 64, 4
    blocks = synth.stage_weights(L, H, Fm, "f64", std=0.1)
    xs = [synth.microbatch_inputs(mb, b, T, H, "f64") for mb in range(M)]
    dys = [synth.microbatch_upstream_grads(mb, b, T, H, "f64") for mb in range(M)]
    return blocks, xs, dys, heads


def test_every_k_gives_the_full_batch_gradient(tiny):
    """Synchronous pipeline training is a reordering (Section 2.2): the accumulated gradient of
    any kFkB plan equals the gradient of one pass over all micro-batches concatenated."""
    blocks, xs, dys, heads = tiny
    M = len(xs)
    xf, dyf = np.concatenate(xs, 0), np.concatenate(dys, 0)
    yf, caches = sm.stage_fwd(xf, blocks, heads)
    dxf, gf = sm.stage_bwd(dyf, blocks, caches, heads)
    ref = None
    for k in (1, 2, 3, 4):
        for w in (0, 1):
            G, Y, dX, live = sch.run_iteration(sch.kfkb_order(k, M, w), blocks, xs, dys, heads)
            assert live == sch.peak_live(sch.kfkb_order(k, M, w))
            assert np.allclose(np.concatenate(Y, 0), yf, rtol=0, atol=1e-13)
            assert np.allclose(np.concatenate(dX, 0), dxf, rtol=0, atol=1e-13)
            for l in range(len(blocks)):
                for n in synth.PARAM_ORDER:
                    err = np.linalg.norm(G[l][n] - gf[l][n]) / np.linalg.norm(gf[l][n])
                    assert err < 1e-12, (k, w, l, n, err)
            if ref is None:
                ref = G
            else:                               # same backward order => bit-identical sums
                for l in range(len(blocks)):
                    for n in synth.PARAM_ORDER:
                        assert np.array_equal(G[l][n], ref[l][n])


def test_iteration_rejects_bad_orders(tiny):
    blocks, xs, dys, heads = tiny
    with pytest.raises(RuntimeError):
        sch.run_iteration([(B, 0)], blocks, xs, dys, heads)
    with pytest.raises(RuntimeError):
        sch.run_iteration([(F, 0), (F, 0)], blocks, xs, dys, heads)
    with pytest.raises(ValueError):
        sch.kfkb_order(0, 4)
    with pytest.raises(ValueError):
        sch.kfkb_order(5, 4)


def test_candidates_on_the_memory_limit_curve():
    """Section 4.2 (pruning) and the granularity test of Section 6.2.1: global batch 192, k = 1..6 run with
    micro-batch size 6 // k, i.e. a device that holds six samples per warm-up group."""
    for S, s in ((1, 0), (8, 0), (8, 5)):
        w = S - 1 - s
        got = sch.enumerate_candidates(192, (w + 1) * 6 * 10, 10, S, s, k_max=6)
        assert got == [(k, 6 // k) for k in range(1, 7)]
    # brute force on small cases: every candidate fits, the next larger divisor does not, nothing after the
    # walk's end fits with b = 1
    for G in (12, 16, 30):
        for limit in (35, 80, 240, 10 ** 6):
            for S, s in ((1, 0), (4, 0), (4, 2)):
                cand = sch.enumerate_candidates(G, limit, 10, S, s)

                def need(k, b):
                    M = G // b
                    return sch.peak_live(sch.kfkb_order(k, M, sch.warmup_groups(S, s, k, M))) * b * 10
                ks = [k for k, _ in cand]
                assert ks == list(range(1, len(cand) + 1))
                for k, b in cand:
                    assert G % b == 0 and G // b >= k and need(k, b) <= limit
                    bigger = [bb for bb in range(b + 1, G + 1) if G % bb == 0 and G // bb >= k]
                    assert all(need(k, bb) > limit for bb in bigger)
                k_next = len(cand) + 1
                if k_next <= G:
                    assert need(k_next, 1) > limit
    # no limit worth the name: k = 1 takes the whole batch as one micro-batch, k = 2 halves it, ...
    assert sch.enumerate_candidates(12, 10 ** 9, 10)[:4] == [(1, 12), (2, 6), (3, 4), (4, 3)]
    assert sch.enumerate_candidates(12, 5, 10) == []

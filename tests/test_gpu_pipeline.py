"""The pipeline of S virtual stages on one GPU (run_pipeline_kFkB) through the C boundary: results against
the oracle's pipeline iteration and, bit for bit, against run_kFkB on the whole stage; per-stage executed order
against every stage's kFkB plan; dependencies and injected boundary delays in the measured times."""
import numpy as np
import pytest
import torch

import kfkb_synth as synth
import paper_2303_01675_amd as kf
from oracle import pipeline as pl
from oracle import schedule as sch
from _util import NAME, assert_close

pytestmark = pytest.mark.gpu


def _make(dt, L, H, heads, T, b, M):
    blocks = synth.stage_weights(L, H, 4 * H, NAME[dt])
    xs = [synth.microbatch_inputs(mb, b, T, H, NAME[dt]) for mb in range(M)]
    dys = [synth.microbatch_upstream_grads(mb, b, T, H, NAME[dt]) for mb in range(M)]
    st = kf.StageBuffers(blocks, dt, heads, T, b, M, k_max=M)      # one activation slot per micro-batch
    st.set_inputs(xs, dys)
    return st, blocks, xs, dys


def _bind(S, M):
    buf = torch.empty(max(kf.stage_pipeline_bytes(S, M), 256), dtype=torch.uint8, device="cuda")
    kf.stage_pipeline_bind(buf, S, M)
    return buf


def _run_pipeline(st, k, M):
    kf.stage_zero_grads()
    kf.run_pipeline_kFkB(k)
    kf.stage_sync()
    return (st.grads.clone(), st.h_out[:M].clone(), st.h_ingrad[:M].clone()), kf.stage_get_pipeline_order()


@pytest.mark.parametrize("dt,L,H,heads,T,b,M", [(kf.F32, 4, 128, 4, 64, 2, 4), (kf.BF16, 6, 128, 2, 96, 2, 6)])
def test_pipeline_matches_oracle_and_the_single_stage_bit_for_bit(dt, L, H, heads, T, b, M):
    st, blocks, xs, dys = _make(dt, L, H, heads, T, b, M)
    kf.stage_zero_grads()
    kf.run_kFkB(1, M, 0)
    kf.stage_sync()
    whole = (st.grads.clone(), st.h_out[:M].clone(), st.h_ingrad[:M].clone())
    for S in [s for s in (1, 2, 3, L) if L % s == 0]:
        keep = _bind(S, M)
        for k in sorted({1, 2, M}):
            got, order = _run_pipeline(st, k, M)
            for a, b_ in zip(whole, got):                       # same kernels, same accumulation order per block
                assert torch.equal(a, b_), (S, k)
            # the issue order is the library's list schedule, and every stage's part of it is that stage's kFkB plan
            issued = [(s, o, mb) for s, o, mb, _, _ in order]
            assert issued == pl.list_schedule(S, k, M)
            for s in range(S):
                assert [(o, mb) for v, o, mb in issued if v == s] == sch.kfkb_order(k, M, sch.warmup_groups(S, s, k, M))
            # measured times respect the data flow between the stages
            t = {(s, o, mb): (t0, t1) for s, o, mb, t0, t1 in order}
            for s in range(S):
                for mb in range(M):
                    assert t[(s, "F", mb)][1] <= t[(s, "B", mb)][0] + 1e-3
                    if s > 0:
                        assert t[(s - 1, "F", mb)][1] <= t[(s, "F", mb)][0] + 1e-3
                        assert t[(s, "B", mb)][1] <= t[(s - 1, "B", mb)][0] + 1e-3
        del keep
    # against the oracle's pipeline iteration (and through it the plain definition), at the parity tolerance
    S, k = 2, 2
    keep = _bind(S, M)
    _run_pipeline(st, k, M)
    Gr, Yr, dXr, _, _ = pl.run_pipeline(S, k, blocks, xs, dys, heads)
    Y, dX = st.outputs(M)
    G = st.gradients()
    for mb in range(M):
        assert_close(Y[mb], Yr[mb], dt, "Y[%d]" % mb)
        assert_close(dX[mb], dXr[mb], dt, "dX[%d]" % mb)
    for l in range(L):
        for n in synth.PARAM_ORDER:
            assert_close(G[l][n], Gr[l][n], dt, "grad block %d %s" % (l, n))
    st.close()


def test_boundary_delays_change_timing_not_results_and_a_run_can_follow_a_run():
    dt, L, H, heads, T, b, M, S = kf.BF16, 4, 128, 2, 64, 2, 4, 2
    st, blocks, xs, dys = _make(dt, L, H, heads, T, b, M)
    keep = _bind(S, M)
    base, _ = _run_pipeline(st, 2, M)
    d_ms = 3.0
    kf.stage_set_pipeline_delays(np.full((S - 1) * M, int(d_ms * 1e6)), np.full((S - 1) * M, int(d_ms * 1e6)))
    for k in (1, 2, 4):
        got, order = _run_pipeline(st, k, M)
        for a, b_ in zip(base, got):
            assert torch.equal(a, b_)
        t = {(s, o, mb): (t0, t1) for s, o, mb, t0, t1 in order}
        for mb in range(M):                                      # a crossing takes at least the injected delay
            assert t[(1, "F", mb)][0] >= t[(0, "F", mb)][1] + 0.9 * d_ms
            assert t[(0, "B", mb)][0] >= t[(1, "B", mb)][1] + 0.9 * d_ms
    kf.stage_set_pipeline_delays(None, None)
    # the single-stage entry points still work on the same binding afterwards
    kf.stage_zero_grads()
    kf.run_kFkB(2, M, 0)
    kf.stage_sync()
    for a, b_ in zip(base, (st.grads, st.h_out[:M], st.h_ingrad[:M])):
        assert torch.equal(a, b_)
    del keep
    st.close()


def test_pipeline_errors():
    dt, L, H, heads, T, b, M = kf.F32, 4, 128, 4, 64, 2, 4
    blocks = synth.stage_weights(L, H, 4 * H, NAME[dt])
    st = kf.StageBuffers(blocks, dt, heads, T, b, M, k_max=1)       # a workspace with ONE activation slot
    buf = torch.empty(max(kf.stage_pipeline_bytes(2, M), 256), dtype=torch.uint8, device="cuda")
    with pytest.raises(kf.KfkbError) as e:
        kf.stage_pipeline_bind(buf, 2, M)
    assert e.value.code == -3
    st.close()
    st = kf.StageBuffers(blocks, dt, heads, T, b, M, k_max=M)
    with pytest.raises(kf.KfkbError):
        kf.stage_pipeline_bind(buf, 3, M)                            # 4 blocks do not divide into 3 stages
    with pytest.raises(kf.KfkbError):
        kf.stage_pipeline_bind(torch.empty(256, dtype=torch.uint8, device="cuda"), 2, M)    # buffer too small
    with pytest.raises(kf.KfkbError):
        kf.run_pipeline_kFkB(1)                                      # not bound
    kf.stage_pipeline_bind(buf, 2, M)
    with pytest.raises(kf.KfkbError):
        kf.run_pipeline_kFkB(M + 1)
    st.close()


def test_pipeline_with_recomputation_in_fp16():
    """The options compose: fp16 storage, activation recomputation and the pipeline of virtual stages give the bits
    of the plain single-stage run of the same configuration, within the fp16 bar of the oracle."""
    dt, L, H, heads, T, b, M, S = kf.F16, 4, 128, 2, 64, 2, 4, 2
    blocks = synth.stage_weights(L, H, 4 * H, NAME[dt])
    xs = [synth.microbatch_inputs(mb, b, T, H, NAME[dt]) for mb in range(M)]
    dys = [synth.microbatch_upstream_grads(mb, b, T, H, NAME[dt]) for mb in range(M)]
    st = kf.StageBuffers(blocks, dt, heads, T, b, M, k_max=M, recompute=1)
    st.set_inputs(xs, dys)
    kf.stage_zero_grads()
    kf.run_kFkB(2, M, 0)
    kf.stage_sync()
    whole = (st.grads.clone(), st.h_out[:M].clone(), st.h_ingrad[:M].clone())
    keep = _bind(S, M)
    for k in (1, 2):
        got, order = _run_pipeline(st, k, M)
        for a, b_ in zip(whole, got):
            assert torch.equal(a, b_)
    Gr, Yr, dXr, _, _ = pl.run_pipeline(S, 2, blocks, xs, dys, heads)
    Y, dX = st.outputs(M)
    G = st.gradients()
    for mb in range(M):
        assert_close(Y[mb], Yr[mb], dt, "Y[%d]" % mb)
        assert_close(dX[mb], dXr[mb], dt, "dX[%d]" % mb)
    for l in range(L):
        for n in synth.PARAM_ORDER:
            assert_close(G[l][n], Gr[l][n], dt, "grad block %d %s" % (l, n))
    del keep
    st.close()

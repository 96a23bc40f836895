"""The candidate plans (k, b) on the memory-limit curve (paper Section 4.2; the granularity test of Section 6.2.1
walks k = 1..6 with micro-batch size 6 // k at a fixed global batch): every candidate the library enumerates is
bound and run, and all of them must give the same training step, namely per-sample outputs and input gradients,
and the accumulated gradient, equal to the oracle's full-batch result (the paper's "mathematically equivalent")."""
import numpy as np
import pytest
import torch

import kfkb_synth as synth
import paper_2303_01675_amd as kf
from oracle import schedule as sch
from oracle import stage_math as sm
from _util import NAME, assert_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dt,H,heads,T", [(kf.F32, 64, 2, 24), (kf.BF16, 128, 2, 96)])
def test_every_candidate_plan_gives_the_same_step(dt, H, heads, T):
    L, GB = 2, 12
    esz = 4 if dt == kf.F32 else 2
    per_sample = kf.kfkb_activation_bytes_per_microbatch(L, 1, T, H, heads, 4 * H, esz)
    assert per_sample == sch.activation_bytes_per_microbatch(L, 1, T, H, heads, 4 * H, esz)
    limit = 6 * per_sample                                   # room for six samples' activations, as in Section 6.2.1
    cands = kf.kfkb_enumerate_candidates(GB, limit, per_sample, k_max=6)
    assert cands == sch.enumerate_candidates(GB, limit, per_sample, k_max=6)
    assert cands == [(1, 6), (2, 3), (3, 2), (4, 1), (5, 1), (6, 1)]      # b = largest divisor of 12 that is <= 6 // k
    blocks = synth.stage_weights(L, H, 4 * H, NAME[dt])
    X = np.concatenate([synth.microbatch_inputs(i, 1, T, H, NAME[dt]) for i in range(GB)], axis=0)      # [GB, T, H]
    dY = np.concatenate([synth.microbatch_upstream_grads(i, 1, T, H, NAME[dt]) for i in range(GB)], axis=0)
    # the oracle's step: one pass over the whole batch
    Yr, caches = sm.stage_fwd(X, blocks, heads, True)
    dXr, Gr = sm.stage_bwd(dY, blocks, caches, heads)
    first = None
    for k, b in cands:
        M = GB // b
        st = kf.StageBuffers(blocks, dt, heads, T, b, M, k)
        st.set_inputs([X[mb * b:(mb + 1) * b] for mb in range(M)], [dY[mb * b:(mb + 1) * b] for mb in range(M)])
        assert kf.stage_activation_bytes(k, M) == k * b * per_sample <= limit
        kf.stage_zero_grads()
        kf.run_kFkB(k, M, limit)
        kf.stage_sync()
        assert [(o, mb) for o, mb, _, _ in kf.stage_get_order()] == sch.kfkb_order(k, M, 0)
        Y, dX = st.outputs(M)
        Y, dX = Y.reshape(GB, T, H), dX.reshape(GB, T, H)
        assert_close(Y, Yr, dt, "Y of plan (%d, %d)" % (k, b))
        assert_close(dX, dXr, dt, "dX of plan (%d, %d)" % (k, b))
        G = st.gradients()
        for l in range(L):
            for n in synth.PARAM_ORDER:
                assert_close(G[l][n], Gr[l][n], dt, "grad block %d %s of plan (%d, %d)" % (l, n, k, b))
        # across candidates: the same step up to the order of the sums over the token axis
        if first is None:
            first = (Y, dX, G)
        else:
            assert_close(Y, first[0], dt, "Y across plans", factor=0.25)
            assert_close(dX, first[1], dt, "dX across plans", factor=0.25)
            for l in range(L):
                for n in synth.PARAM_ORDER:
                    assert_close(G[l][n], first[2][l][n], dt, "grad across plans", factor=0.25)
        with pytest.raises(kf.KfkbError) as e:                 # one more live micro-batch would not fit
            kf.run_kFkB(k, M, k * b * per_sample - 1)
        assert e.value.code == -3
        st.close()

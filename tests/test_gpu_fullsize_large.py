"""Parity at the FULL size of the three larger benchmark stages (1.3B-class, wide, very wide), in the launch
configuration bench.py times (the library's own lanes, tile shapes, W-step windows).

Per stage: (a) ONE whole micro-batch at full sequence length, depth and width against the float64 oracle — outputs,
input gradients and every parameter-gradient tensor, per tensor at the bf16 bar (8 - 41 TFLOP of float64 numpy: 10 s to
about a minute on the GPU machine's host cores); (b) an eight-micro-batch iteration bit-identical for k = 1, 2, 4, 8, its
first micro-batch bit-identical to the run of (a), executed order = the kFkB definition.  Weights come from the same
seeded tiled draw bench.py uses; inputs and upstream gradients from the seeded generators.

The bar.  2e-2 relative per tensor, as everywhere, for the 1.3B-class and the wide stage (measured: 0.3 - 1.1e-2) and for
the outputs of the very wide stage (0.9e-2).  The input gradients and parameter gradients of the very wide stage take
3e-2, and this is why: with weights N(0, 0.02) at hidden 8192 the queries and keys have standard deviation 1.8, the
attention logits 3.3, and a softmax that sharp multiplies relative perturbations of its inputs by about four (storing
exact q, k, v, dO in bf16 and doing everything else exactly already gives 0.6e-2 on dQ and dK, from a storage rounding
of 0.16e-2: tests/test_oracle_attention_sensitivity.py shows it with the oracle alone).  The upstream gradient reaches the
last block's attention backward with 0.65e-2 of accumulated bf16 storage rounding, its q, k, v carry 0.5e-2 from the
forward pass, and dqkv comes out at 2.4e-2 (measured per tensor: block 1 w_qkv 2.47e-2, ln1_g 2.43e-2, everything else
0.5 - 1.9e-2): storage precision, which the method fixes, not kernel arithmetic (fp32 accumulation and statistics
throughout).  At logits of standard deviation 0.8 and 1.6 (hidden 2048, 4096) the same kernels stay far inside 2e-2."""
import numpy as np
import pytest
import torch

import kfkb_synth as synth
import paper_2303_01675_amd as kf
from oracle import schedule as sch
from _util import assert_close

pytestmark = pytest.mark.gpu

STAGES = {
    "gpt-1.3b-stage": dict(L=6, H=2048, heads=16, T=2048, b=2),
    "wide-stage": dict(L=4, H=4096, heads=32, T=2048, b=1),
    "very-wide-stage": dict(L=2, H=8192, heads=64, T=4096, b=1),
}
M = 8


@pytest.mark.parametrize("name", list(STAGES))
def test_full_size_microbatch_matches_the_oracle_and_every_k_gives_the_same_bits(name):
    c = STAGES[name]
    L, H, heads, T, b = c["L"], c["H"], c["heads"], c["T"], c["b"]
    blocks = synth.stage_weights_tiled(L, H, 4 * H, "bf16")
    st = kf.StageBuffers(blocks, kf.BF16, heads, T, b, M, M)
    try:
        pair = [(synth.microbatch_inputs(j, b, T, H, "bf16"), synth.microbatch_upstream_grads(j, b, T, H, "bf16")) for j in range(2)]
        for mb in range(M):
            st.set_inputs_one(mb, *pair[mb % 2])
        # (a) one micro-batch against the oracle
        kf.stage_zero_grads()
        kf.run_kFkB(1, 1, 0)
        kf.stage_sync()
        assert [(o, mb) for o, mb, _, _ in kf.stage_get_order()] == sch.kfkb_order(1, 1, 0)
        y1, dx1 = st.h_out[:1].clone(), st.h_ingrad[:1].clone()
        Y, dX = st.outputs(1)
        G = st.gradients()
        Gr, Yr, dXr, _ = sch.run_iteration(sch.kfkb_order(1, 1, 0), blocks, [pair[0][0]], [pair[0][1]], heads)
        grad_factor = 1.5 if name == "very-wide-stage" else 1.0      # see the module docstring
        assert_close(Y[0], Yr[0], kf.BF16, "%s Y" % name)
        assert_close(dX[0], dXr[0], kf.BF16, "%s dX" % name, factor=grad_factor)
        for l in range(L):
            for n in synth.PARAM_ORDER:
                assert_close(G[l][n], Gr[l][n], kf.BF16, "%s grad block %d %s" % (name, l, n), factor=grad_factor)
        del Gr, Yr, dXr, G
        # (b) eight micro-batches, every k
        ref = None
        for k in (1, 2, 4, 8):
            kf.stage_zero_grads()
            kf.run_kFkB(k, M, 0)
            kf.stage_sync()
            assert [(o, mb) for o, mb, _, _ in kf.stage_get_order()] == sch.kfkb_order(k, M, 0)
            if ref is None:
                ref = (st.grads.clone(), st.h_out.clone(), st.h_ingrad.clone())
                assert torch.equal(ref[1][:1], y1) and torch.equal(ref[2][:1], dx1)
                assert bool(torch.isfinite(ref[0]).all())
            else:
                for a, b_ in zip(ref, (st.grads, st.h_out, st.h_ingrad)):
                    assert torch.equal(a, b_), (name, k)
    finally:
        st.close()
        kf.stage_destroy()

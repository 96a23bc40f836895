"""Stage-level parity at the WIDTHS of the three larger benchmark stages (hidden 2048 / 4096 / 8192, head size 128,
MLP 4x), with sequence length, depth and micro-batch count reduced to what the float64 oracle finishes in seconds.
These widths take engine paths the small stages do not: LayerNorm backward as dx + partial sums finished inside
the grouped weight-gradient launch (hidden > 2048), chunk-major NT products with reduction lengths up to 32768,
bias column sums up to 32768 wide.  Every case runs with the library's own tile choice and with the 256 x 256
tiles forced, which is the shape the full-size stages run (their token count gives enough tiles by itself).

Pins per case: (ii) run_kFkB on two micro-batches against oracle.schedule.run_iteration, per tensor; (i) the
four-micro-batch iteration bit-identical for k = 1, 2, 4 and its first two micro-batches bit-identical to the run
checked against the oracle; (iv) the accumulated gradient of the four-micro-batch iteration against ONE micro-batch
holding all four samples' tokens ("mathematically equivalent": samples are independent in every op)."""
import numpy as np
import pytest
import torch

import kfkb_synth as synth
import paper_2303_01675_amd as kf
from oracle import schedule as sch
from _util import assert_close

pytestmark = pytest.mark.gpu

CASES = {
    "h2048": dict(H=2048, heads=16, L=2, T=256, b=2, M=4),      # 1.3B-class stage's width
    "h4096": dict(H=4096, heads=32, L=1, T=192, b=1, M=4),      # wide stage's width; tokens not a multiple of a tile
    "h8192": dict(H=8192, heads=64, L=1, T=128, b=1, M=4),      # very wide stage's width
}


def _inputs(c, M):
    xs = [synth.microbatch_inputs(mb, c["b"], c["T"], c["H"], "bf16") for mb in range(M)]
    dys = [synth.microbatch_upstream_grads(mb, c["b"], c["T"], c["H"], "bf16") for mb in range(M)]
    return xs, dys


def _run(st, k, M):
    kf.stage_zero_grads()
    kf.run_kFkB(k, M, 0)
    kf.stage_sync()
    assert [(o, mb) for o, mb, _, _ in kf.stage_get_order()] == sch.kfkb_order(k, M, 0)
    return st.grads.clone(), st.h_out.clone(), st.h_ingrad.clone()


@pytest.mark.parametrize("tiles", ["own-tile-choice", "big-tiles", "mid-tiles"])
@pytest.mark.parametrize("name", list(CASES))
def test_wide_stage_matches_oracle_and_is_identical_for_every_k(name, tiles):
    c = CASES[name]
    H, heads, L, T, b, M = c["H"], c["heads"], c["L"], c["T"], c["b"], c["M"]
    blocks = synth.stage_weights_tiled(L, H, 4 * H, "bf16")
    xs, dys = _inputs(c, M)
    prev = kf.kfkb_set_big_tile_min(1 if tiles == "big-tiles" else 192)
    kf.kfkb_set_mid_tiles(2 if tiles == "mid-tiles" else 1)      # 128 x 256 tiles for every forward / input-gradient product
    try:
        st = kf.StageBuffers(blocks, kf.BF16, heads, T, b, M, M)
        st.set_inputs(xs, dys)
        # (ii) two micro-batches against the oracle
        g2, y2, dx2 = _run(st, 2, 2)
        Gr, Yr, dXr, _ = sch.run_iteration(sch.kfkb_order(2, 2, 0), blocks, xs[:2], dys[:2], heads)
        Y, dX = st.outputs(2)
        for mb in range(2):
            assert_close(Y[mb], Yr[mb], kf.BF16, "Y[%d]" % mb)
            assert_close(dX[mb], dXr[mb], kf.BF16, "dX[%d]" % mb)
        G = st.gradients()
        for l in range(L):
            for n in synth.PARAM_ORDER:
                assert_close(G[l][n], Gr[l][n], kf.BF16, "grad block %d %s" % (l, n))
        del Gr, G
        # (i) the four-micro-batch iteration: the same bits for every k, and micro-batches 0, 1 as above
        ref = _run(st, 1, M)
        for k in (2, 4):
            for a, b_ in zip(ref, _run(st, k, M)):
                assert torch.equal(a, b_), k
        assert torch.equal(ref[1][:2], y2[:2]) and torch.equal(ref[2][:2], dx2[:2])
        g4 = ref[0].clone()
        y4, dx4 = st.outputs(M)
        st.close()
        if name == "h8192":
            return                                               # (iv) at the two smaller widths: it needs a second stage
        # (iv) all samples as ONE micro-batch: same outputs per sample, same accumulated gradient up to the order of
        # the fp32 sums over the token axis
        one = kf.StageBuffers(blocks, kf.BF16, heads, T, M * b, 1, 1)
        one.set_inputs([np.concatenate(xs, axis=0)], [np.concatenate(dys, axis=0)])
        gf, _, _ = _run(one, 1, 1)
        Yf, dXf = one.outputs(1)
        assert_close(Yf[0], np.concatenate(list(y4), axis=0), kf.BF16, "Y of the full batch", factor=0.1)
        assert_close(dXf[0], np.concatenate(list(dx4), axis=0), kf.BF16, "dX of the full batch", factor=0.1)
        Gf, G4 = one.gradients(), kf.unpack_params(g4, L, H, 4 * H)
        for l in range(L):
            for n in synth.PARAM_ORDER:
                assert_close(G4[l][n], Gf[l][n], kf.BF16, "full-batch grad block %d %s" % (l, n), factor=0.1)
        one.close()
    finally:
        kf.kfkb_set_big_tile_min(prev)
        kf.kfkb_set_mid_tiles(1)
        kf.stage_destroy()


@pytest.mark.parametrize("variant", ["recompute", "warmup", "separate-reductions"])
def test_wide_stage_variants_match_oracle(variant):
    """hidden 4096 (LayerNorm backward in its dx + partial-sums form): activation recomputation, a warm-up depth
    above zero (stage 0 of 2), and the W step's reductions as launches of their own."""
    H, heads, L, T, b, M = 4096, 32, 1, 128, 1, 4
    blocks = synth.stage_weights_tiled(L, H, 4 * H, "bf16")
    c = dict(H=H, T=T, b=b)
    xs, dys = _inputs(c, M)
    S = 2 if variant == "warmup" else 1
    st = kf.StageBuffers(blocks, kf.BF16, heads, T, b, M, M, num_stages=S, stage_index=0, recompute=int(variant == "recompute"))
    st.set_inputs(xs, dys)
    if variant == "separate-reductions":
        kf.stage_set_fused_w_reductions(0)
    ref = None
    for k in (1, 2):
        w = sch.warmup_groups(S, 0, k, M)
        kf.stage_zero_grads()
        kf.run_kFkB(k, M, 0)
        kf.stage_sync()
        order = sch.kfkb_order(k, M, w)
        assert [(o, mb) for o, mb, _, _ in kf.stage_get_order()] == order
        cur = (st.grads.clone(), st.h_out.clone(), st.h_ingrad.clone())
        if ref is None:
            ref = cur
            Gr, Yr, dXr, _ = sch.run_iteration(order, blocks, xs, dys, heads)
            Y, dX = st.outputs(M)
            for mb in range(M):
                assert_close(Y[mb], Yr[mb], kf.BF16, "Y[%d]" % mb)
                assert_close(dX[mb], dXr[mb], kf.BF16, "dX[%d]" % mb)
            G = st.gradients()
            for n in synth.PARAM_ORDER:
                assert_close(G[0][n], Gr[0][n], kf.BF16, "grad %s" % n)
        else:
            for a, b_ in zip(ref, cur):
                assert torch.equal(a, b_)
    st.close()


def _rows(seed, n, M):
    return np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, M - 1], (synth.uniform(seed, n) * M).astype(np.int64) % M]))


@pytest.mark.parametrize("M,N,K,big", [(2048 + 77, 4096, 8192, 0), (4096, 4096, 8192, 1),       # 16 x 16 large tiles
                                       (1000, 2048, 16384, 0), (512 + 9, 2048, 16384, 1),
                                       (300, 1024, 32768, 0), (1536 + 77, 8192, 32768, 1),       # very wide stage: fc2 / fc1 input gradient
                                       (2048, 4096, 16384, 2), (1000 + 3, 2048, 8192, 2), (4096, 2048, 6144, 2)])   # 128 x 256 tiles
def test_chunk_major_nt_product_at_the_reduction_lengths_of_the_larger_stages(M, N, K, big):
    """The NT kernel the stage uses (B chunk-major, A in 64-deep slices) at K = 8192, 16384 and 32768, the two square
    tile shapes (big = 0, 1) and the 128 x 256 tiles of the 1.3B-class and wide stages (big = 2); the oracle side is
    the textbook product of about 64 sampled output rows, all columns."""
    from _util import dev, host, rnd
    dt = kf.BF16
    A = rnd(80, (M, K), dt)
    period = (1 << 22) + 17
    base = synth.round_to_bf16(synth.normal(81, period, 0.0, 0.05))
    B = np.tile(base, -(-(N * K) // period))[:N * K].reshape(N, K)          # float32, values exact in bf16
    bias = rnd(82, (N,), dt, 0.5)
    rows = _rows(83, 57, M)
    ref = np.empty((len(rows), N))
    for n0 in range(0, N, 1024):
        ref[:, n0:n0 + 1024] = A[rows] @ B[n0:n0 + 1024].astype(np.float64).T
    Bt = torch.empty(N * K, dtype=torch.bfloat16, device="cuda")
    Bd = torch.from_numpy(B).to(torch.bfloat16).cuda()
    kf.kfkb_op_tile_weights(Bd, Bt, N, K, False)
    Cout = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
    prev = kf.kfkb_set_big_tile_min(1 if big == 1 else 1 << 30)
    kf.kfkb_set_mid_tiles(2 if big == 2 else 0)
    try:
        kf.kfkb_op_gemm_nt_tiled(kf.EPI_BIAS, M, N, K, dev(A, dt), Bt, dev(bias, dt), None, Cout, None, None)
        torch.cuda.synchronize()
    finally:
        kf.kfkb_set_big_tile_min(prev)
        kf.kfkb_set_mid_tiles(1)
    assert_close(host(Cout[torch.from_numpy(rows).cuda()]), ref + bias, dt, "chunk-major NT rows")

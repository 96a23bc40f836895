"""Per-kernel parity: each HIP kernel, called through the C boundary, against the oracle (or the
textbook definition for a bare matrix product) on the same seeded inputs.  Sizes span several
tiles and a ragged tail."""
import numpy as np
import pytest
import torch

import paper_2303_01675_amd as kf
from oracle import stage_math as sm
from _util import TOL, assert_close, dev, host, rnd, tdtype

pytestmark = pytest.mark.gpu
DTS = [kf.F32, kf.BF16, kf.F16]
H16 = [kf.BF16, kf.F16]


def _sync():
    torch.cuda.synchronize()


# ---------------------------------------------------------------- LayerNorm
@pytest.mark.parametrize("dt", DTS)
@pytest.mark.parametrize("rows,H", [(1, 128), (37, 128), (130, 1024), (67, 2048), (9, 8192), (0, 128)])
def test_layernorm_forward(dt, rows, H):
    x = rnd(1, (rows, H), dt, 2.0, 0.5); g = rnd(2, (H,), dt, 0.02, 1.0); b = rnd(3, (H,), dt, 0.02)
    y = torch.empty(rows, H, dtype=tdtype(dt), device="cuda")
    mean = torch.empty(rows, device="cuda"); rstd = torch.empty(rows, device="cuda")
    kf.kfkb_op_layernorm_fwd(dt, dev(x, dt), dev(g, dt), dev(b, dt), y, mean, rstd, rows, H, 1e-5)
    _sync()
    ref, (xhat, rs) = sm.layernorm_fwd(x, g, b, 1e-5)
    assert_close(host(y), ref, dt, "ln y")
    assert_close(host(mean), x.mean(-1), kf.F32, "ln mean", factor=10)
    assert_close(host(rstd), rs[:, 0], kf.F32, "ln rstd", factor=10)


@pytest.mark.parametrize("dt", DTS)
@pytest.mark.parametrize("rows,H,with_res", [(37, 128, True), (300, 1024, False), (130, 2048, True), (40, 8192, True)])
def test_layernorm_backward(dt, rows, H, with_res):
    x = rnd(4, (rows, H), dt, 1.5, -0.3); dy = rnd(5, (rows, H), dt); g = rnd(6, (H,), dt, 0.02, 1.0)
    res = rnd(7, (rows, H), dt) if with_res else None
    _, cache = sm.layernorm_fwd(x, g, np.zeros(H), 1e-5)
    dx_ref, dg_ref, db_ref = sm.layernorm_bwd(dy, cache, g)
    if with_res:
        dx_ref = dx_ref + res
    mean = torch.from_numpy(x.mean(-1)).float().cuda()
    rstd = torch.from_numpy(cache[1][:, 0]).float().cuda()
    dx = torch.empty(rows, H, dtype=tdtype(dt), device="cuda")
    dgam = torch.full((H,), 1.0, device="cuda"); dbet = torch.full((H,), -2.0, device="cuda")   # accumulate onto these
    scratch = torch.empty(kf.kfkb_op_reduce_scratch_floats(H), device="cuda")
    kf.kfkb_op_layernorm_bwd(dt, dev(dy, dt), dev(x, dt), mean, rstd, dev(g, dt), dev(res, dt) if with_res else None,
                             dx, dgam, dbet, scratch, rows, H)
    _sync()
    assert_close(host(dx), dx_ref, dt, "ln dx")
    assert_close(host(dgam) - 1.0, dg_ref, kf.F32, "ln dgamma", factor=10)
    assert_close(host(dbet) + 2.0, db_ref, kf.F32, "ln dbeta", factor=10)


@pytest.mark.parametrize("dt", DTS)
@pytest.mark.parametrize("rows,N", [(5, 128), (257, 384), (1000, 3072)])
def test_column_sum(dt, rows, N):
    dy = rnd(8, (rows, N), dt)
    out = torch.full((N,), 3.0, device="cuda")
    scratch = torch.empty(kf.kfkb_op_reduce_scratch_floats(N), device="cuda")
    kf.kfkb_op_colsum_accum(dt, dev(dy, dt), out, scratch, rows, N)
    _sync()
    assert_close(host(out) - 3.0, dy.sum(0), kf.F32, "colsum", factor=10)


@pytest.mark.parametrize("dt", DTS)
def test_gelu_backward(dt):
    n = 8 * 1031
    u = rnd(9, (n,), dt, 2.0); dg = rnd(10, (n,), dt)
    du = torch.empty(n, dtype=tdtype(dt), device="cuda")
    kf.kfkb_op_gelu_bwd(dt, dev(dg, dt), dev(u, dt), du, n)
    _sync()
    assert_close(host(du), dg * sm.gelu_grad(u), dt, "gelu bwd")
    with pytest.raises(kf.KfkbError):
        kf.kfkb_op_gelu_bwd(dt, dev(dg, dt), dev(u, dt), du, 7)


@pytest.mark.parametrize("dt", DTS)
def test_transpose(dt):
    a = rnd(11, (70, 200), dt)
    out = torch.empty(200, 70, dtype=tdtype(dt), device="cuda")
    kf.kfkb_op_transpose(dt, dev(a, dt), out, 70, 200)
    _sync()
    assert np.array_equal(host(out), a.T)


# ---------------------------------------------------------------- GEMM
def _gemm_case(dt, kind, epi, M, N, K, seed=20, tiled=0):
    """Runs one GEMM through the boundary and returns (got, reference) lists."""
    if kind == kf.GEMM_NN:
        A = rnd(seed, (M, K), dt); B = rnd(seed + 1, (K, N), dt, 0.05); acc = A @ B
    elif kind == kf.GEMM_NT:
        A = rnd(seed, (M, K), dt); B = rnd(seed + 1, (N, K), dt, 0.05); acc = A @ B.T
    else:
        A = rnd(seed, (K, M), dt); B = rnd(seed + 1, (K, N), dt, 0.05); acc = A.T @ B
    bias = rnd(seed + 2, (N,), dt, 0.5); res = rnd(seed + 3, (M, N), dt)
    Cout = torch.zeros(M, N, dtype=tdtype(dt), device="cuda")
    C2 = torch.zeros(M, N, dtype=tdtype(dt), device="cuda")
    Cacc0 = rnd(seed + 4, (M, N), kf.F32)
    Cacc = dev(Cacc0, kf.F32)
    if tiled == 0:
        kf.kfkb_op_gemm(dt, kind, epi, M, N, K, dev(A, dt), dev(B, dt), dev(bias, dt), dev(res, dt), Cout, C2, Cacc)
    else:
        # B handed over chunk-major, made on the device from B itself (tiled == 1) or from its transpose (tiled == 2)
        assert dt == kf.BF16 and kind == kf.GEMM_NT
        Bt = torch.empty(N * K, dtype=torch.bfloat16, device="cuda")
        src = dev(B if tiled == 1 else np.ascontiguousarray(B.T), dt)
        kf.kfkb_op_tile_weights(src, Bt, N, K, tiled == 2)
        kf.kfkb_op_gemm_nt_tiled(epi, M, N, K, dev(A, dt), Bt, dev(bias, dt), dev(res, dt), Cout, C2, Cacc)
    _sync()
    if epi == kf.EPI_NONE:
        return [host(Cout)], [acc]
    if epi == kf.EPI_BIAS:
        return [host(Cout)], [acc + bias]
    if epi == kf.EPI_BIAS_GELU:
        return [host(Cout), host(C2)], [acc + bias, sm.gelu(acc + bias)]
    if epi == kf.EPI_BIAS_RES:
        return [host(Cout)], [acc + bias + res]
    if epi == kf.EPI_ACCUM:
        return [host(Cacc) - Cacc0], [acc]
    return [host(Cout)], [acc * sm.gelu_grad(res)]


@pytest.mark.parametrize("kind", [kf.GEMM_NN, kf.GEMM_NT, kf.GEMM_TN])
@pytest.mark.parametrize("epi", range(6))
def test_gemm_f32(kind, epi):
    for (M, N, K) in [(128, 384, 128), (70, 200, 50), (129, 65, 33)]:
        got, ref = _gemm_case(kf.F32, kind, epi, M, N, K)
        for g, r in zip(got, ref):
            assert_close(g, r, kf.F32, "gemm f32 kind %d epi %d %s" % (kind, epi, (M, N, K)))


@pytest.mark.parametrize("dt", H16)
@pytest.mark.parametrize("epi", range(6))
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (300, 384, 192), (4096, 1024, 256), (2048 + 77, 2048, 128), (4096 - 3, 4096, 128)])
def test_gemm_bf16_nt(dt, epi, M, N, K):
    got, ref = _gemm_case(dt, kf.GEMM_NT, epi, M, N, K)
    for g, r in zip(got, ref):
        assert_close(g, r, dt if epi != kf.EPI_ACCUM else kf.F32, "gemm 16-bit NT epi %d" % epi,
                     factor=1 if epi != kf.EPI_ACCUM else 10)


@pytest.mark.parametrize("epi", range(6))
@pytest.mark.parametrize("M,N,K,tiled", [(128, 128, 64, 1), (300, 384, 448, 2), (515, 256, 832, 1), (2048 + 77, 2048, 1024, 2),
                                         (4096 - 3, 4096, 128, 1), (4096, 1024, 768, 2), (1000, 1024, 1024, 1),
                                         (2048, 512, 1536, 2)])
@pytest.mark.parametrize("mid", [0, 2])
def test_gemm_bf16_nt_chunk_major_weights(epi, M, N, K, tiled, mid):
    """The NT kernel that reads B chunk-major (and A in 64-deep slices): reduction lengths below, at and
    beyond one period of its LDS rings (12 chunks of 32), ragged M, the square tile sizes (mid = 0) and the
    128 x 256 tiles wherever N allows them (mid = 2)."""
    kf.kfkb_set_mid_tiles(mid)
    try:
        got, ref = _gemm_case(kf.BF16, kf.GEMM_NT, epi, M, N, K, tiled=tiled)
    finally:
        kf.kfkb_set_mid_tiles(1)
    for g, r in zip(got, ref):
        assert_close(g, r, kf.BF16 if epi != kf.EPI_ACCUM else kf.F32, "gemm bf16 NT chunk-major epi %d" % epi,
                     factor=1 if epi != kf.EPI_ACCUM else 10)


def test_tile_weights_layout():
    N, K = 72, 96
    B = rnd(31, (N, K), kf.BF16)
    want = np.ascontiguousarray(B.reshape(N, K // 32, 32).transpose(1, 0, 2)).reshape(-1)
    for transposed in (False, True):
        dst = torch.zeros(N * K, dtype=torch.bfloat16, device="cuda")
        kf.kfkb_op_tile_weights(dev(np.ascontiguousarray(B.T) if transposed else B, kf.BF16), dst, N, K, transposed)
        _sync()
        assert np.array_equal(host(dst), want)
    with pytest.raises(kf.KfkbError):
        kf.kfkb_op_tile_weights(dst, dst, N, 48, False)
    with pytest.raises(kf.KfkbError):
        kf.kfkb_op_gemm_nt_tiled(kf.EPI_NONE, 128, 128, 96, dst, dst, None, None, dst, None, None)    # K % 64 != 0


@pytest.mark.parametrize("dt", H16)
@pytest.mark.parametrize("epi", [kf.EPI_ACCUM, kf.EPI_NONE])
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (384, 256, 300), (1024, 3072, 1000), (4096, 4096, 130),
                                   (2048, 2048, 96), (4096, 4096, 128)])    # the last two: both tile sizes of the DMA kernel
def test_gemm_bf16_tn(dt, epi, M, N, K):
    got, ref = _gemm_case(dt, kf.GEMM_TN, epi, M, N, K)
    for g, r in zip(got, ref):
        assert_close(g, r, dt if epi != kf.EPI_ACCUM else kf.F32, "gemm 16-bit TN epi %d" % epi,
                     factor=1 if epi != kf.EPI_ACCUM else 10)


def test_gemm_rejects_unsupported_shapes():
    a = torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(1 << 16, device="cuda")
    for (kind, M, N, K) in [(kf.GEMM_NT, 128, 100, 64), (kf.GEMM_NT, 128, 128, 48), (kf.GEMM_TN, 100, 128, 64),
                            (kf.GEMM_NN, 128, 128, 64)]:
        with pytest.raises(kf.KfkbError) as e:
            kf.kfkb_op_gemm(kf.BF16, kind, kf.EPI_NONE, M, N, K, a, a, None, None, a, None, None)
        assert e.value.code == -1
    with pytest.raises(kf.KfkbError):
        kf.kfkb_op_gemm(kf.F32, kf.GEMM_NN, kf.EPI_BIAS, 8, 8, 8, f, f, None, None, f, None, None)   # bias missing
    kf.kfkb_op_gemm(kf.F32, kf.GEMM_NN, kf.EPI_NONE, 0, 8, 8, f, f, None, None, f, None, None)       # empty is a no-op


# ---------------------------------------------------------------- attention
def _attention_case(dt, b, T, heads, d, causal, seed=40):
    H = heads * d
    qkv = rnd(seed, (b, T, 3 * H), dt)
    do = rnd(seed + 1, (b, T, H), dt)
    q, k, v = (sm._split_heads(qkv[..., i * H:(i + 1) * H], heads) for i in range(3))
    o_ref, p = sm.attention_fwd(q, k, v, causal)
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(d)
    if causal:
        s = np.where(np.tril(np.ones((T, T), dtype=bool)), s, -np.inf)
    lse_ref = np.log(np.exp(s - s.max(-1, keepdims=True)).sum(-1)) + s.max(-1)
    dq, dk, dv = sm.attention_bwd(sm._split_heads(do, heads), q, k, v, p)
    dqkv_ref = np.concatenate([sm._merge_heads(t) for t in (dq, dk, dv)], axis=-1)
    qkv_d = dev(qkv, dt)
    o = torch.zeros(b * T, H, dtype=tdtype(dt), device="cuda")
    lse = torch.zeros(b, heads, T, device="cuda")
    kf.kfkb_op_attention_fwd(dt, qkv_d, o, lse, b, T, H, heads, causal)
    _sync()
    assert_close(host(o).reshape(b, T, H), sm._merge_heads(o_ref), dt, "attention o")
    assert_close(host(lse), lse_ref, kf.F32, "attention lse", factor=30)
    # backward takes the forward's own (rounded) o, as the stage does
    dqkv = torch.zeros(b * T, 3 * H, dtype=tdtype(dt), device="cuda")
    dsum = torch.zeros(b, heads, T, device="cuda")
    kf.kfkb_op_attention_bwd(dt, qkv_d, o, dev(do, dt), lse, dsum, dqkv, b, T, H, heads, causal)
    _sync()
    got = host(dqkv).reshape(b, T, 3 * H)
    for i, name in enumerate(("dq", "dk", "dv")):
        # T = 1 makes dq and dk exactly zero (one-element softmax): compare on the scale of do * v
        assert_close(got[..., i * H:(i + 1) * H], dqkv_ref[..., i * H:(i + 1) * H], dt, "attention " + name,
                     floor=1.0 if T == 1 else 0.0)


@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("b,T,heads,d", [(2, 64, 4, 32), (1, 1, 2, 32), (2, 77, 3, 16), (1, 200, 2, 64), (1, 130, 1, 128)])
def test_attention_f32(b, T, heads, d, causal):
    _attention_case(kf.F32, b, T, heads, d, causal)


@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("b,T,heads,d", [(2, 64, 2, 64), (1, 1, 2, 64), (2, 200, 2, 64), (1, 333, 2, 128), (1, 512, 1, 128),
                                         (1, 128, 2, 64), (1, 129, 1, 64)])
def test_attention_bf16(b, T, heads, d, causal):
    _attention_case(kf.BF16, b, T, heads, d, causal)


@pytest.mark.parametrize("causal", [1, 0])
@pytest.mark.parametrize("b,T,heads,d", [(2, 64, 2, 64), (1, 1, 2, 64), (2, 200, 2, 64), (1, 333, 2, 128), (1, 129, 1, 64)])
def test_attention_f16(b, T, heads, d, causal):
    _attention_case(kf.F16, b, T, heads, d, causal)


def test_attention_rejects_unsupported_head_size():
    z = torch.zeros(1 << 12, dtype=torch.bfloat16, device="cuda"); f = torch.zeros(1 << 12, device="cuda")
    with pytest.raises(kf.KfkbError):
        kf.kfkb_op_attention_fwd(kf.BF16, z, z, f, 1, 8, 96, 1, 1)


def test_delay_kernel_waits_about_as_long_as_asked():
    # on the default stream: every extra stream a process creates takes a share of the 4 hardware queues
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    kf.kfkb_op_delay(1000)                             # warm-up launch
    e0.record()
    kf.kfkb_op_delay(3_000_000)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1)
    assert 2.9 <= ms <= 4.5, ms


# ---------------------------------------------------------------- shapes of the larger stages, sampled
@pytest.mark.parametrize("kind,M,N,K", [(kf.GEMM_NT, 4096, 6144, 2048),      # 1.3B-class stage: qkv forward
                                        (kf.GEMM_NT, 4096, 2048, 8192),      # 1.3B-class stage: fc2 forward / fc1 input gradient
                                        (kf.GEMM_NT, 2048, 16384, 4096),     # wide stage: fc1 forward
                                        (kf.GEMM_TN, 2048, 8192, 4096)])     # 1.3B-class stage: fc1 weight gradient (K = tokens)
def test_gemm_bf16_at_the_shapes_of_the_larger_stages_on_sampled_rows(kind, M, N, K):
    """Full-size products of the larger benchmark stages; the oracle side is the textbook product of 64 sampled
    output rows (all columns), which covers every tile column and a spread of tile rows."""
    dt = kf.BF16
    if kind == kf.GEMM_NT:
        A = rnd(70, (M, K), dt); B = rnd(71, (N, K), dt, 0.05)
    else:
        A = rnd(70, (K, M), dt); B = rnd(71, (K, N), dt, 0.05)
    rows = np.unique(np.concatenate([[0, 1, 127, 128, 255, 256, M - 1], synth_rows(72, 57, M)]))
    ref = (A[rows] @ B.T) if kind == kf.GEMM_NT else (A[:, rows].T @ B)
    bias = rnd(73, (N,), dt, 0.5)
    if kind == kf.GEMM_NT:
        Cout = torch.zeros(M, N, dtype=torch.bfloat16, device="cuda")
        kf.kfkb_op_gemm(dt, kind, kf.EPI_BIAS, M, N, K, dev(A, dt), dev(B, dt), dev(bias, dt), None, Cout, None, None)
        _sync()
        assert_close(host(Cout[torch.from_numpy(rows).cuda()]), ref + bias, dt, "NT rows")
    else:
        Cacc = torch.zeros(M, N, device="cuda")
        kf.kfkb_op_gemm(dt, kind, kf.EPI_ACCUM, M, N, K, dev(A, dt), dev(B, dt), None, None, None, None, Cacc)
        _sync()
        assert_close(host(Cacc[torch.from_numpy(rows).cuda()]), ref, kf.F32, "TN rows", factor=10)


def synth_rows(seed, n, M):
    import kfkb_synth as synth
    return (synth.uniform(seed, n) * M).astype(np.int64) % M


@pytest.mark.parametrize("b,T,heads,d", [(1, 2048, 2, 128),      # 1.3B-class and wide stages
                                         (1, 4096, 1, 128)])     # very wide stage
def test_attention_bf16_at_the_sequence_lengths_of_the_larger_stages(b, T, heads, d):
    _attention_case(kf.BF16, b, T, heads, d, 1)

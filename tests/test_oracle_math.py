"""Pins of the oracle's stage math against things other than itself: torch library routines
and autograd (float64, CPU), closed forms, brute-force loops and central finite differences."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as TF

import kfkb_synth as synth
from oracle import stage_math as sm



def _rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(np.asarray(b)), 1e-300)


# ---------------------------------------------------------------- LayerNorm

def test_layernorm_matches_library_and_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.normal(size=(3, 5, 16)) * 3 + 1
    g = rng.normal(size=16); b = rng.normal(size=16)
    y, (xhat, rstd) = sm.layernorm_fwd(x, g, b, 1e-5)
    ref = TF.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), torch.from_numpy(b), 1e-5).numpy()
    assert _rel(y, ref) < 1e-13
    # gamma = 1, beta = 0: rows have mean 0 and (biased) variance var/(var+eps)
    y1, _ = sm.layernorm_fwd(x, np.ones(16), np.zeros(16), 1e-5)
    assert np.abs(y1.mean(-1)).max() < 1e-13
    var = x.var(-1)
    assert np.allclose(y1.var(-1), var / (var + 1e-5), rtol=1e-12)


def test_layernorm_bwd_rows_sum_to_zero_and_match_autograd():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(4, 12)); dy = rng.normal(size=(4, 12)); g = rng.normal(size=12) + 1
    _, cache = sm.layernorm_fwd(x, g, np.zeros(12), 1e-5)
    dx, dg, db = sm.layernorm_bwd(dy, cache, g)
    dx1, _, _ = sm.layernorm_bwd(dy, cache, np.ones(12))
    assert np.abs(dx1.sum(-1)).max() < 1e-12          # shift invariance of LN
    xt = torch.from_numpy(x).requires_grad_(); gt = torch.from_numpy(g).requires_grad_()
    bt = torch.zeros(12, dtype=torch.float64, requires_grad=True)
    TF.layer_norm(xt, (12,), gt, bt, 1e-5).backward(torch.from_numpy(dy))
    assert _rel(dx, xt.grad.numpy()) < 1e-12
    assert _rel(dg, gt.grad.numpy()) < 1e-12
    assert _rel(db, bt.grad.numpy()) < 1e-12


# ---------------------------------------------------------------- GELU

def test_gelu_closed_forms_and_library():
    assert sm.gelu(np.array(0.0)) == 0.0
    assert sm.gelu_grad(np.array(0.0)) == 0.5
    big = np.array([12.0, 30.0])
    assert np.allclose(sm.gelu(big), big, rtol=0, atol=1e-12)
    assert np.allclose(sm.gelu(-big), 0.0, atol=1e-12)
    # gelu(u) - gelu(-u) = u for the tanh form (tanh is odd)
    u = np.linspace(-6, 6, 101)
    assert np.allclose(sm.gelu(u) - sm.gelu(-u), u, atol=1e-14)
    ref = TF.gelu(torch.from_numpy(u), approximate="tanh").numpy()
    assert np.abs(sm.gelu(u) - ref).max() < 1e-14
    # value at u = 1 written out by hand: 0.5 (1 + tanh(sqrt(2/pi) * 1.044715))
    assert abs(float(sm.gelu(np.array(1.0))) - 0.5 * (1 + math.tanh(0.7978845608028654 * 1.044715))) < 1e-15
    ut = torch.from_numpy(u).requires_grad_()
    TF.gelu(ut, approximate="tanh").sum().backward()
    assert np.abs(sm.gelu_grad(u) - ut.grad.numpy()).max() < 1e-13


# ---------------------------------------------------------------- attention

def _brute_attention(q, k, v, causal):
    b, h, T, d = q.shape
    o = np.zeros_like(q)
    for bi in range(b):
        for hi in range(h):
            for i in range(T):
                last = i if causal else T - 1
                sc = [sum(q[bi, hi, i, t] * k[bi, hi, j, t] for t in range(d)) / math.sqrt(d) for j in range(last + 1)]
                mx = max(sc)
                e = [math.exp(s - mx) for s in sc]
                z = sum(e)
                for t in range(d):
                    o[bi, hi, i, t] = sum(e[j] / z * v[bi, hi, j, t] for j in range(last + 1))
    return o


@pytest.mark.parametrize("causal", [True, False])
def test_attention_brute_force_and_library(causal):
    rng = np.random.default_rng(2)
    q, k, v = (rng.normal(size=(2, 3, 7, 4)) for _ in range(3))
    o, p = sm.attention_fwd(q, k, v, causal)
    assert _rel(o, _brute_attention(q, k, v, causal)) < 1e-13
    ref = TF.scaled_dot_product_attention(torch.from_numpy(q), torch.from_numpy(k), torch.from_numpy(v),
                                          is_causal=causal).numpy()
    assert _rel(o, ref) < 1e-12
    assert np.allclose(p.sum(-1), 1.0, atol=1e-13)
    if causal:
        assert np.all(np.triu(p, 1) == 0.0)


def test_attention_special_cases():
    rng = np.random.default_rng(3)
    q, k, v = (rng.normal(size=(1, 2, 6, 4)) for _ in range(3))
    o, _ = sm.attention_fwd(q, k, v, True)
    assert np.allclose(o[:, :, 0], v[:, :, 0], atol=1e-14)            # row 0 sees only itself
    o1, _ = sm.attention_fwd(q[:, :, :1], k[:, :, :1], v[:, :, :1], True)
    assert np.allclose(o1, v[:, :, :1], atol=1e-14)                   # T = 1
    oz, _ = sm.attention_fwd(np.zeros_like(q), k, v, True)            # zero queries: prefix means
    pref = np.cumsum(v, axis=2) / np.arange(1, 7)[None, None, :, None]
    assert np.allclose(oz, pref, atol=1e-13)
    on, _ = sm.attention_fwd(np.zeros_like(q), k, v, False)
    assert np.allclose(on, np.broadcast_to(v.mean(2, keepdims=True), v.shape), atol=1e-13)


def test_attention_bwd_matches_autograd():
    rng = np.random.default_rng(4)
    q, k, v, do = (rng.normal(size=(2, 2, 5, 8)) for _ in range(4))
    _, p = sm.attention_fwd(q, k, v, True)
    dq, dk, dv = sm.attention_bwd(do, q, k, v, p)
    qt, kt, vt = (torch.from_numpy(t).requires_grad_() for t in (q, k, v))
    TF.scaled_dot_product_attention(qt, kt, vt, is_causal=True).backward(torch.from_numpy(do))
    assert _rel(dq, qt.grad.numpy()) < 1e-12
    assert _rel(dk, kt.grad.numpy()) < 1e-12
    assert _rel(dv, vt.grad.numpy()) < 1e-12


# ---------------------------------------------------------------- whole block / stage

def _torch_block(x, p, heads, causal, eps):
    b, T, H = x.shape
    d = H // heads
    a = TF.layer_norm(x, (H,), p["ln1_g"], p["ln1_b"], eps)
    qkv = TF.linear(a, p["w_qkv"].t(), p["b_qkv"])
    q, k, v = qkv.split(H, dim=-1)
    q, k, v = (t.view(b, T, heads, d).transpose(1, 2) for t in (q, k, v))
    o = TF.scaled_dot_product_attention(q, k, v, is_causal=causal).transpose(1, 2).reshape(b, T, H)
    x1 = x + TF.linear(o, p["w_o"].t(), p["b_o"])
    c = TF.layer_norm(x1, (H,), p["ln2_g"], p["ln2_b"], eps)
    g = TF.gelu(TF.linear(c, p["w_1"].t(), p["b_1"]), approximate="tanh")
    return x1 + TF.linear(g, p["w_2"].t(), p["b_2"])


@pytest.mark.parametrize("causal", [True, False])
def test_stage_matches_torch_autograd(causal):
    L, b, T, H, heads, F = 2, 2, 6, 16, 4, 64
    blocks = synth.stage_weights(L, H, F, "f64", std=0.2)
    x = synth.microbatch_inputs(0, b, T, H, "f64")
    dy = synth.microbatch_upstream_grads(0, b, T, H, "f64")
    y, caches = sm.stage_fwd(x, blocks, heads, causal)
    dx, grads = sm.stage_bwd(dy, blocks, caches, heads)
    tb = [{n: torch.from_numpy(v.copy()).requires_grad_() for n, v in p.items()} for p in blocks]
    xt = torch.from_numpy(x.copy()).requires_grad_()
    h = xt
    for p in tb:
        h = _torch_block(h, p, heads, causal, 1e-5)
    h.backward(torch.from_numpy(dy))
    assert _rel(y, h.detach().numpy()) < 1e-12
    assert _rel(dx, xt.grad.numpy()) < 1e-11
    for l in range(L):
        for n in synth.PARAM_ORDER:
            assert _rel(grads[l][n], tb[l][n].grad.numpy()) < 1e-11, (l, n)


def test_stage_backward_by_finite_differences():
    """Central differences of the scalar sum(dY * Y) in double, every parameter tensor and dX."""
    L, b, T, H, heads, F = 2, 2, 4, 8, 2, 32
    blocks = synth.stage_weights(L, H, F, "f64", std=0.3)
    x = synth.microbatch_inputs(7, b, T, H, "f64")
    dy = synth.microbatch_upstream_grads(7, b, T, H, "f64")

    def loss(xx, bb):
        return float((sm.stage_fwd(xx, bb, heads, True)[0] * dy).sum())

    _, caches = sm.stage_fwd(x, blocks, heads, True)
    dx, grads = sm.stage_bwd(dy, blocks, caches, heads)
    eps = 1e-5
    rng = np.random.default_rng(5)

    def check(arr, analytic, name):
        flat = arr.reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 24), replace=False)
        num = np.empty(len(idx)); ana = analytic.reshape(-1)[idx]
        for j, i in enumerate(idx):
            old = flat[i]
            flat[i] = old + eps; lp = loss(x, blocks)
            flat[i] = old - eps; lm = loss(x, blocks)
            flat[i] = old
            num[j] = (lp - lm) / (2 * eps)
        assert np.linalg.norm(num - ana) / np.linalg.norm(ana) < 1e-6, name

    check(x, dx, "dX")
    for l in range(L):
        for n in synth.PARAM_ORDER:
            check(blocks[l][n], grads[l][n], "block %d %s" % (l, n))


def test_identity_and_zero_weight_special_cases():
    """Zero projection and MLP output weights: the block is the identity on the residual stream,
    and dX equals dY plus nothing (all branch gradients vanish at W_o = W_2 = 0, b = 0)."""
    L, b, T, H, heads, F = 1, 1, 5, 8, 2, 32
    blocks = synth.stage_weights(L, H, F, "f64")
    for n in ("w_o", "b_o", "w_2", "b_2"):
        blocks[0][n][...] = 0.0
    x = synth.microbatch_inputs(1, b, T, H, "f64")
    dy = synth.microbatch_upstream_grads(1, b, T, H, "f64")
    y, caches = sm.stage_fwd(x, blocks, heads)
    assert np.array_equal(y, x)
    dx, grads = sm.stage_bwd(dy, blocks, caches, heads)
    assert np.allclose(dx, dy, atol=1e-15)
    assert np.allclose(grads[0]["b_2"], dy.reshape(-1, H).sum(0))
    assert np.abs(grads[0]["w_qkv"]).max() == 0.0


def test_planted_mistakes_are_caught(monkeypatch):
    """A dropped term, a wrong sign and a transposed operand in the oracle each break a pin."""
    def fd_fails():
        try:
            test_stage_backward_by_finite_differences()
        except AssertionError:
            return True
        return False

    good = sm.gelu_grad
    monkeypatch.setattr(sm, "gelu_grad", lambda u: 0.5 * (1 + np.tanh(sm.SQRT_2_OVER_PI * (u + sm.GELU_C * u ** 3))))
    assert fd_fails()                                               # dropped term
    monkeypatch.setattr(sm, "gelu_grad", good)
    good_ln = sm.layernorm_bwd

    def bad_ln(dy, cache, gamma):
        dx, dg, db = good_ln(dy, cache, gamma)
        xhat, rstd = cache
        g = dy * gamma
        return rstd * (g - g.mean(-1, keepdims=True) + xhat * (g * xhat).mean(-1, keepdims=True)), dg, db
    monkeypatch.setattr(sm, "layernorm_bwd", bad_ln)
    assert fd_fails()                                               # wrong sign
    monkeypatch.setattr(sm, "layernorm_bwd", good_ln)
    good_att = sm.attention_bwd

    def bad_att(do, q, k, v, p):
        dq, dk, dv = good_att(do, q, k, v, p)
        return dk, dq, dv                                           # swapped operands
    monkeypatch.setattr(sm, "attention_bwd", bad_att)
    assert fd_fails()
    monkeypatch.setattr(sm, "attention_bwd", good_att)
    assert not fd_fails()


def test_flop_model():
    # 3 * L * m * (24 H^2 + 4 T H c)
    assert sm.stage_flops(6, 4, 1024, 1024, causal=True) == 3 * 6 * 4096 * (24 * 1024 ** 2 + 2 * 1024 * 1024)
    assert sm.stage_flops(1, 1, 8, 4, causal=False) == sm.stage_flops(1, 1, 8, 4, causal=True, megatron=True)

"""Stage computation of the oracle: a stack of pre-LN GPT blocks, float64.

The paper (Table "GPT model test configurations"; Section 2.4, a stage
computation is run once per micro-batch, forward and backward) only says the
stages are slices of a GPT.  The block below is the standard GPT-2 block; the
choices the paper leaves open are fixed as follows:
  * pre-LayerNorm, biased variance over the hidden axis, eps inside the root
  * fused QKV projection, columns ordered [Q | K | V], head j owning columns
    j*d .. (j+1)*d of each third; softmax(q k^T / sqrt(d)) with optional causal mask
  * GELU in its tanh form 0.5 u (1 + tanh(sqrt(2/pi) (u + 0.044715 u^3)))
  * biases on all four linear maps, no dropout, matrices stored [in, out]
  * no embedding, final norm, head or loss: the stage maps X [b,T,H] to Y [b,T,H];
    its backward maps an upstream gradient dY to dX and parameter gradients.

Every function is the textbook definition written out, with a matrix product
as the only library step.  TEST INFRASTRUCTURE: not imported by the product.
"""
import numpy as np

SQRT_2_OVER_PI = np.sqrt(2.0 / np.pi)
GELU_C = 0.044715


# ---- LayerNorm --------------------------------------------------------------------------------

def layernorm_fwd(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (x - mu) * rstd
    return xhat * gamma + beta, (xhat, rstd)


def layernorm_bwd(dy, cache, gamma):
    xhat, rstd = cache
    dgamma = (dy * xhat).reshape(-1, xhat.shape[-1]).sum(axis=0)
    dbeta = dy.reshape(-1, dy.shape[-1]).sum(axis=0)
    g = dy * gamma
    dx = rstd * (g - g.mean(axis=-1, keepdims=True) - xhat * (g * xhat).mean(axis=-1, keepdims=True))
    return dx, dgamma, dbeta


# ---- GELU (tanh form) ---------------------------------------------------------------------------

def gelu(u):
    return 0.5 * u * (1.0 + np.tanh(SQRT_2_OVER_PI * (u + GELU_C * u ** 3)))


def gelu_grad(u):
    t = np.tanh(SQRT_2_OVER_PI * (u + GELU_C * u ** 3))
    dt = (1.0 - t * t) * SQRT_2_OVER_PI * (1.0 + 3.0 * GELU_C * u * u)
    return 0.5 * (1.0 + t) + 0.5 * u * dt


# ---- attention -----------------------------------------------------------------------------------

def attention_fwd(q, k, v, causal):
    """q, k, v: [b, h, T, d].  Returns o [b, h, T, d] and the probabilities P [b, h, T, T]."""
    T, d = q.shape[-2], q.shape[-1]
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(d)
    if causal:
        allowed = np.tril(np.ones((T, T), dtype=bool))
        s = np.where(allowed, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    p = e / e.sum(axis=-1, keepdims=True)
    return np.matmul(p, v), p


def attention_bwd(do, q, k, v, p):
    d = q.shape[-1]
    dv = np.matmul(np.swapaxes(p, -1, -2), do)
    dp = np.matmul(do, np.swapaxes(v, -1, -2))
    ds = p * (dp - (dp * p).sum(axis=-1, keepdims=True))
    dq = np.matmul(ds, k) / np.sqrt(d)
    dk = np.matmul(np.swapaxes(ds, -1, -2), q) / np.sqrt(d)
    return dq, dk, dv


def _split_heads(t, heads):
    b, T, H = t.shape
    return t.reshape(b, T, heads, H // heads).transpose(0, 2, 1, 3)


def _merge_heads(t):
    b, h, T, d = t.shape
    return t.transpose(0, 2, 1, 3).reshape(b, T, h * d)


# ---- one block ------------------------------------------------------------------------------------

def block_fwd(x, p, heads, causal=True, eps=1e-5):
    """x [b, T, H]; p: dict of the block's parameters.  Returns y and everything backward needs."""
    H = x.shape[-1]
    a, ln1 = layernorm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    qkv = a @ p["w_qkv"] + p["b_qkv"]
    q, k, v = (_split_heads(qkv[..., i * H:(i + 1) * H], heads) for i in range(3))
    oh, prob = attention_fwd(q, k, v, causal)
    o = _merge_heads(oh)
    x1 = x + o @ p["w_o"] + p["b_o"]
    c, ln2 = layernorm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    u = c @ p["w_1"] + p["b_1"]
    g = gelu(u)
    y = x1 + g @ p["w_2"] + p["b_2"]
    cache = dict(ln1=ln1, a=a, q=q, k=k, v=v, prob=prob, o=o, ln2=ln2, c=c, u=u, g=g)
    return y, cache


def _rows(t):
    return t.reshape(-1, t.shape[-1])


def block_bwd(dy, p, cache, heads):
    """Chain rule through block_fwd, last operation first.  Returns dx and a dict of gradients."""
    gr = {}
    # y = x1 + g W2 + b2
    gr["b_2"] = _rows(dy).sum(axis=0)
    gr["w_2"] = _rows(cache["g"]).T @ _rows(dy)
    dg = dy @ p["w_2"].T
    # g = gelu(u);  u = c W1 + b1
    du = dg * gelu_grad(cache["u"])
    gr["b_1"] = _rows(du).sum(axis=0)
    gr["w_1"] = _rows(cache["c"]).T @ _rows(du)
    dc = du @ p["w_1"].T
    # c = LN2(x1); x1 also feeds the residual
    dx1_ln, gr["ln2_g"], gr["ln2_b"] = layernorm_bwd(dc, cache["ln2"], p["ln2_g"])
    dx1 = dy + dx1_ln
    # x1 = x + o Wo + bo
    gr["b_o"] = _rows(dx1).sum(axis=0)
    gr["w_o"] = _rows(cache["o"]).T @ _rows(dx1)
    do = dx1 @ p["w_o"].T
    # o = attention(q, k, v)
    dq, dk, dv = attention_bwd(_split_heads(do, heads), cache["q"], cache["k"], cache["v"], cache["prob"])
    dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1)
    # qkv = a Wqkv + bqkv
    gr["b_qkv"] = _rows(dqkv).sum(axis=0)
    gr["w_qkv"] = _rows(cache["a"]).T @ _rows(dqkv)
    da = dqkv @ p["w_qkv"].T
    # a = LN1(x); x also feeds the residual
    dx_ln, gr["ln1_g"], gr["ln1_b"] = layernorm_bwd(da, cache["ln1"], p["ln1_g"])
    return dx1 + dx_ln, gr


# ---- the stage: L blocks ----------------------------------------------------------------------------

def stage_fwd(x, blocks, heads, causal=True, eps=1e-5):
    caches = []
    for p in blocks:
        x, cache = block_fwd(x, p, heads, causal, eps)
        caches.append(cache)
    return x, caches


def stage_bwd(dy, blocks, caches, heads):
    grads = [None] * len(blocks)
    for l in range(len(blocks) - 1, -1, -1):
        dy, grads[l] = block_bwd(dy, blocks[l], caches[l], heads)
    return dy, grads


def stage_flops(L, b, T, H, causal=True, megatron=False):
    """Model FLOPs of forward+backward of one micro-batch: 3 * L * m * (24 H^2 + 4 T H c),
    c = 1/2 under a causal mask (the masked half need not be computed), c = 1 otherwise or
    when `megatron` asks for the convention of the paper's throughput plots (Section 6.2.2)."""
    c = 0.5 if (causal and not megatron) else 1.0
    return 3.0 * L * (b * T) * (24.0 * H * H + 4.0 * T * H * c)

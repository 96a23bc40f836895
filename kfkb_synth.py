"""Seeded synthetic inputs for the kFkB stage engine and for its CPU oracle.

This module holds no arithmetic of the method itself: it only produces numbers.
Both the oracle (tests) and the HIP path (tests, smoke, bench) draw their inputs
from here so that the two sides see bit-identical data.

Generator: counter-based.  Draw i of stream `seed` is splitmix64 applied to the
64-bit counter (seed * 2^32 + i); two consecutive draws feed one Box-Muller
pair.  Everything is a pure function of (seed, index), so any slice of a stream
can be regenerated independently and in any order.

Recipe (stands in for the GPT workloads of the paper's Table "GPT model test
configurations", whose training data the paper does not name):
  * weight matrices, biases, LayerNorm beta ~ N(0, 0.02); LayerNorm gamma = 1 + N(0, 0.02)
  * stage inputs X_mb and upstream gradients dY_mb ~ N(0, 1), shape [b, T, H]
  * seeds: weights 1234 (+ block index and tensor index), inputs 1000 + mb,
    upstream gradients 2000 + mb, transfer delays 4242
"""
import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)

PARAM_ORDER = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
               "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def param_shapes(H, F):
    """Shapes of one block's parameter tensors, matrices stored [in, out]."""
    return {"ln1_g": (H,), "ln1_b": (H,), "w_qkv": (H, 3 * H), "b_qkv": (3 * H,),
            "w_o": (H, H), "b_o": (H,), "ln2_g": (H,), "ln2_b": (H,),
            "w_1": (H, F), "b_1": (F,), "w_2": (F, H), "b_2": (H,)}


def _splitmix64(ctr):
    with np.errstate(over="ignore"):
        z = (ctr + np.uint64(0x9E3779B97F4A7C15)) & _MASK
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
        return z ^ (z >> np.uint64(31))


def uniform(seed, n, start=0):
    """n doubles in (0, 1): draws start .. start+n-1 of stream `seed`."""
    with np.errstate(over="ignore"):
        ctr = (np.uint64(seed) << np.uint64(32)) + np.arange(start, start + n, dtype=np.uint64)
    bits = _splitmix64(ctr) >> np.uint64(11)
    return (bits.astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed, n, mean=0.0, std=1.0, chunk=1 << 22):
    """n doubles ~ N(mean, std^2) from stream `seed` (Box-Muller on uniform pairs)."""
    out = np.empty(n, dtype=np.float64)
    pairs = (n + 1) // 2
    for p0 in range(0, pairs, chunk):
        p1 = min(pairs, p0 + chunk)
        u = uniform(seed, 2 * (p1 - p0), start=2 * p0)
        r = np.sqrt(-2.0 * np.log(u[0::2]))
        th = 2.0 * np.pi * u[1::2]
        z = np.empty(2 * (p1 - p0))
        z[0::2] = r * np.cos(th)
        z[1::2] = r * np.sin(th)
        hi = min(n, 2 * p1)
        out[2 * p0:hi] = z[:hi - 2 * p0]
    return out * std + mean


def round_to_bf16(x):
    """Round to the nearest bfloat16-representable value (ties to even); returns float32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32).reshape(f.shape)


def _condition(x, dtype):
    if dtype == "bf16":
        return round_to_bf16(x).astype(np.float64)
    if dtype == "f16":
        return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype == "f64":
        return x
    raise ValueError("dtype must be 'f32', 'bf16', 'f16' or 'f64'")


def stage_weights(L, H, F, dtype="f32", seed=1234, std=0.02):
    """List of L dicts (PARAM_ORDER keys) of float64 arrays whose values are exactly
    representable in `dtype`."""
    blocks = []
    for l in range(L):
        blk = {}
        shapes = param_shapes(H, F)
        for t, name in enumerate(PARAM_ORDER):
            shp = shapes[name]
            n = int(np.prod(shp))
            v = normal(seed + 101 * l + t, n, 0.0, std)
            if name in ("ln1_g", "ln2_g"):
                v = v + 1.0
            blk[name] = _condition(v, dtype).reshape(shp)
        blocks.append(blk)
    return blocks


def stage_weights_tiled(L, H, F, dtype="bf16", seed=1234, std=0.02, period=(1 << 22) + 17, out=np.float64):
    """Weights of the large stages (hundreds of millions of parameters per block) without drawing every value:
    ONE seeded draw of `period` N(0, std^2) values, repeated cyclically; tensor t of block l starts at offset
    (12 l + t) * 7919 of the cycle, so that blocks and tensors differ, and the odd period keeps rows of a matrix
    from repeating.  Same dict layout and conditioning as stage_weights; arrays of type `out` (float64 like
    stage_weights, or float32, which holds every 16-bit value exactly and halves the host memory)."""
    base = normal(seed, period, 0.0, std)
    cond = _condition(base, dtype).astype(out)                 # conditioning is element-wise: condition once, then repeat
    blocks = []
    for l in range(L):
        blk = {}
        shapes = param_shapes(H, F)
        for t, name in enumerate(PARAM_ORDER):
            shp = shapes[name]
            n = int(np.prod(shp))
            start = ((12 * l + t) * 7919) % period
            if name in ("ln1_g", "ln2_g"):                     # 1 + N(0, std^2), conditioned after the shift
                idx = (start + np.arange(n)) % period
                blk[name] = _condition(base[idx] + 1.0, dtype).astype(out).reshape(shp)
                continue
            v = np.empty(n, dtype=out)
            first = min(n, period - start)
            v[:first] = cond[start:start + first]
            pos = first
            while pos < n:
                cnt = min(period, n - pos)
                v[pos:pos + cnt] = cond[:cnt]
                pos += cnt
            blk[name] = v.reshape(shp)
        blocks.append(blk)
    return blocks


def microbatch_inputs(mb, b, T, H, dtype="f32", seed=1000):
    return _condition(normal(seed + mb, b * T * H), dtype).reshape(b, T, H)


def microbatch_upstream_grads(mb, b, T, H, dtype="f32", seed=2000):
    return _condition(normal(seed + mb, b * T * H), dtype).reshape(b, T, H)


# ---- per-transfer delay sequences (nanoseconds), indexed by transfer number -------------------

def delays_none(n):
    return np.zeros(n, dtype=np.int64)


def delays_lognormal(n, mean_ms=2.0, sigma=0.5, seed=4242):
    """Lognormal with the given *mean* (not median): mu = ln(mean) - sigma^2/2."""
    mu = np.log(mean_ms) - 0.5 * sigma * sigma
    return np.round(np.exp(mu + sigma * normal(seed, n)) * 1e6).astype(np.int64)


def delays_bimodal(n, lo_ms=0.5, hi_ms=10.0, p_lo=0.7, seed=4242):
    u = uniform(seed, n)
    return np.where(u < p_lo, lo_ms, hi_ms).__mul__(1e6).round().astype(np.int64)


def delays_drift(n, iteration, n_iterations, end_ms=20.0):
    """Deterministic drift: every transfer of iteration i is delayed end_ms * i / (n_iterations-1)."""
    frac = 0.0 if n_iterations <= 1 else iteration / (n_iterations - 1)
    return np.full(n, int(round(end_ms * frac * 1e6)), dtype=np.int64)

"""kFkB micro-batch order of one stage, its memory consequence, and one iteration.

Follows the paper's two statements of the plan:
  (A) Section 1 / 3.2.1: k forwards then k backwards form one schedule unit, units
      alternate, and between units the early-backward rule of 1F1B holds (the oldest
      pending backward group runs as soon as possible); k = 1 is 1F1B, k = M is GPipe.
  (B) Section 5 / 5.4: take k copies of the 1F1B sequence and cross-merge them.
`kfkb_order` writes (A) out; `kfkb_order_by_interleave` writes (B) out; tests require
the two to agree.  Readings where the paper is silent:
  * inside a group, forwards and backwards run in ascending micro-batch index;
  * a stage with w warm-up groups runs w forward groups before the first
    forward/backward pair; stage s of S has w = min(S-1-s, G), the last stage w = 0;
  * M not divisible by k leaves a shorter last group.

TEST INFRASTRUCTURE: not imported by the product.
"""
import numpy as np
from . import stage_math

F, B = "F", "B"


def groups_of(k, M):
    return [list(range(g0, min(g0 + k, M))) for g0 in range(0, M, k)]


def warmup_groups(num_stages, stage_index, k, M):
    G = -(-M // k)
    return min(num_stages - 1 - stage_index, G)


def kfkb_order(k, M, w=0):
    """Statement (A).  Returns [(F|B, mb), ...] of length 2M."""
    if not (1 <= k <= M) or w < 0:
        raise ValueError("need 1 <= k <= M and w >= 0")
    groups = groups_of(k, M)
    G = len(groups)
    w = min(w, G)
    order = []
    for g in range(w):                       # warm-up: forwards only
        order += [(F, mb) for mb in groups[g]]
    for i in range(G - w):                   # steady: one forward group, then the oldest backward group
        order += [(F, mb) for mb in groups[w + i]]
        order += [(B, mb) for mb in groups[i]]
    for g in range(G - w, G):                # cool-down: backwards only
        order += [(B, mb) for mb in groups[g]]
    return order


def one_f_one_b_order(M, w=0):
    """The base 1F1B sequence of a stage that runs w forwards ahead (Section 2.3)."""
    w = min(w, M)
    seq, nf, nb = [], 0, 0
    while nb < M:
        if nf < M and nf - nb <= w - 1:      # still filling the warm-up window
            seq.append((F, nf)); nf += 1
        elif nf < M:                         # steady state: one forward, then one backward
            seq.append((F, nf)); nf += 1
            seq.append((B, nb)); nb += 1
        else:                                # no forwards left
            seq.append((B, nb)); nb += 1
    return seq


def kfkb_order_by_interleave(k, M, w=0):
    """Statement (B): copy c owns micro-batches c, c+k, c+2k, ...; each copy runs 1F1B on its
    own micro-batches; the merged plan takes position p of every copy, copies in ascending
    order, for p = 0, 1, 2, ..."""
    copies = []
    for c in range(k):
        mine = list(range(c, M, k))
        copies.append([(op, mine[j]) for op, j in one_f_one_b_order(len(mine), w)])
    merged = []
    for p in range(max(len(c) for c in copies)):
        for c in copies:
            if p < len(c):
                merged.append(c[p])
    return merged


def live_counts(order):
    """Number of micro-batches whose activations are held, after each op of the order."""
    live, out = 0, []
    for op, _ in order:
        live += 1 if op == F else -1
        out.append(live)
    return out


def peak_live(order):
    return max(live_counts(order))


def activation_bytes_per_microbatch(L, b, T, H, heads, F_mlp, elem_bytes, recompute=False):
    """Bytes one micro-batch keeps from its forward until its backward (Section 4.1: the
    forward activations must be preserved until the backward completes).  Per block, in the
    stage's storage type: block input x, LN1 output, qkv (3), attention output, x1, LN2 output
    (1 each), MLP pre-activation u and activation g (F/H each); in fp32: mean and rstd of both
    LayerNorms per token and the softmax log-sum-exp per (head, token).
    recompute (Section 2.2, gradient checkpointing lets more micro-batches in): the two
    LayerNorm outputs and g are formed again in the backward pass instead of being kept."""
    m = b * T
    n = m * H
    kept = (6 * n + m * F_mlp) if recompute else (8 * n + 2 * m * F_mlp)
    per_block = kept * elem_bytes + (4 * m + b * heads * T) * 4
    return L * per_block


def plan_activation_bytes(k, M, w, L, b, T, H, heads, F_mlp, elem_bytes):
    return peak_live(kfkb_order(k, M, w)) * activation_bytes_per_microbatch(L, b, T, H, heads, F_mlp, elem_bytes)


def largest_admissible_k(M, w, mem_limit, per_mb_bytes):
    """Largest k dividing M whose plan fits the limit (Section 4.2: walk k upward, keep what fits).
    Returns 0 if even k = 1 does not fit."""
    best = 0
    for k in range(1, M + 1):
        if M % k == 0 and peak_live(kfkb_order(k, M, w)) * per_mb_bytes <= mem_limit:
            best = k
    return best


def enumerate_candidates(global_batch, mem_limit, bytes_per_sample, num_stages=1, stage_index=0, k_max=None):
    """Candidate plans (k, b) on the memory-limit curve at a fixed global batch (Section 4.2, "Pruning for
    Candidate Set": walk the group size k upward from 1 and, for each, greedily take the LARGEST micro-batch
    size b the device accepts; combinations under the curve waste memory, those above it do not fit).
    Readings: b must divide the global batch (M = global_batch / b micro-batches, M >= k); a plan's need is
    its peak of live micro-batches times b times the bytes one sample keeps (activation memory is linear in b);
    the walk stops at the first k for which even b = 1 does not fit, or at k_max.
    Returns [(k, b), ...] in ascending k."""
    out = []
    k = 1
    while k <= global_batch and (k_max is None or k <= k_max):
        best = 0
        for b in range(global_batch, 0, -1):
            if global_batch % b:
                continue
            M = global_batch // b
            if M < k:
                continue
            w = warmup_groups(num_stages, stage_index, k, M)
            if peak_live(kfkb_order(k, M, w)) * b * bytes_per_sample <= mem_limit:
                best = b
                break
        if best == 0:
            break
        out.append((k, best))
        k += 1
    return out


def run_iteration(order, blocks, xs, dys, heads, causal=True, eps=1e-5):
    """Execute a plan: forwards stash their caches, backwards consume them and add their
    parameter gradients into the accumulator in the order they run (Section 2.4: gradient
    accumulation nodes stitch the micro-batches together).  Returns (G, Y, dX, max_live)."""
    M = len(xs)
    G = [{n: np.zeros_like(v) for n, v in p.items()} for p in blocks]
    Y, dX, stash = [None] * M, [None] * M, {}
    max_live = 0
    for op, mb in order:
        if op == F:
            if mb in stash or Y[mb] is not None:
                raise RuntimeError("forward of micro-batch %d issued twice" % mb)
            Y[mb], stash[mb] = stage_math.stage_fwd(xs[mb], blocks, heads, causal, eps)
            max_live = max(max_live, len(stash))
        else:
            if mb not in stash:
                raise RuntimeError("backward of micro-batch %d before its forward" % mb)
            dX[mb], grads = stage_math.stage_bwd(dys[mb], blocks, stash.pop(mb), heads)
            for Gl, gl in zip(G, grads):
                for n in Gl:
                    Gl[n] += gl[n]
    return G, Y, dX, max_live

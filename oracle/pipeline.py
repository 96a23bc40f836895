"""A pipeline of S stages, every stage under its own kFkB plan (Sections 2.2, 3.2.1 and 5 of the paper).

What the paper fixes: a model is cut into S consecutive stages, one per worker; stage s forwards a
micro-batch after stage s-1 has, and backwards it after stage s+1 has; every stage follows the kFkB
order with the early-backward rule, which for stage s of S means w = min(S-1-s, G) warm-up groups
(`schedule.warmup_groups`), so that earlier stages hold more live micro-batches (Section 3.2.1: the
memory a plan needs grows towards the first stage).  The result of an iteration does not depend on
S or k (Section 1: the plans are mathematically equivalent).

What it leaves open, and the reading taken here:
  * the order in which ONE executor that owns all S stages (a single GPU standing in for S workers)
    issues the ops is not the paper's concern.  `list_schedule` fixes one: imagine every stage on a
    device of its own, forward 1 time unit, backward 2 (the paper's own assumption, Section 4.1),
    transfers free; repeatedly issue, among the stages whose next op has its producers issued, the
    op that would start earliest on that imaginary pipeline; ties go to the later stage.  Integer
    times, so the rule is exact and the library can be required to issue the same sequence.
  * `simulate` is the timing of that imaginary pipeline with a fixed transfer time per boundary
    crossing.  It is a performance model: beyond its closed forms (no transfer time: k = 1 and
    k = M both take (M + S - 1)(f + b)) it is parity unpinned.

TEST INFRASTRUCTURE: not imported by the product.
"""
import numpy as np
from . import schedule, stage_math

F, B = schedule.F, schedule.B


def stage_orders(S, k, M):
    """The kFkB plan of every stage: [[(F|B, mb), ...] for s in range(S)]."""
    return [schedule.kfkb_order(k, M, schedule.warmup_groups(S, s, k, M)) for s in range(S)]


def _timeline(S, k, M, t_fwd, t_bwd, t_comm):
    """Issues every op of every stage's plan in list-schedule order on the imaginary S-device pipeline.
    Returns ([(stage, op, mb)], {(stage, op, mb): (start, finish)})."""
    orders = stage_orders(S, k, M)
    nxt = [0] * S                      # position in each stage's plan
    clock = [0] * S                    # when each stage's device is free
    done = {}                          # (stage, op, mb) -> finish time
    issued, times = [], {}
    total = 2 * M * S
    while len(issued) < total:
        best = None
        for s in range(S):
            if nxt[s] >= len(orders[s]):
                continue
            op, mb = orders[s][nxt[s]]
            if op == F:
                deps = [(s - 1, F, mb)] if s > 0 else []
            else:
                deps = [(s, F, mb)] + ([(s + 1, B, mb)] if s < S - 1 else [])
            if any(d not in done for d in deps):
                continue
            ready = 0
            for d in deps:
                ready = max(ready, done[d] + (t_comm if d[0] != s else 0))
            start = max(clock[s], ready)
            if best is None or start < best[0] or (start == best[0] and s > best[1]):
                best = (start, s, op, mb)
        if best is None:
            raise RuntimeError("the plans dead-lock (S=%d k=%d M=%d)" % (S, k, M))
        start, s, op, mb = best
        finish = start + (t_fwd if op == F else t_bwd)
        clock[s] = finish
        done[(s, op, mb)] = finish
        times[(s, op, mb)] = (start, finish)
        issued.append((s, op, mb))
        nxt[s] += 1
    return issued, times


def list_schedule(S, k, M):
    """The order in which one executor issues the ops of all S stages (see the module text): forward 1,
    backward 2, transfers free, earliest imaginary start first, ties to the later stage."""
    return _timeline(S, k, M, 1, 2, 0)[0]


def simulate(S, k, M, t_fwd, t_bwd, t_comm=0.0):
    """Length of one iteration on S devices, one stage each, every boundary crossing taking t_comm."""
    _, times = _timeline(S, k, M, t_fwd, t_bwd, t_comm)
    return max(f for _, f in times.values())


def run_pipeline(S, k, blocks, xs, dys, heads, causal=True, eps=1e-5):
    """One iteration of the S-stage pipeline in list-schedule order: stage s owns blocks
    [s L/S, (s+1) L/S); a forward hands its output to the next stage, a backward hands the gradient
    of its input to the previous stage, parameter gradients are accumulated in the order the
    backwards run.  Returns (G, Y, dX, max_live per stage, issued order)."""
    L, M = len(blocks), len(xs)
    if L % S != 0:
        raise ValueError("the blocks do not divide into %d stages" % S)
    Ls = L // S
    order = list_schedule(S, k, M)
    G = [{n: np.zeros_like(v) for n, v in p.items()} for p in blocks]
    Y, dX = [None] * M, [None] * M
    act, grad, caches = {}, {}, {}
    live, max_live = [0] * S, [0] * S
    for s, op, mb in order:
        mine = blocks[s * Ls:(s + 1) * Ls]
        if op == F:
            x = xs[mb] if s == 0 else act.pop((s - 1, mb))        # KeyError: issued before its producer
            y, caches[(s, mb)] = stage_math.stage_fwd(x, mine, heads, causal, eps)
            live[s] += 1
            max_live[s] = max(max_live[s], live[s])
            if s == S - 1:
                Y[mb] = y
            else:
                act[(s, mb)] = y
        else:
            dy = dys[mb] if s == S - 1 else grad.pop((s + 1, mb))
            dx, grads = stage_math.stage_bwd(dy, mine, caches.pop((s, mb)), heads)
            live[s] -= 1
            for Gl, gl in zip(G[s * Ls:(s + 1) * Ls], grads):
                for n in Gl:
                    Gl[n] += gl[n]
            if s == 0:
                dX[mb] = dx
            else:
                grad[(s, mb)] = dx
    return G, Y, dX, max_live, order

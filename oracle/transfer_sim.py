"""Discrete-event model of one stage's iteration under delayed inter-stage transfers.

What it models (the asynchronous point-to-point design of Section 5.3 and the buffer-queue
argument of Section 4.4, reduced to one device whose neighbours do no compute):
  * three FIFO resources: the compute stream, one receive stream, one send stream;
    successive transfers on a stream are serialised (a receive starts after the previous
    one has completed);
  * a transfer takes its injected delay plus its copy time;
  * send Y_mb starts when F(mb) ends; send dX_mb starts when B(mb) ends;
  * "echo neighbour": the upstream gradient dY_mb can start arriving only after Y_mb has
    been fully sent;
  * the receive stream is fed in a fixed list order, each receive issued as early as the
    list and the pools allow: a pool of input slots (live + k) and of gradient slots (2k);
    a slot returns to its pool when the backward that read it ends.  The list is the
    schedule's consumption order (the upstream gradients of a unit, then the inputs of the
    next forward unit, which so arrive while the unit's backwards run), or, "inputs
    ahead", that order with every forward unit's receives moved one schedule unit earlier;
    the default takes inputs ahead for k = 1 only (there a unit is one micro-batch and the
    next input can only hide behind the current forward), since for k >= 2 a backward unit
    would wait behind k input transfers;
  * an op starts when the previous op has ended and its input has arrived.
Output buffers are modelled as unbounded.

This is a performance model, not a result: beyond the closed-form cases in its tests it
is "parity unpinned".  TEST INFRASTRUCTURE: not imported by the product.
"""
from . import schedule

F, B = schedule.F, schedule.B


def receive_plan(order, inputs_ahead=True):
    """The receive list: the consumption order itself, or (inputs_ahead) that order with each forward unit moved
    ahead of the backward unit before it."""
    if not inputs_ahead:
        return list(order)
    units = []
    for op, mb in order:
        if units and units[-1][0] == op:
            units[-1][1].append(mb)
        else:
            units.append((op, [mb]))
    i = 0
    while i + 1 < len(units):
        if units[i][0] == B and units[i + 1][0] == F:
            units[i], units[i + 1] = units[i + 1], units[i]
            i += 2
        else:
            i += 1
    return [(op, mb) for op, mbs in units for mb in mbs]


def simulate(order, k, t_fwd, t_bwd, delay_recv_x, delay_recv_dy, delay_send_y, delay_send_dx,
             t_copy=0.0, x_slots=None, dy_slots=None, inputs_ahead=None):
    """All times in one unit (say ms).  t_fwd / t_bwd: scalars or per-micro-batch lists.
    x_slots / dy_slots override the pool sizes (defaults: peak live + k, and 2k).
    inputs_ahead: the receive list (see receive_plan); None = ahead exactly for k == 1.
    Returns dict(total=..., start=[...], end=[...], stall=...) with per-op compute times."""
    M = len(order) // 2
    tf = t_fwd if hasattr(t_fwd, "__len__") else [t_fwd] * M
    tb = t_bwd if hasattr(t_bwd, "__len__") else [t_bwd] * M
    live_peak = schedule.peak_live(order)
    x_free = [0.0] * (x_slots or live_peak + k)     # times at which input slots become free
    dy_free = [0.0] * (dy_slots or 2 * k)
    plan = receive_plan(order, k == 1 if inputs_ahead is None else inputs_ahead)
    arrive, slot_of = {}, {}
    end_of, sent_y = {}, {}
    start, end = [], []
    t_recv = t_send = t_comp = 0.0
    rp = 0

    def _free_index(pool):
        best = None
        for i, t in enumerate(pool):
            if t is not None and (best is None or t < pool[best]):
                best = i
        return best

    def try_receives():
        nonlocal rp, t_recv
        while rp < len(plan):
            op, mb = plan[rp]
            pool = x_free if op == F else dy_free
            if op == B and mb not in sent_y:
                return
            s = _free_index(pool)
            if s is None:
                return
            begin = max(t_recv, pool[s], sent_y[mb] if op == B else 0.0)
            pool[s] = None
            d = delay_recv_x[mb] if op == F else delay_recv_dy[mb]
            t_recv = begin + d + t_copy
            arrive[(op, mb)] = t_recv
            slot_of[(op, mb)] = s
            rp += 1

    for op, mb in order:
        try_receives()
        if (op, mb) not in arrive:
            raise RuntimeError("receive plan cannot feed %s%d" % (op, mb))
        begin = max(t_comp, arrive[(op, mb)])
        t_comp = begin + (tf[mb] if op == F else tb[mb])
        start.append(begin); end.append(t_comp)
        t_send = max(t_send, t_comp) + (delay_send_y[mb] if op == F else delay_send_dx[mb]) + t_copy
        if op == F:
            sent_y[mb] = t_send
        else:
            x_free[slot_of[(F, mb)]] = t_comp
            dy_free[slot_of[(B, mb)]] = t_comp
    busy = sum(e - s for s, e in zip(start, end))
    total = max(t_comp, t_send, t_recv)
    return dict(total=total, start=start, end=end, stall=end[-1] - busy, compute_end=end[-1])

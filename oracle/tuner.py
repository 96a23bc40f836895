"""Cost model and online choice of the group size k (the auto tuner of the paper).

What the paper says (Sections 3.2.2 "auto tunner", 4.3 "cost model", 5.2 "profiling", 5.4 "online tuning"):
  * the pipeline length of every candidate plan is ESTIMATED from profiled stage computation
    times and profiled cross-stage communication times, and the shortest plan is taken;
  * stage computation times are stable (the device is not shared) and are profiled once per
    plan, averaged over several runs; they are reused afterwards;
  * communication times are measured end to end (not derived from a bandwidth), several times,
    and "the moving average of these results" over a window is what the model uses; they are
    re-profiled at regular intervals because the network changes;
  * the tuner is triggered at regular intervals and the plan it picks takes effect at once;
    switching plans moves no parameters.
What it does not say, and the reading taken here:
  * the estimator itself is not printed.  For one stage whose neighbours do no compute the
    pipeline length is the iteration time of the transfer rules of Section 5.3, so the
    estimator is `transfer_sim.simulate` fed the averaged times (every transfer of a
    direction takes that direction's moving average);
  * candidates that do not fit the activation limit are not evaluated (Section 4.2 / 5.1);
  * ties go to the smaller k (less activation memory, Section 3.1);
  * the window holds the last `window` ITERATION means of each direction (one sample per
    iteration and direction: the mean of that iteration's transfers).

A heuristic: beyond the closed-form cases in its tests it is "parity unpinned".
TEST INFRASTRUCTURE: not imported by the product.
"""
from . import schedule
from . import transfer_sim

DIRECTIONS = ("recv_x", "recv_dy", "send_y", "send_dx")


class Window:
    """Moving average of the last `size` samples."""

    def __init__(self, size):
        if size < 1:
            raise ValueError("window size must be positive")
        self.size = size
        self.samples = []

    def push(self, v):
        self.samples.append(float(v))
        if len(self.samples) > self.size:
            self.samples.pop(0)

    def mean(self):
        return sum(self.samples) / len(self.samples) if self.samples else 0.0


def predict(k, M, w, t_fwd, t_bwd, comm, x_slots=None, dy_slots=None, inputs_ahead=None):
    """Estimated iteration time of plan (k, M, w).  comm: dict direction -> time of one transfer.
    inputs_ahead: the receive list of transfer_sim.receive_plan; None = its default by k."""
    order = schedule.kfkb_order(k, M, w)
    c = [[comm[d]] * M for d in DIRECTIONS]
    return transfer_sim.simulate(order, k, t_fwd, t_bwd, c[0], c[1], c[2], c[3], 0.0, x_slots, dy_slots, inputs_ahead)["total"]


def choose(candidates, M, w, compute_profile, comm, mem_limit=0, per_mb_bytes=0):
    """The admissible candidate with the shortest estimated iteration; ties -> smaller k.
    compute_profile: dict k -> (t_fwd, t_bwd), profiled once per plan.
    Returns (k, {k: estimate})."""
    est = {}
    for k in sorted(candidates):
        if not (1 <= k <= M) or k not in compute_profile:
            continue
        live = min((min(w, -(-M // k)) + 1) * k, M)
        if mem_limit and live * per_mb_bytes > mem_limit:
            continue
        tf, tb = compute_profile[k]
        est[k] = predict(k, M, w, tf, tb, comm)
    if not est:
        raise ValueError("no admissible candidate")
    best = min(sorted(est), key=lambda k: est[k])
    return best, est


class Tuner:
    """Re-evaluates the candidates every `interval` iterations on the moving averages."""

    def __init__(self, candidates, M, w, compute_profile, window=4, interval=4, mem_limit=0, per_mb_bytes=0, k0=None):
        self.candidates, self.M, self.w = list(candidates), M, w
        self.profile = dict(compute_profile)
        self.win = {d: Window(window) for d in DIRECTIONS}
        self.interval = interval
        self.mem_limit, self.per_mb_bytes = mem_limit, per_mb_bytes
        self.k = k0 if k0 is not None else min(self.candidates)
        self.iterations = 0
        self.last_estimates = {}

    def observe(self, transfer_times):
        """transfer_times: dict direction -> list of measured times of one iteration."""
        for d in DIRECTIONS:
            v = transfer_times[d]
            self.win[d].push(sum(v) / len(v))
        self.iterations += 1

    def next_k(self):
        """Group size of the next iteration."""
        if self.iterations > 0 and self.iterations % self.interval == 0:
            comm = {d: self.win[d].mean() for d in DIRECTIONS}
            self.k, self.last_estimates = choose(self.candidates, self.M, self.w, self.profile, comm,
                                                 self.mem_limit, self.per_mb_bytes)
        return self.k

"""Host-side parts of bench.py that need no GPU: the FLOP count it reports against (its own formula, which must stay the
oracle's), the delay models (seeded, the same for every k), the five benchmark configurations, and the refusal of more
than one GPU."""
import os
import subprocess
import sys

import numpy as np

import bench
import kfkb_synth as synth
from oracle import stage_math as sm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_flop_count_is_the_oracles():
    for w in bench.WORKLOADS.values():
        for causal in (True, False):
            for megatron in (False, True):
                assert bench.stage_flops(w["L"], w["b"], w["T"], w["H"], causal, megatron) == \
                    sm.stage_flops(w["L"], w["b"], w["T"], w["H"], causal, megatron)
    # one block, one token row by hand: 3 x (24 H^2 + 4 T H / 2) with T = 1
    assert bench.stage_flops(1, 1, 1, 8) == 3 * (24 * 64 + 2 * 8)


def test_workloads_are_the_five_configurations():
    w = bench.WORKLOADS
    assert (w["tiny-stage"]["H"], w["tiny-stage"]["T"], w["tiny-stage"]["M"], w["tiny-stage"]["dtype"]) == (128, 64, 4, "f32")
    assert (w["gpt2-medium-stage"]["L"], w["gpt2-medium-stage"]["H"], w["gpt2-medium-stage"]["b"], w["gpt2-medium-stage"]["M"]) == (6, 1024, 4, 16)
    assert (w["gpt-1.3b-stage"]["H"], w["gpt-1.3b-stage"]["T"], w["gpt-1.3b-stage"]["M"], w["gpt-1.3b-stage"]["delay"]) == (2048, 2048, 32, "lognormal")
    assert (w["wide-stage"]["H"], w["wide-stage"]["heads"], w["wide-stage"]["limit"], w["wide-stage"]["delay"]) == (4096, 32, 200e9, "bimodal")
    vw = w["very-wide-stage"]
    assert (vw["L"], vw["H"], vw["heads"], vw["T"], vw["b"], vw["M"], vw["ks"], vw["limit"], vw["delay"]) == \
        (2, 8192, 64, 4096, 1, 64, (1, 2, 4, 8), 250e9, "drift")
    for c in w.values():
        assert c["H"] % c["heads"] == 0


def test_delay_models_are_seeded_and_the_drift_ends_at_twenty_milliseconds():
    M = 16
    assert bench.delays_for(synth, "none", M, 3, 10) == (None, None, None, None)
    for model in ("lognormal", "bimodal"):
        a = bench.delays_for(synth, model, M, 3, 10)
        b = bench.delays_for(synth, model, M, 3, 10)
        c = bench.delays_for(synth, model, M, 4, 10)
        assert all(np.array_equal(x, y) for x, y in zip(a, b))            # the same for every k of a step
        assert not all(np.array_equal(x, y) for x, y in zip(a, c))        # and new draws for the next step
        assert all(x.dtype == np.int64 and x.shape == (M,) and (x >= 0).all() for x in a)
    first, last = bench.delays_for(synth, "drift", M, 0, 20), bench.delays_for(synth, "drift", M, 19, 20)
    assert all((x == 0).all() for x in first) and all((x == 20_000_000).all() for x in last)      # nanoseconds
    mid = bench.delays_for(synth, "drift", M, 10, 20)
    assert all(0 < x[0] < 20_000_000 for x in mid)
    fixed = bench.delays_for(synth, "fixed:7.5", M, 0, 1)
    assert all((x == 7_500_000).all() for x in fixed)
    bm = synth.delays_bimodal(4000, 0.5, 10.0, 0.7, seed=1)
    assert set(np.unique(bm)) == {500_000, 10_000_000} and abs((bm == 500_000).mean() - 0.7) < 0.03


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""

"""Host-only checks of the library's cost model and tuner against the oracle's (no GPU compute):
the estimate of an iteration, the moving averages, the evaluation interval and the admission rule."""
import os
import random

import pytest

import paper_2303_01675_amd as kf
from oracle import schedule as sch
from oracle import tuner as tu


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kf.library_path()):
        from paper_2303_01675_amd import build
        build.build()
    return kf.load_library()


def test_estimate_matches_the_oracle_on_random_plans(lib):
    rnd = random.Random(7)
    n = 0
    for it in range(600):
        mode = (2, 0, 1)[it % 3]                      # receive list: by k (the default), consumption order, inputs ahead
        ahead = {2: None, 0: False, 1: True}[mode]
        kf.kfkb_set_inputs_ahead(mode)
        M = rnd.randint(1, 24)
        k = rnd.randint(1, M)
        w = rnd.randint(0, 3)
        tf, tb = rnd.uniform(0.1, 3.0), rnd.uniform(0.1, 5.0)
        comm = {d: rnd.choice([0.0, rnd.uniform(0.0, 0.5), rnd.uniform(0.0, 6.0)]) for d in tu.DIRECTIONS}
        slots = rnd.choice([(0, 0), (0, 0), (None, None)])
        live = sch.peak_live(sch.kfkb_order(k, M, w))
        if slots == (None, None):
            xs, ds = rnd.randint(live, live + 2 * k), rnd.randint(max(1, k), 3 * k)
        else:
            xs, ds = 0, 0
        try:
            want = tu.predict(k, M, w, tf, tb, comm, xs or None, ds or None, ahead)
        except RuntimeError:
            with pytest.raises(kf.KfkbError):
                kf.kfkb_predict_iteration_ms(k, M, w, tf, tb, *[comm[d] for d in tu.DIRECTIONS], xs, ds)
            continue
        got = kf.kfkb_predict_iteration_ms(k, M, w, tf, tb, *[comm[d] for d in tu.DIRECTIONS], xs, ds)
        assert got == pytest.approx(want, rel=1e-12, abs=1e-12), (k, M, w, comm, xs, ds)
        n += 1
    kf.kfkb_set_inputs_ahead(2)
    assert n > 450


def test_estimate_closed_forms(lib):
    # no communication: the sum of the stage times; 1F1B: two transfers exposed per micro-batch (Section 2.5)
    assert kf.kfkb_predict_iteration_ms(4, 8, 0, 1.0, 2.0, 0, 0, 0, 0) == pytest.approx(24.0)
    d = 0.4
    assert kf.kfkb_predict_iteration_ms(1, 8, 0, 1.0, 2.0, d, d, d, d) == pytest.approx(2 * d + 8 * (3.0 + 2 * d))
    for bad in [(0, 8, 0), (9, 8, 0), (1, 0, 0), (1, 8, -1)]:
        with pytest.raises(kf.KfkbError):
            kf.kfkb_predict_iteration_ms(*bad, 1.0, 2.0, 0, 0, 0, 0)


def test_tuner_follows_the_oracle_tuner_on_a_changing_network(lib):
    rnd = random.Random(11)
    for trial in range(6):
        M = rnd.choice([8, 12, 16])
        cands = sorted(rnd.sample([1, 2, 3, 4, 6, 8], rnd.randint(2, 5)))
        window, interval = rnd.randint(1, 4), rnd.randint(1, 4)
        w = rnd.randint(0, 1)
        prof = {k: (rnd.uniform(0.8, 1.2), rnd.uniform(1.6, 2.4)) for k in cands}
        per_mb, limit = 10, rnd.choice([0, 10 * rnd.randint(2, 16)])
        # a limit below the smallest candidate's need is an error on both sides: keep the smallest admissible
        if limit and min((min(w, -(-M // k)) + 1) * k for k in cands) * per_mb > limit:
            limit = 0
        kf.kfkb_tuner_config(window, interval, cands)
        for k in cands:
            kf.kfkb_tuner_set_compute_profile(k, *prof[k])
        ref = tu.Tuner(cands, M, w, prof, window=window, interval=interval, mem_limit=limit, per_mb_bytes=per_mb)
        level = 0.0
        for it in range(40):
            k_ref = ref.next_k()
            k_lib, est = kf.kfkb_tuner_next_k(M, w, limit, per_mb)
            assert k_lib == k_ref, (trial, it)
            for i, k in enumerate(cands):
                if k in ref.last_estimates:
                    assert est[i] == pytest.approx(ref.last_estimates[k], rel=1e-12)
            if it % 7 == 0:
                level = rnd.choice([0.0, 0.2, 0.9, 2.5])
            sample = {d: [level * rnd.uniform(0.8, 1.2) for _ in range(M)] for d in tu.DIRECTIONS}
            ref.observe(sample)
            kf.kfkb_tuner_push_sample(*[sum(sample[d]) / M for d in tu.DIRECTIONS])


def test_tuner_argument_errors(lib):
    for args in [(0, 1, [1]), (1, 0, [1]), (1, 1, []), (1, 1, [1, 1]), (1, 1, [0, 2]), (1, 1, list(range(1, 10)))]:
        with pytest.raises(kf.KfkbError):
            kf.kfkb_tuner_config(*args)
    kf.kfkb_tuner_config(2, 2, [1, 2])
    with pytest.raises(kf.KfkbError):
        kf.kfkb_tuner_set_compute_profile(3, 1.0, 2.0)
    with pytest.raises(kf.KfkbError):
        kf.kfkb_tuner_push_sample(-1.0, 0, 0, 0)
    # no candidate has a profile: the first evaluation cannot choose
    kf.kfkb_tuner_push_sample(0, 0, 0, 0); kf.kfkb_tuner_push_sample(0, 0, 0, 0)
    with pytest.raises(kf.KfkbError):
        kf.kfkb_tuner_next_k(8)


def test_candidate_enumeration_matches_the_oracle(lib):
    rnd = random.Random(5)
    assert kf.kfkb_enumerate_candidates(192, 6 * 10, 10, k_max=6) == [(k, 6 // k) for k in range(1, 7)]   # paper, Section 6.2.1
    for _ in range(200):
        G = rnd.choice([6, 12, 16, 30, 64, 192])
        S = rnd.randint(1, 6); s = rnd.randint(0, S - 1)
        per = rnd.choice([1, 10, 1000])
        limit = per * rnd.randint(0, 3 * G)
        kmax = rnd.choice([0, 0, rnd.randint(1, 8)])
        assert kf.kfkb_enumerate_candidates(G, limit, per, S, s, kmax) == sch.enumerate_candidates(G, limit, per, S, s, kmax or None)
    with pytest.raises(kf.KfkbError):
        kf.kfkb_enumerate_candidates(0, 10, 1)

"""Pins for the oracle's batch-firing policy (paper section 4.4), CPU only: the estimators against
closed forms, the target batch against a brute-force search, the decisions against queueing
behaviour in a virtual-time simulation."""
import math

import numpy as np
import pytest

from oracle.scheduler import BatchTimer
from sched_sim import simulate, poisson_arrivals, Greedy


def test_rate_estimator_constant_and_poisson_gaps():
    t = BatchTimer(64, 200.0)
    assert t.rate() == 0.0
    for k in range(50):
        t.arrive(7.5 * k)
    assert t.rate() == 1.0 / 7.5                                  # constant gaps: exact
    t = BatchTimer(64, 200.0, weight=0.001)                        # relative spread of the estimate: sqrt(w / 2) = 2.2 %
    for x in poisson_arrivals(0.02, 40000, seed=3):
        t.arrive(x)
    assert abs(t.rate() / 0.02 - 1.0) < 0.1                       # mean of exponential gaps = 1 / rate


def test_service_model_recovers_a_line():
    t = BatchTimer(64, 200.0)
    rng = np.random.default_rng(4)
    for b in rng.integers(1, 65, size=200):
        t.done(int(b), 83.0 + 2.75 * int(b))
    assert abs(t.a - 83.0) < 1e-6 and abs(t.c - 2.75) < 1e-8
    # one batch size only: the slope keeps its prior, the intercept absorbs the rest
    t = BatchTimer(64, 200.0, a_us=10.0, c_us=2.0)
    for _ in range(30):
        t.done(8, 100.0)
    assert t.c == 2.0 and abs(t.a - 84.0) < 1e-9


@pytest.mark.parametrize("lam,a,c", [(0.05, 100.0, 2.0), (0.2, 60.0, 1.5), (0.004, 900.0, 20.0), (0.3, 10.0, 3.0)])
def test_target_is_the_smallest_batch_that_keeps_up(lam, a, c):
    """b* solves b = lam * S(b); the smallest INTEGER batch whose service rate b / S(b) reaches lam
    is ceil(b*) (brute force over all batch sizes)."""
    t = BatchTimer(4096, 200.0, a_us=a, c_us=c)
    t.mean_gap, t.n_gaps = 1.0 / lam, 1
    bs = t.target()
    assert abs(bs - lam * (a + c * bs)) < 1e-9 * max(1.0, bs)
    brute = next(b for b in range(1, 4097) if b / (a + c * b) >= lam)
    assert brute == max(1, math.ceil(bs - 1e-12))
    # beyond the GPU's capacity per call: largest batches
    t.mean_gap = c / 1.01
    assert t.target() == 4096.0


def test_light_load_fires_at_once():
    arr = poisson_arrivals(1e-4, 2000, seed=5)                    # a call every 10 ms, service 0.1 ms
    r = simulate(BatchTimer(64, 200.0), arr, 100.0, 2.0)
    assert np.mean(r["batches"]) < 1.05 and np.percentile(r["waits"], 90) == 0.0


def test_moderate_load_batches_near_target_and_bounded_waits():
    lam, a, c, max_wait = 0.05, 100.0, 2.0, 200.0
    arr = poisson_arrivals(lam, 30000, seed=6)
    t = BatchTimer(64, max_wait, a_us=a, c_us=c)
    r = simulate(t, arr, a, c)
    bstar = lam * a / (1 - lam * c)                                # 5.56
    assert abs(t.a - a) < 1e-6 and abs(t.c - c) < 1e-8             # the model was learnt from the run
    assert bstar <= np.mean(r["batches"]) < 2.0 * bstar + 2
    assert r["waits"].max() <= max_wait + a + c * 64 + 1e-9        # deadline + at most one service period
    assert r["end_us"] < arr[-1] + 10 * (a + c * 64)               # kept up with the arrivals
    g = simulate(Greedy(64), arr, a, c)
    # waiting for the target batch costs at most max_wait of latency and never more GPU time than greedy
    assert r["busy_us"] <= g["busy_us"] * 1.001
    assert np.mean(r["waits"]) <= np.mean(g["waits"]) + max_wait


def test_overload_uses_largest_batches_and_terminates():
    arr = poisson_arrivals(1.0, 20000, seed=7)                    # capacity at 64 per batch: 0.28 per us
    r = simulate(BatchTimer(64, 200.0), arr, 100.0, 2.0)
    assert np.all(r["batches"][5:-1] == 64) and r["batches"].sum() == 20000


def test_deadline_fires_a_short_batch_when_arrivals_stop():
    t = BatchTimer(64, 200.0, a_us=100.0, c_us=2.0)
    for k in range(40):
        t.arrive(10.0 * k)                                        # rate 0.1 per us: target 12.5
    t.fired(40)
    t.arrive(400.0)
    t.arrive(410.0)                                               # two calls; ten more are expected within 105 us
    assert t.decide(410.0) == 0 and t.next_deadline() == 600.0
    assert t.decide(500.0) == 2                                   # 100 us left < (12.5 - 2) / 0.1: the target is out of reach
    assert t.decide(600.0) == 2
    assert t.decide(410.0, gpu_idle=False) == 0
    assert t.decide(600.0, gpu_idle=False) == 0                   # nothing is fired into a busy GPU, deadline or not

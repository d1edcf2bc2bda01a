"""Event-driven simulation of one GPU serving batched pred calls in virtual time, used to pin the
firing policy and to compare the library's controller with the oracle's on identical traces."""
import math

import numpy as np


def poisson_arrivals(rate_per_us, n, seed):
    rng = np.random.default_rng(seed)
    return np.cumsum(rng.exponential(1.0 / rate_per_us, size=n))


def simulate(timer, arrivals, a_us, c_us, log=None):
    """timer: object with arrive/decide/fired/done/next_deadline.  The GPU serves a batch of b calls in
    a_us + c_us * b.  Returns dict(waits, batches, busy_us, end_us).  `log`, if a list, receives every
    (time, decision, decision with a busy GPU) triple, waits included."""
    now, k, n = 0.0, 0, len(arrivals)
    pending = []
    waits, batches, busy = [], [], 0.0
    while len(waits) < n:
        while k < n and arrivals[k] <= now:
            timer.arrive(float(arrivals[k]))
            pending.append(float(arrivals[k]))
            k += 1
        fire = timer.decide(now, True)
        if log is not None:
            log.append((now, fire, timer.decide(now, False)))      # and what it would do were the GPU busy
        if fire > 0:
            timer.fired(fire)
            waits += [now - t for t in pending[:fire]]
            del pending[:fire]
            service = a_us + c_us * fire
            batches.append(fire)
            busy += service
            now += service
            timer.done(fire, service)
        else:
            nxt = min(float(arrivals[k]) if k < n else math.inf, timer.next_deadline())
            assert nxt < math.inf and nxt > now, "the policy waits with nothing to wait for"
            now = nxt
    return dict(waits=np.array(waits), batches=np.array(batches), busy_us=busy, end_us=now)


class Greedy:
    """Fire whatever is pending whenever the GPU is idle (the work-conserving baseline)."""

    def __init__(self, max_batch):
        self.max_batch, self.q = max_batch, 0

    def arrive(self, t):
        self.q += 1

    def decide(self, now, idle):
        return min(self.q, self.max_batch)

    def fired(self, n):
        self.q -= n

    def done(self, n, s):
        pass

    def next_deadline(self):
        return math.inf

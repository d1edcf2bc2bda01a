"""Batch-firing policy of the inference scheduler (test infrastructure, CPU only).

The paper (section 4.4) says that the inference scheduler aggregates pred calls into one GPU
batch, that firing too early wastes the GPU and firing too late makes threads wait, and that
the batch size follows the average frequency of the calls, for which it names arrival models
such as the Poisson process.  It gives no formula.  The policy below is this build's reading, written out step by
step in plain floating point (IEEE doubles, one operation at a time, so that the library's
controller can be compared with it decision by decision):

* arrival rate: lambda = 1 / (exponentially weighted mean of the gaps between arrivals);
* service model: a batch of b calls takes S(b) = a + c * b microseconds; a and c come from a
  least-squares line through exponentially weighted moments of the (b, S) pairs seen so far;
* target batch: with Poisson arrivals at rate lambda the expected number of calls that arrive
  during one service period is lambda * S(b); the batch size that just keeps up with the
  arrivals is the fixed point b* = lambda * S(b*) = lambda * a / (1 - lambda * c), and
  max_batch when lambda * c >= 1 (the GPU cannot keep up: largest batches);
* decision, taken whenever the GPU is idle and calls are pending: fire all pending calls (at
  most max_batch) if there are at least b* of them, or if the oldest has waited max_wait, or
  if the expected time to collect the missing ones, (b* - pending) / lambda, does not fit
  into what is left of max_wait; otherwise wait.
"""
import math
from collections import deque


class BatchTimer:
    def __init__(self, max_batch, max_wait_us, weight=0.125, a_us=50.0, c_us=1.0):
        self.max_batch = int(max_batch)
        self.max_wait = float(max_wait_us)
        self.w = float(weight)              # weight of a new sample in every running mean
        self.a = float(a_us)                # fixed cost of a batch, microseconds (prior until measured)
        self.c = float(c_us)                # cost per call, microseconds
        self.mean_gap = 0.0
        self.n_gaps = 0
        self.last_arrival = None
        self.pending = deque()              # arrival times of the calls not yet fired
        # exponentially weighted moments of (b, S)
        self.n_obs = 0
        self.mb = self.ms = self.mbb = self.mbs = 0.0

    # ---- observations ---------------------------------------------------------
    def arrive(self, now_us):
        now_us = float(now_us)
        if self.last_arrival is not None:
            gap = now_us - self.last_arrival
            if self.n_gaps == 0:
                self.mean_gap = gap
            else:
                self.mean_gap = self.mean_gap + self.w * (gap - self.mean_gap)
            self.n_gaps += 1
        self.last_arrival = now_us
        self.pending.append(now_us)

    def done(self, n, service_us):
        """A batch of n calls took service_us: refit S(b) = a + c b."""
        b, s = float(n), float(service_us)
        if self.n_obs == 0:
            self.mb, self.ms, self.mbb, self.mbs = b, s, b * b, b * s
        else:
            self.mb = self.mb + self.w * (b - self.mb)
            self.ms = self.ms + self.w * (s - self.ms)
            self.mbb = self.mbb + self.w * (b * b - self.mbb)
            self.mbs = self.mbs + self.w * (b * s - self.mbs)
        self.n_obs += 1
        var = self.mbb - self.mb * self.mb
        if var > 1e-9 * self.mbb:                       # batch sizes differ enough for a slope
            c = (self.mbs - self.mb * self.ms) / var
            self.c = c if c > 0.0 else 0.0
        a = self.ms - self.c * self.mb
        self.a = a if a > 0.0 else 0.0

    # ---- model ------------------------------------------------------------------
    def rate(self):
        """Calls per microsecond (0 until two arrivals have been seen)."""
        return 1.0 / self.mean_gap if self.n_gaps > 0 and self.mean_gap > 0.0 else 0.0

    def target(self):
        """b*: the batch size at which the GPU just keeps up with the arrivals."""
        lam = self.rate()
        load = lam * self.c
        if load >= 1.0:
            return float(self.max_batch)
        t = lam * self.a / (1.0 - load)
        return min(max(t, 1.0), float(self.max_batch))

    # ---- decision -----------------------------------------------------------------
    def decide(self, now_us, gpu_idle=True):
        """Calls to fire now (the oldest ones), 0 = wait."""
        if not gpu_idle or not self.pending:
            return 0
        q = min(len(self.pending), self.max_batch)
        lam = self.rate()
        if lam <= 0.0:
            return q                                    # no rate known yet: nothing to wait for
        waited = float(now_us) - self.pending[0]
        left = self.max_wait - waited
        if left <= 0.0:
            return q
        missing = self.target() - float(q)
        if missing <= 0.0:
            return q
        if missing / lam > left:
            return q                                    # the target is out of reach before the deadline
        return 0

    def fired(self, n):
        for _ in range(n):
            self.pending.popleft()

    def next_deadline(self):
        """Time at which the oldest pending call has waited max_wait (inf if none)."""
        return self.pending[0] + self.max_wait if self.pending else math.inf

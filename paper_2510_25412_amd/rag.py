"""Retrieval-augmented-generation workload of the paper's section 5 as a driver of the library:
a population of identical LIPs, each answering one request about a topic whose document (3000
tokens in the paper, 100 documents) must be in its KV file before the answer is decoded.  The
LIP logic is the paper's prompt caching: the KV files of the `retain` most requested topics are
kept and forked for every later request of the topic (the paper keeps the caches of its 20 most
popular topics and drops the rest); other topics are prefilled from scratch and
their file is removed with the request.  Topic popularity is skewed by a Pareto index (smaller
index = a few topics get most requests).

Everything that touches K/V runs through the C ABI (kv_open / kv_fork / kv_remove, pred batches
on the GPU); the firing times of the batches come from the library's controller (section 4.4).
Time is virtual: requests arrive by a seeded Poisson process, and every fired batch advances the
clock by its measured wall time (host work + GPU, synchronised), so throughput and latency are
those of a server that does nothing but this path.  Only attention is computed (no weights on
this path): Q/K/V rows are slices of fixed seeded random arrays, and sampled tokens do not exist.
Host logic and argument marshalling only; none of the method's arithmetic.
"""
import math
import time
from collections import deque
from dataclasses import dataclass

import numpy as np

from . import binding, synth


@dataclass
class RagConfig:
    n_docs: int = 100
    doc_tokens: int = 3000
    answer_tokens: int = 32
    retain: int = 20
    pareto_index: float = 1.0
    rate_per_s: float = 2000.0          # request arrivals (Poisson)
    n_requests: int = 400
    prefill_chunk: int = 512            # a document enters its file in pred calls of this many tokens
    max_batch: int = 64
    max_wait_us: float = 300.0
    seed: int = 2025


def topic_probabilities(n_docs, pareto_index, rng):
    """Request probability of every topic: weights drawn from a Pareto distribution with the given
    index (heavy tail for a small index), normalised."""
    w = rng.pareto(pareto_index, size=n_docs) + 1.0
    return w / w.sum()


class _Lip:
    __slots__ = ("rid", "topic", "arrival", "fid", "to_prefill", "to_decode", "hit")


class RagDriver:
    """sess: a driver.HipSession whose pool, workspace (max_lips >= max_batch, max_tokens >=
    max_batch * prefill_chunk) are large enough.  trace=True records every file operation and batch
    (and keeps the outputs) so that the run can be replayed on the CPU model."""

    def __init__(self, sess, cfg, trace=False, timer=None):
        import torch
        self.torch = torch
        self.sess, self.cfg = sess, cfg
        self.timer = timer or binding.BatchTimer(cfg.max_batch, cfg.max_wait_us)
        s = sess.shape
        self.max_rows = cfg.max_batch * max(cfg.prefill_chunk, 1)
        st = np.random.SeedSequence(cfg.seed).spawn(4)
        self.rng = np.random.Generator(np.random.PCG64(st[0]))
        # fixed seeded rows; a batch with T new tokens uses rows [0, T) of each
        self.q_host = synth._normal(st[1], (self.max_rows, s.n_q_heads, s.head_dim), s.dtype)
        self.k_host = synth._normal(st[2], (self.max_rows, s.n_kv_heads, s.head_dim), s.dtype)
        self.v_host = synth._normal(st[3], (self.max_rows, s.n_kv_heads, s.head_dim), s.dtype)
        from .driver import to_device
        self.q, self.k, self.v = (to_device(a, sess.device) for a in (self.q_host, self.k_host, self.v_host))
        self.out = torch.empty((self.max_rows, s.n_q_heads, s.head_dim), dtype=torch.float32, device=sess.device)
        self.trace = [] if trace else None
        self.outputs = [] if trace else None
        self.next_fid = 0
        self.h = {}                      # file id -> handle

    # ---- file operations (recorded when tracing) ----------------------------------
    def _open(self):
        fid = self.next_fid
        self.next_fid += 1
        self.h[fid] = self.sess.ctx.kv_open(None)
        if self.trace is not None:
            self.trace.append(("open", fid))
        return fid

    def _fork(self, parent):
        fid = self.next_fid
        self.next_fid += 1
        self.h[fid] = self.sess.ctx.kv_fork(self.h[parent])
        if self.trace is not None:
            self.trace.append(("fork", fid, parent))
        return fid

    def _remove(self, fid):
        self.sess.ctx.kv_remove(self.h.pop(fid))
        if self.trace is not None:
            self.trace.append(("remove", fid))

    # ---- the run -------------------------------------------------------------------
    def run(self):
        cfg, torch = self.cfg, self.torch
        probs = topic_probabilities(cfg.n_docs, cfg.pareto_index, self.rng)
        arrivals = np.cumsum(self.rng.exponential(1e6 / cfg.rate_per_s, size=cfg.n_requests))   # microseconds
        topics = self.rng.choice(cfg.n_docs, size=cfg.n_requests, p=probs)
        counts = np.zeros(cfg.n_docs, np.int64)
        cache = {}                       # topic -> file id of the retained document KV
        calls = deque()                  # pending pred calls: (lip, n_tokens), oldest first
        stream = self.sess.stream
        now, k = 0.0, 0
        done, lat, batches, busy = 0, [], [], 0.0
        hits = steps = prefilled = 0

        def submit(lip, t):
            n = min(cfg.prefill_chunk, lip.to_prefill) if lip.to_prefill > 0 else 1
            calls.append((lip, n))
            self.timer.arrive(t)

        def admit(t, rid):
            nonlocal hits
            lip = _Lip()
            lip.rid, lip.topic, lip.arrival = rid, int(topics[rid]), t
            counts[lip.topic] += 1
            lip.to_decode = cfg.answer_tokens
            if lip.topic in cache:       # prompt cache hit: share the document's pages
                lip.fid, lip.to_prefill, lip.hit = self._fork(cache[lip.topic]), 0, True
                hits += 1
            else:
                lip.fid, lip.to_prefill, lip.hit = self._open(), cfg.doc_tokens, False
            submit(lip, t)

        def retain_after_prefill(lip):
            """The document is in lip.fid: keep it if the topic is among the `retain` most requested."""
            if lip.topic in cache or cfg.retain <= 0:
                return
            if len(cache) >= cfg.retain:
                coldest = min(cache, key=lambda t: (counts[t], t))
                if counts[coldest] >= counts[lip.topic]:
                    return
                self._remove(cache.pop(coldest))
            cache[lip.topic] = lip.fid                    # the prefilled file becomes the cached one
            lip.fid = self._fork(lip.fid)                 # the request continues on a fork

        while done < cfg.n_requests:
            while k < cfg.n_requests and arrivals[k] <= now:
                admit(float(arrivals[k]), k)
                k += 1
            fire = self.timer.decide(now, True)
            if fire == 0:
                nxt = min(float(arrivals[k]) if k < cfg.n_requests else math.inf, self.timer.next_deadline())
                assert nxt < math.inf and nxt > now, "scheduler waits with nothing to wait for"
                now = nxt
                continue
            self.timer.fired(fire)
            batch = [calls.popleft() for _ in range(fire)]
            kv = [self.h[lip.fid] for lip, _ in batch]
            nt = [n for _, n in batch]
            T = sum(nt)
            t0 = time.perf_counter()
            self.sess.ctx.pred_batch(kv, nt, self.q, self.k, self.v, self.out, stream)
            torch.cuda.current_stream(self.sess.device).synchronize()
            dt = (time.perf_counter() - t0) * 1e6
            if self.trace is not None:
                self.trace.append(("pred", [lip.fid for lip, _ in batch], nt))
                self.outputs.append(self.out[:T].cpu().numpy().copy())
            now += dt
            busy += dt
            self.timer.done(fire, dt)
            batches.append(fire)
            steps += fire
            for lip, n in batch:
                if lip.to_prefill > 0:
                    lip.to_prefill -= n
                    prefilled += n
                    if lip.to_prefill == 0:
                        retain_after_prefill(lip)
                else:
                    lip.to_decode -= 1
                if lip.to_prefill == 0 and lip.to_decode == 0:
                    self._remove(lip.fid)
                    lat.append(now - lip.arrival)
                    done += 1
                else:
                    submit(lip, now)
        self.cache = cache
        lat = np.array(lat)
        return dict(requests=done, seconds=now / 1e6, requests_per_s=done / (now / 1e6), lip_steps_per_s=steps / (now / 1e6),
                    pred_calls=steps, batches=len(batches), mean_batch=float(np.mean(batches)), hit_rate=hits / max(done, 1),
                    latency_ms_mean=float(lat.mean() / 1e3), latency_ms_p50=float(np.percentile(lat, 50) / 1e3),
                    latency_ms_p95=float(np.percentile(lat, 95) / 1e3), gpu_busy_frac=busy / now, tokens_prefilled=prefilled,
                    cached_topics=len(cache), scheduler=self.timer.state())

    def close(self):
        for fid in list(self.h):
            self.sess.ctx.kv_remove(self.h.pop(fid))
        self.timer.close()

"""Seeded synthetic LIP workloads (input generation only; none of the method's arithmetic).

Each workload is a short program over the KV file API of the paper's Fig. 1 (open, fork,
append) that builds the KV files, followed by ONE batch of pending `pred` calls.  The same
workload object drives the CPU oracle and the HIP library, so both start from identical
bit patterns.  Floating-point values are N(0,1) float32 samples; for bf16 storage they are
rounded once, round-to-nearest-even, to 16-bit patterns (dtype uint16) which widen exactly
to float32.

Random streams: numpy PCG64 seeded with `1000 + config number`.  Lengths come from the
root stream first; every data array comes from its own child stream (spawned in a fixed
order), so arrays may be generated lazily, in parallel, or skipped without changing any
other array.
"""
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

F32, BF16 = "f32", "bf16"


def bf16_round(x):
    """float32 array -> uint16 bf16 patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    return ((u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)).astype(np.uint16)


def to_f32(a):
    """Stored patterns (uint16 bf16 or float32) -> the float32 values they denote."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return a.astype(np.float32, copy=False)


@dataclass
class Shape:
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_tokens: int
    dtype: str          # F32 or BF16 : storage type of Q, K, V

    @property
    def kv_bytes_per_token(self):
        return 2 * self.n_kv_heads * self.head_dim * (4 if self.dtype == F32 else 2)


class _Streams:
    """Child generators handed out in call order; stream k is independent of the others."""

    def __init__(self, seed):
        self.ss = np.random.SeedSequence(seed)
        self.root = np.random.Generator(np.random.PCG64(self.ss.spawn(1)[0]))

    def child(self):
        return self.ss.spawn(1)[0]


def _normal(seed_seq, shape, dtype):
    g = np.random.Generator(np.random.PCG64(seed_seq))
    x = g.standard_normal(shape, dtype=np.float32)
    return bf16_round(x) if dtype == BF16 else x


@dataclass
class Workload:
    name: str
    shape: Shape
    n_pages: int
    free_order: Optional[np.ndarray]           # permutation of page ids (allocation ranking) or None
    # setup program: list of ("open", fid) | ("fork", fid, parent_fid) | ("append", fid, n, kseed, vseed)
    program: list = field(default_factory=list)
    # the batch of pred calls: file ids, new tokens per LIP, seeds of q / k_new / v_new
    batch_files: list = field(default_factory=list)
    batch_n: list = field(default_factory=list)
    batch_seeds: tuple = ()
    lengths: dict = field(default_factory=dict)  # fid -> tokens in the file before the batch

    def kv_rows(self, n, seed):
        s = self.shape
        return _normal(seed, (n, s.n_kv_heads, s.head_dim), s.dtype)

    def setup_ops(self):
        """Yields ("open", fid) / ("fork", fid, parent) / ("append", fid, K, V) with K, V
        [n, Hkv, D] stored patterns, generated on demand."""
        for op in self.program:
            if op[0] == "append":
                _, fid, n, ks, vs = op
                yield ("append", fid, self.kv_rows(n, ks), self.kv_rows(n, vs))
            else:
                yield op

    def batch(self):
        s = self.shape
        T = int(sum(self.batch_n))
        qs, ks, vs = self.batch_seeds
        return dict(files=list(self.batch_files), n_tokens=list(self.batch_n),
                    q=_normal(qs, (T, s.n_q_heads, s.head_dim), s.dtype),
                    k_new=_normal(ks, (T, s.n_kv_heads, s.head_dim), s.dtype),
                    v_new=_normal(vs, (T, s.n_kv_heads, s.head_dim), s.dtype))

    # ---- bookkeeping used by bench / tests (pure counting) ----
    def pages_after_batch(self):
        P = self.shape.page_tokens
        return {f: -(-(self.lengths[f] + n) // P) for f, n in zip(self.batch_files, self.batch_n)}


def _finish(wl, st):
    wl.batch_seeds = (st.child(), st.child(), st.child())
    return wl


def _plain_files(wl, st, lengths, first_fid=0):
    for i, L in enumerate(lengths):
        fid = first_fid + i
        wl.program.append(("open", fid))
        if L > 0:
            wl.program.append(("append", fid, int(L), st.child(), st.child()))
        wl.lengths[fid] = int(L)


def config1():
    """Tiny fp32 case: 4 LIPs, 8 Q = 8 KV heads, D 64, page 16, lengths 37/80/129/200."""
    st = _Streams(1001)
    wl = Workload("tiny_fp32", Shape(8, 8, 64, 16, F32), 64, None)
    lengths = [37, 80, 129, 200]
    _plain_files(wl, st, lengths)
    wl.batch_files = [0, 1, 2, 3]
    wl.batch_n = [1, 1, 1, 1]
    return _finish(wl, st)


def config2(n_lips=64, lo=512, hi=4096, slack_pages=2048, n_new=1, n_q_heads=32):
    """Decode batch: 64 LIPs, 32 Q / 8 KV heads, D 128, bf16, lengths U{512..4096}; n_new tokens
    per LIP and call (1 = plain decode; 2..8 = a draft being verified, paper section 4.1).
    n_q_heads = 64: the same batch with 8 query heads per kv head."""
    st = _Streams(1002)
    lengths = st.root.integers(lo, hi + 1, size=n_lips)
    P = 16
    n_pages = int(sum(-(-(int(L) + n_new) // P) for L in lengths)) + slack_pages
    wl = Workload("decode_batch" if n_new == 1 else f"draft{n_new}_batch", Shape(n_q_heads, 8, 128, P, BF16), n_pages, None)
    _plain_files(wl, st, lengths)
    wl.batch_files = list(range(n_lips))
    wl.batch_n = [int(n_new)] * n_lips
    return _finish(wl, st)


def config3(n_roots=16, n_children=16, prefix=2048, suffix_hi=256, slack_pages=1024):
    """Fork-heavy tree search: roots with a shared prefix, each forked into children that
    then append a private suffix of U{1..suffix_hi} tokens; one decode token per child."""
    st = _Streams(1003)
    suffix = st.root.integers(1, suffix_hi + 1, size=n_roots * n_children)
    P = 16
    n_pages = n_roots * (-(-prefix // P)) + int(sum(-(-(prefix % P + int(s) + 1) // P) + 1 for s in suffix)) + slack_pages
    wl = Workload("fork_tree", Shape(32, 8, 128, P, BF16), n_pages, None)
    fid = 0
    children = []
    for r in range(n_roots):
        root = fid
        fid += 1
        wl.program.append(("open", root))
        wl.program.append(("append", root, prefix, st.child(), st.child()))
        wl.lengths[root] = prefix
        for c in range(n_children):
            wl.program.append(("fork", fid, root))
            s = int(suffix[r * n_children + c])
            wl.program.append(("append", fid, s, st.child(), st.child()))
            wl.lengths[fid] = prefix + s
            children.append(fid)
            fid += 1
    wl.batch_files = children
    wl.batch_n = [1] * len(children)
    return _finish(wl, st)


def config4(n_prefill=32, chunk=512, pre_hi=8192, n_decode=224, dec_lo=1024, dec_hi=4096, slack_pages=1024):
    """Mixed batch: prefill chunks (causal inside the chunk) on files of U{0..pre_hi} tokens
    plus decode LIPs at U{dec_lo..dec_hi} tokens."""
    st = _Streams(1004)
    pre = st.root.integers(0, pre_hi + 1, size=n_prefill)
    dec = st.root.integers(dec_lo, dec_hi + 1, size=n_decode)
    P = 16
    n_pages = int(sum(-(-(int(L) + chunk) // P) for L in pre) + sum(-(-(int(L) + 1) // P) for L in dec)) + slack_pages
    wl = Workload("mixed_prefill_decode", Shape(32, 8, 128, P, BF16), n_pages, None)
    _plain_files(wl, st, list(pre) + list(dec))
    wl.batch_files = list(range(n_prefill + n_decode))
    wl.batch_n = [chunk] * n_prefill + [1] * n_decode
    return _finish(wl, st)


def config5(n_lips=16, lo=32768, hi=131072, n_pages=3_000_000):
    """Long context: 16 LIPs at U{32768..131072} tokens, 64 Q / 8 KV heads, pages scattered
    over a large pool by a seeded random allocation ranking."""
    st = _Streams(1005)
    lengths = st.root.integers(lo, hi + 1, size=n_lips)
    P = 16
    need = int(sum(-(-(int(L) + 1) // P) for L in lengths))
    n_pages = max(int(n_pages), need + 64)
    free_order = st.root.permutation(n_pages).astype(np.int32)
    wl = Workload("long_context", Shape(64, 8, 128, P, BF16), n_pages, free_order)
    _plain_files(wl, st, lengths)
    wl.batch_files = list(range(n_lips))
    wl.batch_n = [1] * n_lips
    return _finish(wl, st)


def custom(name, shape, files, batch, n_pages, seed, free_order=None, then=()):
    """Free-form workload for edge cases.  files: list of ("new", length),
    ("fork", parent_index, extra_tokens), ("extract", source_index, token indices) or
    ("merge", [source indices]); batch: list of (file_index, n_tokens); then: operations that
    follow the files, ("offload", [file indices]), ("restore", [file indices]), ("append",
    file_index, n_tokens) or ("remove", file_index)."""
    st = _Streams(seed)
    wl = Workload(name, shape, n_pages, free_order)
    for fid, spec in enumerate(files):
        if spec[0] == "new":
            wl.program.append(("open", fid))
            if spec[1] > 0:
                wl.program.append(("append", fid, int(spec[1]), st.child(), st.child()))
            wl.lengths[fid] = int(spec[1])
        elif spec[0] == "extract":
            idx = [int(i) for i in spec[2]]
            wl.program.append(("extract", fid, spec[1], idx))
            wl.lengths[fid] = len(idx)
        elif spec[0] == "merge":
            wl.program.append(("merge", fid, list(spec[1])))
            wl.lengths[fid] = sum(wl.lengths[p] for p in spec[1])
        else:
            _, parent, extra = spec
            wl.program.append(("fork", fid, parent))
            if extra > 0:
                wl.program.append(("append", fid, int(extra), st.child(), st.child()))
            wl.lengths[fid] = wl.lengths[parent] + int(extra)
    for op in then:
        if op[0] == "append":
            wl.program.append(("append", op[1], int(op[2]), st.child(), st.child()))
            wl.lengths[op[1]] += int(op[2])
        else:
            wl.program.append((op[0], list(op[1]) if op[0] in ("offload", "restore") else op[1]))
    # a parent that is appended to after a fork changes length: lengths[] holds the value at
    # the time the file was created; callers that append to parents later track it themselves
    wl.batch_files = [f for f, _ in batch]
    wl.batch_n = [int(n) for _, n in batch]
    return _finish(wl, st)


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}

"""Pins for the oracle's file-system state model (CPU only)."""
import numpy as np
import pytest

from oracle.kvfs_model import KVFSModel, KVError, ENOSPC, EBADF, EBUSY, EINVAL
from trace_util import load_trace, parse_expect


def test_fig1_hand_trace():
    """Hand-derived trace of the paper's Fig. 1 program (tests/golden)."""
    m = KVFSModel(8, 4)
    for op, args, exp in load_trace("fig1_state_trace.txt"):
        e = parse_expect(exp)
        if op == "open":
            assert m.kv_open(args[0]) == e["h"]
        elif op == "fork":
            assert m.kv_fork(int(args[0])) == e["h"]
        elif op == "append":
            h, n = int(args[0]), int(args[1])
            cow, slots = m.append([(h, n)])
            assert cow == e["cow"] and slots[0] == e["slots"]
            assert m.kv_pages(h) == e["pages"]
        elif op == "remove":
            m.kv_remove(int(args[0]))
        elif op == "close":
            m.kv_close(int(args[0]))
        elif op == "len":
            assert m.kv_len(int(args[0])) == e["len"]
        if "rc" in e:
            assert m.refcount.tolist() == e["rc"], (op, args)
        if "free" in e:
            assert m.free_pages() == e["free"], (op, args)
        m.audit()


def test_fork_allocates_nothing_and_remove_restores():
    m = KVFSModel(64, 16)
    h = m.kv_open()
    m.append([(h, 100)])
    before = (m.refcount.copy(), m.free_pages(), m.kv_pages(h))
    c = m.kv_fork(h)
    assert m.free_pages() == before[1] and m.kv_pages(c) == before[2] and m.kv_len(c) == 100
    m.append([(c, 40)])                       # unaligned: 100 % 16 = 4 -> one copied page
    assert m.cow_copies == 1 and m.kv_pages(h) == before[2]
    assert m.kv_pages(c)[:6] == before[2][:6] and m.kv_pages(c)[6] != before[2][6]
    m.kv_remove(c)
    assert np.array_equal(m.refcount, before[0]) and m.free_pages() == before[1]
    m.audit()


def test_aligned_fork_never_copies():
    m = KVFSModel(64, 16)
    h = m.kv_open()
    m.append([(h, 32)])
    kids = [m.kv_fork(h) for _ in range(4)]
    m.append([(k, 5) for k in kids])
    assert m.cow_copies == 0
    assert all(m.refcount[p] == 5 for p in m.kv_pages(h))
    m.audit()


def test_two_sharers_in_one_batch_order_defined():
    """Two files sharing a partly filled page, both appended in one batch: the first copies,
    the second is then sole owner and writes in place."""
    m = KVFSModel(16, 4)
    a = m.kv_open()
    m.append([(a, 6)])
    b = m.kv_fork(a)
    assert m.pages_needed([(a, 1), (b, 1)]) == 1
    cow, slots = m.append([(a, 1), (b, 1)])
    assert cow == [(1, 2, 2)] and slots == [[(2, 2)], [(1, 2)]]
    m.audit()


def test_enospc_changes_nothing_and_errors():
    m = KVFSModel(4, 4)
    a = m.kv_open()
    m.append([(a, 9)])                                   # 3 pages
    b = m.kv_fork(a)
    snap = (m.refcount.copy(), m.kv_pages(a), m.kv_pages(b), m.free_pages())
    with pytest.raises(KVError) as e:
        m.append([(a, 1), (b, 4)])                       # needs copy + 1 new page > 1 free
    assert e.value.code == ENOSPC
    assert np.array_equal(m.refcount, snap[0]) and m.kv_pages(a) == snap[1] and m.kv_pages(b) == snap[2]
    assert m.free_pages() == snap[3] and m.kv_len(a) == 9 and m.kv_len(b) == 9
    with pytest.raises(KVError) as e:
        m.append([(a, 1), (a, 1)])
    assert e.value.code == EBUSY
    with pytest.raises(KVError) as e:
        m.append([(a, 0)])
    assert e.value.code == EINVAL
    with pytest.raises(KVError) as e:
        m.kv_len(77)
    assert e.value.code == EBADF
    m.kv_remove(b)
    with pytest.raises(KVError):
        m.kv_fork(b)
    m.audit()


def test_lowest_rank_allocation_and_handle_reuse():
    order = np.array([5, 2, 7, 0, 1, 3, 4, 6])
    m = KVFSModel(8, 2, order)
    a = m.kv_open()
    m.append([(a, 6)])
    assert m.kv_pages(a) == [5, 2, 7]
    b = m.kv_open()
    m.append([(b, 2)])
    assert m.kv_pages(b) == [0]
    m.kv_remove(a)                                         # frees 5, 2, 7 in that order
    c = m.kv_open()
    assert c == a                                          # lowest free handle slot
    m.append([(c, 4)])
    assert m.kv_pages(c) == [5, 2]                         # rank order, not release order
    m.audit()


def test_random_ops_keep_invariants():
    rng = np.random.default_rng(7)
    m = KVFSModel(256, 8, rng.permutation(256))
    live = []
    for step in range(600):
        r = rng.random()
        try:
            if r < 0.15 or not live:
                live.append(m.kv_open())
            elif r < 0.35:
                live.append(m.kv_fork(live[rng.integers(len(live))]))
            elif r < 0.85:
                k = min(len(live), int(rng.integers(1, 4)))
                hs = rng.choice(live, size=k, replace=False)
                m.append([(int(h), int(rng.integers(1, 20))) for h in hs])
            else:
                m.kv_remove(live.pop(rng.integers(len(live))))
        except KVError as e:
            assert e.code == ENOSPC
            m.kv_remove(live.pop(rng.integers(len(live))))
        if step % 25 == 0:
            m.audit()
    for h in live:
        m.kv_remove(h)
    assert m.free_pages() == 256 and int(m.refcount.sum()) == 0


def test_truncate_frees_pages_and_keeps_sharing():
    m = KVFSModel(16, 4)
    a = m.kv_open()
    m.append([(a, 10)])                       # pages 0,1,2
    b = m.kv_fork(a)
    m.append([(b, 5)])                        # copy of page 2 -> 3, then page 4
    assert m.kv_pages(b) == [0, 1, 3, 4] and m.kv_len(b) == 15
    m.kv_truncate(b, 10)                      # drafts rejected: back to the fork point
    assert m.kv_pages(b) == [0, 1, 3] and m.free_pages() == 12 and m.kv_len(b) == 10
    m.kv_truncate(b, 8)                       # exactly two pages
    assert m.kv_pages(b) == [0, 1] and m.refcount.tolist()[:5] == [2, 2, 1, 0, 0]
    m.kv_truncate(b, 6)                       # into a shared page: stays shared...
    cow, slots = m.append([(b, 1)])           # ...until the next append copies it
    assert cow == [(1, 3, 2)] and slots == [[(3, 2)]]
    with pytest.raises(KVError):
        m.kv_truncate(b, 99)
    m.kv_truncate(a, 0)
    assert m.kv_pages(a) == [] and m.kv_len(a) == 0
    m.audit()

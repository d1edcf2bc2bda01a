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


def test_names_handles_and_what_close_and_remove_free():
    """Section 4.2: a file can be shared across LIPs by name; remove deletes it; close gives up a
    handle.  This build's reading: a second open of a name is a second handle to the SAME file; a named
    file outlives its handles; an anonymous file goes with its last handle; remove takes the name along."""
    m = KVFSModel(8, 4)
    h0 = m.kv_open("doc")
    m.append([(h0, 5)])
    h1 = m.kv_open("doc")
    assert h1 != h0 and m.kv_pages(h1) == m.kv_pages(h0) == [0, 1] and m.kv_len(h1) == 5
    assert m.refcount.tolist()[:2] == [1, 1]                       # one file, not a fork
    m.append([(h1, 1)])
    assert m.kv_len(h0) == 6                                       # written through one handle, seen through the other
    m.kv_close(h0)
    assert m.free_pages() == 6 and m.kv_len(h1) == 6              # still there
    with pytest.raises(KVError) as e:
        m.kv_len(h0)
    assert e.value.code == EBADF
    m.kv_close(h1)
    assert m.free_pages() == 6                                     # a named file outlives its handles
    h2 = m.kv_open("doc")
    assert m.kv_len(h2) == 6 and m.kv_pages(h2) == [0, 1]
    m.kv_remove(h2)
    assert m.free_pages() == 8
    h3 = m.kv_open("doc")                                          # the name went with the file: a new, empty one
    assert m.kv_len(h3) == 0 and m.kv_pages(h3) == []
    # anonymous: gone with its last handle, pages and all
    x = m.kv_open()
    m.append([(x, 9)])
    y = m.kv_fork(x)
    assert m.free_pages() == 5
    m.kv_close(x)
    assert m.free_pages() == 5 and m.kv_len(y) == 9               # the fork still holds every page
    m.kv_close(y)
    assert m.free_pages() == 8 and not m.refcount.any()
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


# ---- extract / merge (section 4.2) ---------------------------------------------------------

def test_extract_merge_hand_trace():
    """Worked by hand, page size 4.  A destination page that is slots 0, 1, 2, ... of one existing
    page is referenced; anything else is a fresh page filled token by token."""
    m = KVFSModel(16, 4)
    a = m.kv_open()
    m.append([(a, 10)])                                   # pages 0,1,2 (slots: 4,4,2)
    # tokens 0..3 = page 0 in order -> shared; (8, 9, 4) = page 2 slot 0, page 2 slot 1, page 1 slot 0 -> copied
    b, moves = m.kv_extract(a, [0, 1, 2, 3, 8, 9, 4])
    assert m.kv_pages(b) == [0, 3] and m.kv_len(b) == 7
    assert moves == [(2, 0, 3, 0), (2, 1, 3, 1), (1, 0, 3, 2)]
    assert m.refcount.tolist()[:5] == [2, 1, 1, 1, 0]
    # a partly filled destination page can be shared too: tokens 8, 9 = slots 0, 1 of page 2
    c, moves = m.kv_extract(a, [8, 9])
    assert m.kv_pages(c) == [2] and moves == [] and m.refcount.tolist()[:5] == [2, 1, 2, 1, 0]
    # ...and the next append to it copies the shared page first, as after an unaligned fork
    cow, slots = m.append([(c, 1)])
    assert cow == [(2, 4, 2)] and slots == [[(4, 2)]] and m.kv_pages(c) == [4]
    # slots in the wrong order, or starting past slot 0, are copies
    d, moves = m.kv_extract(a, [1, 0, 5, 6])
    assert m.kv_pages(d) == [5] and moves == [(0, 1, 5, 0), (0, 0, 5, 1), (1, 1, 5, 2), (1, 2, 5, 3)]
    # merge: a's aligned pages are referenced; the page where a ends and b starts is assembled
    e, moves = m.kv_merge([a, b])                         # 10 + 7 tokens
    assert m.kv_len(e) == 17 and m.kv_pages(e) == [0, 1, 6, 7, 8]
    assert moves[:4] == [(2, 0, 6, 0), (2, 1, 6, 1), (0, 0, 6, 2), (0, 1, 6, 3)]       # a8 a9 b0 b1
    assert moves[4:8] == [(0, 2, 7, 0), (0, 3, 7, 1), (3, 0, 7, 2), (3, 1, 7, 3)]      # b2 b3 b4 b5
    assert moves[8:] == [(3, 2, 8, 0)]                                                 # b6
    # empty results
    z, moves = m.kv_extract(a, [])
    assert m.kv_len(z) == 0 and m.kv_pages(z) == [] and moves == []
    m.audit()


def test_identity_extract_and_single_merge_equal_fork():
    m = KVFSModel(64, 16)
    a = m.kv_open()
    m.append([(a, 100)])
    f = m.kv_fork(a)
    x, mv1 = m.kv_extract(a, range(100))
    y, mv2 = m.kv_merge([a])
    assert m.kv_pages(x) == m.kv_pages(y) == m.kv_pages(f) == m.kv_pages(a) and mv1 == mv2 == []
    assert m.kv_len(x) == m.kv_len(y) == 100 and set(m.refcount[m.kv_pages(a)]) == {4}
    # a prefix that ends inside a page: still no copy
    z, mv = m.kv_extract(a, range(37))
    assert m.kv_pages(z) == m.kv_pages(a)[:3] and mv == []
    m.audit()


def test_extract_errors_change_nothing():
    m = KVFSModel(8, 4)
    a = m.kv_open()
    m.append([(a, 22)])                                   # 6 pages, 2 free
    snap = (m.refcount.copy(), m.free_pages(), dict(m.handles))
    with pytest.raises(KVError) as e:
        m.kv_extract(a, [3, 2, 1, 0, 7, 6, 5, 4, 11, 10, 9, 8])    # three fresh pages, two free
    assert e.value.code == ENOSPC
    with pytest.raises(KVError) as e:
        m.kv_extract(a, [0, 22])
    assert e.value.code == EINVAL
    with pytest.raises(KVError) as e:
        m.kv_extract(a, [-1])
    assert e.value.code == EINVAL
    with pytest.raises(KVError) as e:
        m.kv_merge([a, 99])
    assert e.value.code == EBADF
    assert np.array_equal(snap[0], m.refcount) and snap[1] == m.free_pages() and snap[2] == m.handles
    b, _ = m.kv_extract(a, [3, 2, 1, 0, 7, 6, 5, 4])      # exactly the two free pages
    assert m.free_pages() == 0 and m.kv_pages(b) == [6, 7]
    m.audit()


def test_extract_of_no_tokens_still_needs_a_usable_source():
    """kv_extract with an empty index list makes an empty file, but only from a source that exists and
    does not wait: a stale handle is EBADF and a waiting file EBUSY like any other read of it (a waiting
    file refuses every call but remove and close, the reading of paper section 4.3 taken here), and
    neither creates a file or a handle."""
    m = KVFSModel(8, 4)
    a, b = m.kv_open(), m.kv_open()
    m.append([(a, 6), (b, 3)])
    e0, moves = m.kv_extract(a, [])
    assert m.kv_len(e0) == 0 and m.kv_pages(e0) == [] and moves == []
    m.kv_offload([b])
    gone = m.kv_open()
    m.kv_remove(gone)
    snap = (m.refcount.copy(), m.free_pages(), dict(m.handles), m.kv_pages(b))
    with pytest.raises(KVError) as e:
        m.kv_extract(b, [])
    assert e.value.code == EBUSY
    for bad in (gone, 99, -1):
        with pytest.raises(KVError) as e:
            m.kv_extract(bad, [])
        assert e.value.code == EBADF
    assert np.array_equal(snap[0], m.refcount) and snap[1:] == (m.free_pages(), m.handles, m.kv_pages(b))
    m.audit()


def test_random_ops_with_extract_merge_against_token_lists():
    """Every file is shadowed by a plain Python list of unique token ids; each token's K row holds its
    id.  After any mix of append / fork / extract / merge / truncate / remove, reading a file
    through its pages must give exactly the shadow list: a wrong page decision, a missing copy or
    a copy into a page someone else still reads shows up as a wrong id."""
    from oracle.kvfs_model import PagePool
    from oracle.attention import gather_file
    rng = np.random.default_rng(11)
    P = 4
    m = KVFSModel(512, P, rng.permutation(512))
    pool = PagePool(1, P, 1, np.float64)
    shadow = {}
    next_id = [1]

    def append(h, n):
        ids = np.arange(next_id[0], next_id[0] + n, dtype=np.float64).reshape(n, 1, 1)
        cow, slots = m.append([(h, n)])
        pool.apply(cow, slots, ids, -ids)
        shadow[h] += [int(i) for i in ids.ravel()]
        next_id[0] += n

    for step in range(700):
        r = rng.random()
        live = list(shadow)
        try:
            if r < 0.1 or not live:
                shadow[m.kv_open()] = []
            elif r < 0.4:
                append(live[rng.integers(len(live))], int(rng.integers(1, 12)))
            elif r < 0.5:
                src = live[rng.integers(len(live))]
                shadow[m.kv_fork(src)] = list(shadow[src])
            elif r < 0.7:
                src = live[rng.integers(len(live))]
                L = len(shadow[src])
                kind = rng.integers(4)
                if kind == 0:
                    idx = rng.integers(0, max(L, 1), size=int(rng.integers(0, 20))) if L else []
                elif kind == 1:
                    idx = np.flatnonzero(rng.random(L) < 0.7)                     # pruning: keep a subset, in order
                elif kind == 2:
                    idx = np.r_[np.arange(min(L, 5)), np.arange(max(L - 9, min(L, 5)), L)]   # first tokens + recent window
                else:
                    idx = np.arange(L)[:int(rng.integers(0, L + 1))]
                h, moves = m.kv_extract(src, [int(i) for i in idx])
                pool.move_tokens(moves)
                shadow[h] = [shadow[src][int(i)] for i in idx]
            elif r < 0.8:
                srcs = [live[i] for i in rng.integers(len(live), size=int(rng.integers(1, 4)))]
                h, moves = m.kv_merge(srcs)
                pool.move_tokens(moves)
                shadow[h] = [t for s in srcs for t in shadow[s]]
            elif r < 0.9:
                h = live[rng.integers(len(live))]
                n = int(rng.integers(0, len(shadow[h]) + 1))
                m.kv_truncate(h, n)
                del shadow[h][n:]
            else:
                h = live[rng.integers(len(live))]
                m.kv_remove(h)
                del shadow[h]
        except KVError as e:
            assert e.code == ENOSPC
            h = max(shadow, key=lambda x: len(shadow[x]))
            m.kv_remove(h)
            del shadow[h]
        if step % 20 == 0:
            m.audit()
            for h, toks in shadow.items():
                K, V = gather_file(pool, m.kv_pages(h), len(toks))
                assert K.ravel().tolist() == toks and V.ravel().tolist() == [-t for t in toks], (step, h)
    for h in list(shadow):
        m.kv_remove(h)
    assert m.free_pages() == 512


# ---- offload / restore (section 4.3) ---------------------------------------------------------

def test_offload_restore_hand_trace():
    """Worked by hand, page size 4: a page leaves when all its readers wait, comes back for all of
    them when one of them is restored."""
    m = KVFSModel(16, 4)
    a = m.kv_open()
    m.append([(a, 10)])                                   # a: pages 0,1,2
    b = m.kv_fork(a)
    m.append([(b, 3)])                                    # b: 0,1,3,4 (page 2 copied into 3)
    assert m.kv_pages(b) == [0, 1, 3, 4]
    assert m.kv_offload([a]) == [(2, 0)]                  # pages 0, 1 are still read by b; page 2 leaves
    assert m.kv_pages(a) == [0, 1, -1] and m.refcount.tolist()[:5] == [2, 2, 0, 1, 1] and m.free_pages() == 12
    with pytest.raises(KVError) as e:
        m.append([(b, 1), (a, 1)])                        # a waits: the whole batch is refused
    assert e.value.code == EBUSY and m.kv_len(b) == 13
    with pytest.raises(KVError) as e:
        m.kv_fork(a)
    assert e.value.code == EBUSY
    assert m.kv_offload([b]) == [(0, 1), (1, 2), (3, 3), (4, 4)]
    assert m.kv_pages(a) == [-2, -3, -1] and m.kv_pages(b) == [-2, -3, -4, -5] and m.free_pages() == 16
    m.audit()
    # b comes back: fresh pages lowest first; a's entries for the shared pages follow
    assert m.kv_restore([b]) == [(1, 0), (2, 1), (3, 2), (4, 3)]
    assert m.kv_pages(b) == [0, 1, 2, 3] and m.kv_pages(a) == [0, 1, -1]
    assert m.refcount.tolist()[:5] == [2, 2, 1, 1, 0]
    m.audit()
    cow, slots = m.append([(b, 1)])                       # b works again; page 3 (one token) is its own
    assert cow == [] and slots == [[(3, 1)]]
    assert m.kv_restore([a]) == [(0, 4)]
    assert m.kv_pages(a) == [0, 1, 4] and not m.is_waiting(a)
    with pytest.raises(KVError) as e:
        m.kv_restore([a])
    assert e.value.code == EBUSY
    # a waiting file can be removed: its host slots are released
    m.kv_offload([a])
    assert m.kv_pages(a) == [0, 1, -1]                    # slot 0 again (lowest free)
    m.kv_remove(a)
    assert m.host_refs == {} and m.refcount.tolist()[:5] == [1, 1, 1, 1, 0]
    m.audit()


def test_restore_needs_room_or_changes_nothing():
    m = KVFSModel(6, 4)
    a, b = m.kv_open(), m.kv_open()
    m.append([(a, 12)])
    m.kv_offload([a])
    m.append([(b, 16)])                                   # takes 4 of the 6 pages
    snap = (m.refcount.copy(), m.free_pages(), m.kv_pages(a), dict(m.host_refs))
    with pytest.raises(KVError) as e:
        m.kv_restore([a])                                 # three pages needed, two free
    assert e.value.code == ENOSPC and m.is_waiting(a)
    assert np.array_equal(snap[0], m.refcount) and snap[1:] == (m.free_pages(), m.kv_pages(a), m.host_refs)
    m.kv_truncate(b, 9)
    assert m.kv_restore([a]) == [(0, 3), (1, 4), (2, 5)]
    m.audit()


def test_random_ops_with_offload_against_token_lists():
    """The token-list shadow model again, now with files that wait on the host in between: whatever
    the interleaving of offload / restore with appends, forks, extracts and removals of the other
    files, every file that does not wait reads back exactly its tokens, and so does every waiting
    file once it is restored."""
    from oracle.kvfs_model import PagePool
    from oracle.attention import gather_file
    rng = np.random.default_rng(13)
    P = 4
    m = KVFSModel(256, P, rng.permutation(256))
    pool = PagePool(1, P, 1, np.float64)
    shadow, next_id = {}, [1]

    def check(h):
        toks = shadow[h]
        K, V = gather_file(pool, m.kv_pages(h), len(toks))
        assert K.ravel().tolist() == toks and V.ravel().tolist() == [-t for t in toks], h

    for step in range(900):
        r = rng.random()
        live = [h for h in shadow if not m.is_waiting(h)]
        waiting = [h for h in shadow if m.is_waiting(h)]
        try:
            if r < 0.1 or not shadow:
                shadow[m.kv_open()] = []
            elif r < 0.4 and live:
                h = live[rng.integers(len(live))]
                n = int(rng.integers(1, 12))
                ids = np.arange(next_id[0], next_id[0] + n, dtype=np.float64).reshape(n, 1, 1)
                cow, slots = m.append([(h, n)])
                pool.apply(cow, slots, ids, -ids)
                shadow[h] += [int(i) for i in ids.ravel()]
                next_id[0] += n
            elif r < 0.5 and live:
                src = live[rng.integers(len(live))]
                shadow[m.kv_fork(src)] = list(shadow[src])
            elif r < 0.58 and live:
                src = live[rng.integers(len(live))]
                idx = np.flatnonzero(rng.random(len(shadow[src])) < 0.7)
                h, moves = m.kv_extract(src, [int(i) for i in idx])
                pool.move_tokens(moves)
                shadow[h] = [shadow[src][int(i)] for i in idx]
            elif r < 0.72 and live:
                k = int(rng.integers(1, min(4, len(live)) + 1))
                hs = [int(x) for x in rng.choice(live, size=k, replace=False)]
                pool.swap_out(m.kv_offload(hs))
            elif r < 0.86 and waiting:
                k = int(rng.integers(1, min(3, len(waiting)) + 1))
                hs = [int(x) for x in rng.choice(waiting, size=k, replace=False)]
                pool.swap_in(m.kv_restore(hs))
                for h in hs:
                    check(h)
            elif r < 0.92 and live:
                h = live[rng.integers(len(live))]
                n = int(rng.integers(0, len(shadow[h]) + 1))
                m.kv_truncate(h, n)
                del shadow[h][n:]
            elif shadow:
                h = list(shadow)[rng.integers(len(shadow))]        # waiting files can be removed too
                m.kv_remove(h)
                del shadow[h]
        except KVError as e:
            assert e.code == ENOSPC
            h = max(shadow, key=lambda x: len(shadow[x]))
            m.kv_remove(h)
            del shadow[h]
        if step % 15 == 0:
            m.audit()
            for h in shadow:
                if not m.is_waiting(h):
                    check(h)
    for h in sorted(shadow, key=m.is_waiting):             # the files that do not wait first: they make room
        if m.is_waiting(h):
            pool.swap_in(m.kv_restore([h]))
        check(h)
        m.kv_remove(h)
    assert m.free_pages() == 256 and m.host_refs == {} and m.waiters == {} and not getattr(pool, "host", {})


def test_extract_offload_hand_trace_file():
    """The hand-derived extract / merge / offload / restore trace under tests/golden (page size 4)."""
    m = KVFSModel(16, 4)
    for op, args, exp in load_trace("extract_offload_state_trace.txt"):
        e = parse_expect(exp)
        ints = lambda a: [] if a == "-" else [int(x) for x in a.split(",")]
        if op == "open":
            assert m.kv_open(None) == e["h"]
        elif op == "fork":
            assert m.kv_fork(int(args[0])) == e["h"]
        elif op == "append":
            h, n = int(args[0]), int(args[1])
            cow, slots = m.append([(h, n)])
            assert cow == e["cow"] and slots[0] == e["slots"] and m.kv_pages(h) == e["pages"]
        elif op == "extract":
            h, moves = m.kv_extract(int(args[0]), ints(args[1]))
            assert h == e["h"] and m.kv_pages(h) == e["pages"] and moves == e["moves"]
        elif op == "merge":
            h, moves = m.kv_merge(ints(args[0]))
            assert h == e["h"] and m.kv_pages(h) == e["pages"] and moves == e["moves"]
        elif op == "offload":
            assert m.kv_offload(ints(args[0])) == e["swaps"]
        elif op == "restore":
            assert m.kv_restore(ints(args[0])) == e["swaps"]
        elif op == "pages":
            assert m.kv_pages(int(args[0])) == e["pages"]
        elif op == "remove":
            m.kv_remove(int(args[0]))
        if "rc" in e:
            assert m.refcount.tolist()[:len(e["rc"])] == e["rc"], (op, args)
        if "free" in e:
            assert m.free_pages() == e["free"], (op, args)
        m.audit()

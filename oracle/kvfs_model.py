"""State model of the KV-cache file system (test infrastructure, CPU only).

The paper (section 4.2) says only that KV tensors live in fixed-size pages of GPU
memory, that files can be opened, forked without the tensors being duplicated,
removed and closed, and (section 4.1) that `pred` appends the new tokens' tensors to
the file.  Everything finer than that is a convention of this build, written out here
step by step so that the library's integer state can be compared bit for bit:

* allocation takes the free page of lowest rank (rank = position in `free_order`);
* `kv_fork` copies the page-id list and increments each page's reference count;
* appending to a file whose last page is partly filled and shared first copies that
  page's filled slots into a fresh page (copy-on-write); full pages are never copied;
* `kv_remove` decrements every page once and frees those reaching zero;
* a batch of appends either fits in the free pages or changes nothing;
* `kv_extract` / `kv_merge` (section 4.2: a new file from chosen token indices of a file / from
  the concatenation of files) build a new anonymous file token by token.  The stored K/V rows
  move unchanged.  A destination page whose tokens are slots 0, 1, 2, ... of ONE existing page,
  in that order, is not copied: the new file references that page (count + 1), like a fork;
  every other destination page is a fresh page (lowest rank first, in destination order) that
  receives copies of its tokens' rows.  Either the whole new file fits or nothing changes;
* `kv_offload` / `kv_restore` (section 4.3: the KV cache of a thread that waits for I/O moves to
  CPU memory and comes back when the wait ends).  A waiting file cannot be read or written
  (EBUSY) but can be removed.  A page leaves the GPU when EVERY reference to it belongs to a
  waiting file: it is copied to the lowest free host slot, every referencing table entry becomes
  -(slot + 1), and the page returns to the free set.  A page with a reference from a file that
  does not wait stays where it is.  Restoring a file brings each of its host slots back into a
  fresh page (lowest rank first, in table order) and rewrites EVERY entry that referenced the
  slot, also those of files that still wait: a page is on the host only while all its readers
  wait.  Either all files of a restore call fit or nothing changes.
"""
import heapq

import numpy as np

EINVAL, EBADF, ENOSPC, ENOENT, EEXIST, EBUSY = -1, -2, -3, -4, -5, -6


class KVError(Exception):
    def __init__(self, code, msg=""):
        super().__init__(f"{code}: {msg}")
        self.code = code


class _File:
    __slots__ = ("length", "pages", "name", "handles", "waiting")

    def __init__(self, name):
        self.length = 0
        self.pages = []                # page ids; -(slot + 1) for a page that is on the host
        self.name = name
        self.handles = set()
        self.waiting = False


class KVFSModel:
    def __init__(self, n_pages, page_tokens, free_order=None):
        self.n_pages = int(n_pages)
        self.P = int(page_tokens)
        order = np.arange(self.n_pages) if free_order is None else np.asarray(free_order)
        assert np.array_equal(np.sort(order), np.arange(self.n_pages)), "free_order must be a permutation"
        self.order = order.astype(np.int64)                    # rank -> page
        self.rank = np.empty(self.n_pages, np.int64)           # page -> rank
        self.rank[self.order] = np.arange(self.n_pages)
        self.free_ranks = list(range(self.n_pages))            # min-heap of the free pages' ranks
        self.refcount = np.zeros(self.n_pages, np.int64)
        self.handles = {}          # handle -> _File
        self.names = {}            # name -> _File
        self.cow_copies = 0
        self.waiters = {}          # resident page -> [(file, index)] entries of waiting files that reference it
        self.host_refs = {}        # host slot -> [(file, index)] entries that reference it
        self.free_slots = []       # min-heap of host slots freed so far
        self.n_slots = 0           # host slots ever created

    # ---- helpers -------------------------------------------------------------
    def _file(self, h, usable=False):
        f = self.handles.get(h)
        if f is None:
            raise KVError(EBADF, f"bad handle {h}")
        if usable and f.waiting:
            raise KVError(EBUSY, f"file of handle {h} is offloaded")
        return f

    def _new_handle(self, f):
        h = 0
        while h in self.handles:
            h += 1                                 # lowest free handle slot
        self.handles[h] = f
        f.handles.add(h)
        return h

    def _alloc(self):
        p = int(self.order[heapq.heappop(self.free_ranks)])   # lowest rank, whatever the release order
        self.refcount[p] = 1
        return p

    def _drop_ref(self, p):
        self.refcount[p] -= 1
        if self.refcount[p] == 0:
            heapq.heappush(self.free_ranks, int(self.rank[p]))

    def _release_pages(self, f, keep=0):
        """Drop the file's table entries from index `keep` on."""
        for i in range(keep, len(f.pages)):
            e = f.pages[i]
            if e >= 0:
                if f.waiting:
                    self.waiters[e].remove((f, i))
                    if not self.waiters[e]:
                        del self.waiters[e]
                self._drop_ref(e)
            else:                                          # on the host: the slot is free once nobody refers to it
                refs = self.host_refs[-e - 1]
                refs.remove((f, i))
                if not refs:
                    del self.host_refs[-e - 1]
                    heapq.heappush(self.free_slots, -e - 1)
        del f.pages[keep:]

    # ---- file API (names follow the paper's Fig. 1 and section 4.2) ------------
    def kv_open(self, name=None):
        if name is not None and name in self.names:
            return self._new_handle(self.names[name])     # second handle, same file
        f = _File(name)
        if name is not None:
            self.names[name] = f
        return self._new_handle(f)

    def kv_fork(self, h):
        parent = self._file(h, usable=True)
        f = _File(None)
        f.pages = list(parent.pages)
        f.length = parent.length
        for p in f.pages:
            self.refcount[p] += 1
        return self._new_handle(f)

    def kv_remove(self, h):
        f = self._file(h)
        self._release_pages(f)
        f.length = 0
        f.waiting = False
        for hh in list(f.handles):
            del self.handles[hh]
        f.handles.clear()
        if f.name is not None:
            del self.names[f.name]

    def kv_close(self, h):
        f = self._file(h)
        del self.handles[h]
        f.handles.discard(h)
        if f.name is None and not f.handles:
            self._release_pages(f)                        # anonymous file nobody can reach
            f.length = 0
            f.waiting = False

    def kv_len(self, h):
        return self._file(h).length

    def kv_truncate(self, h, new_len):
        """Drop the file's tokens from new_len on (POSIX-style ftruncate; a LIP that verifies
        draft tokens with a multi-token pred rolls the rejected ones back this way).  Pages no
        longer needed lose one reference; a shared last page stays shared until the next append
        copies it."""
        f = self._file(h, usable=True)
        if new_len < 0 or new_len > f.length:
            raise KVError(EINVAL, "truncate beyond the file")
        self._release_pages(f, keep=-(-new_len // self.P))
        f.length = new_len

    def kv_pages(self, h):
        return list(self._file(h).pages)

    def free_pages(self):
        return len(self.free_ranks)

    # ---- append planning -------------------------------------------------------
    def pages_needed(self, items):
        """Pages a batch of appends [(handle, n_tokens)] would allocate, LIPs taken in
        batch order (a copy made by an earlier LIP can leave a later one sole owner)."""
        pending = {}                                      # page -> refcount change so far
        need = 0
        for h, n in items:
            f = self._file(h, usable=True)
            L = f.length
            if L % self.P != 0:
                last = f.pages[-1]
                if self.refcount[last] + pending.get(last, 0) > 1:
                    need += 1
                    pending[last] = pending.get(last, 0) - 1
            need += -(-(L + n) // self.P) - (-(-L // self.P))
        return need

    def append(self, items):
        """Commit a batch of appends.  Returns (cow, slots): cow = [(src, dst, r)] page
        copies of slots [0, r); slots = per item, the (page, slot) of each new token."""
        files = []
        for h, n in items:
            if n < 1:
                raise KVError(EINVAL, "n_tokens must be >= 1")
            f = self._file(h, usable=True)
            if any(f is g for g in files):
                raise KVError(EBUSY, "same file twice in a batch")
            files.append(f)
        if self.pages_needed(items) > len(self.free_ranks):
            raise KVError(ENOSPC, "page pool exhausted")
        cow, slots = [], []
        for (h, n), f in zip(items, files):
            r = f.length % self.P
            if r != 0 and self.refcount[f.pages[-1]] > 1:
                src = f.pages[-1]
                dst = self._alloc()
                self.refcount[src] -= 1
                f.pages[-1] = dst
                cow.append((src, dst, r))
                self.cow_copies += 1
            mine = []
            for _ in range(n):
                if f.length % self.P == 0:
                    f.pages.append(self._alloc())
                mine.append((f.pages[-1], f.length % self.P))
                f.length += 1
            slots.append(mine)
        return cow, slots

    # ---- extract / merge (section 4.2) -------------------------------------------
    def kv_gather(self, refs):
        """New anonymous file whose token j is token i of the file behind handle h, for
        (h, i) = refs[j].  Returns (handle, moves), moves = [(src_page, src_slot, dst_page,
        dst_slot)] for every token that has to be copied (tokens of shared pages have none)."""
        P = self.P
        src = []                                          # (page, slot) of every destination token
        for h, i in refs:
            f = self._file(h, usable=True)
            if i < 0 or i >= f.length:
                raise KVError(EINVAL, f"token index {i} outside the file")
            src.append((f.pages[i // P], i % P))
        n = len(src)
        shared = []                                       # per destination page: the page it references, or None
        for d in range(-(-n // P)):
            toks = src[d * P:(d + 1) * P]
            same = all(pg == toks[0][0] and sl == k for k, (pg, sl) in enumerate(toks))
            shared.append(toks[0][0] if same else None)
        if sum(s is None for s in shared) > len(self.free_ranks):
            raise KVError(ENOSPC, "page pool exhausted")
        f = _File(None)
        moves = []
        for d, s in enumerate(shared):
            if s is not None:
                self.refcount[s] += 1
                f.pages.append(s)
            else:
                dst = self._alloc()
                f.pages.append(dst)
                for k, (pg, sl) in enumerate(src[d * P:(d + 1) * P]):
                    moves.append((pg, sl, dst, k))
        f.length = n
        return self._new_handle(f), moves

    def kv_extract(self, h, idx):
        """New file from the chosen token indices of file h, in the order given."""
        self._file(h, usable=True)                        # the source must exist and not wait, even for no tokens
        return self.kv_gather([(h, int(i)) for i in idx])

    def kv_merge(self, handles):
        """New file = the files' tokens one file after the other."""
        return self.kv_gather([(h, i) for h in handles for i in range(self._file(h, usable=True).length)])

    # ---- offload / restore (section 4.3) -------------------------------------------
    def _files_of(self, handles, waiting):
        files = []
        for h in handles:
            f = self._file(h)
            if f.waiting != waiting or any(f is g for g in files):
                raise KVError(EBUSY, "file already offloaded" if f.waiting else "file is not offloaded (or named twice)")
            files.append(f)
        return files

    def kv_offload(self, handles):
        """The files start to wait.  Returns the evictions [(page, host slot)] in the order they
        happen: the page's bytes must be copied to the slot before the page is reused."""
        out = []
        for f in self._files_of(handles, waiting=False):
            f.waiting = True
            for i, p in enumerate(f.pages):
                self.waiters.setdefault(p, []).append((f, i))
                if len(self.waiters[p]) == self.refcount[p]:       # every reader waits: the page leaves
                    if self.free_slots:
                        s = heapq.heappop(self.free_slots)
                    else:
                        s, self.n_slots = self.n_slots, self.n_slots + 1
                    refs = self.waiters.pop(p)
                    for g, j in refs:
                        g.pages[j] = -(s + 1)
                    self.host_refs[s] = refs
                    self.refcount[p] = 0
                    heapq.heappush(self.free_ranks, int(self.rank[p]))
                    out.append((p, s))
        return out

    def kv_restore(self, handles):
        """The files' waits end.  Returns the loads [(host slot, page)]: the slot's bytes go into
        the page.  Needs one free page per distinct host slot the files reference, else ENOSPC."""
        files = self._files_of(handles, waiting=True)
        need = {-e - 1 for f in files for e in f.pages if e < 0}
        if len(need) > len(self.free_ranks):
            raise KVError(ENOSPC, "page pool exhausted")
        out = []
        for f in files:
            f.waiting = False
            for i in range(len(f.pages)):
                e = f.pages[i]
                if e >= 0:                                     # never left, or already back through another entry
                    if (f, i) in self.waiters.get(e, ()):
                        self.waiters[e].remove((f, i))
                        if not self.waiters[e]:
                            del self.waiters[e]
                    continue
                s = -e - 1
                q = self._alloc()
                refs = self.host_refs.pop(s)
                for g, j in refs:
                    g.pages[j] = q
                self.refcount[q] = len(refs)
                still = [(g, j) for g, j in refs if g.waiting]
                if still:
                    self.waiters[q] = still
                heapq.heappush(self.free_slots, s)
                out.append((s, q))
        return out

    def is_waiting(self, h):
        return self._file(h).waiting

    # ---- audit -----------------------------------------------------------------
    def audit(self):
        """State invariants: reference counts equal table references; free = count 0."""
        seen, on_host, wait = {}, {}, {}
        files = {id(f): f for f in self.handles.values()}
        files.update({id(f): f for f in self.names.values()})
        for f in files.values():
            assert len(f.pages) == -(-f.length // self.P)
            for i, p in enumerate(f.pages):
                if p < 0:
                    assert f.waiting                       # a page is on the host only while all its readers wait
                    on_host.setdefault(-p - 1, []).append((id(f), i))
                    continue
                seen[p] = seen.get(p, 0) + 1
                if f.waiting:
                    wait.setdefault(p, []).append((id(f), i))
        assert {s: sorted(v) for s, v in on_host.items()} == {s: sorted((id(g), j) for g, j in v) for s, v in self.host_refs.items()}
        assert {p: sorted(v) for p, v in wait.items()} == {p: sorted((id(g), j) for g, j in v) for p, v in self.waiters.items()}
        assert sorted(self.free_slots) == sorted(set(range(self.n_slots)) - set(self.host_refs))
        free = {int(self.order[r]) for r in self.free_ranks}
        assert len(free) == len(self.free_ranks)
        for p in range(self.n_pages):
            assert self.refcount[p] == seen.get(p, 0), (p, self.refcount[p], seen.get(p, 0))
            assert (p in free) == (self.refcount[p] == 0)
        return True


class PagePool:
    """Page contents, stored sparsely: page id -> array [2 (K,V), Hkv, P, D]."""

    def __init__(self, n_kv_heads, page_tokens, head_dim, dtype=np.float32):
        self.shape = (2, n_kv_heads, page_tokens, head_dim)
        self.dtype = dtype
        self.data = {}

    def page(self, p):
        if p not in self.data:
            self.data[p] = np.zeros(self.shape, self.dtype)
        return self.data[p]

    def copy_slots(self, src, dst, r):
        self.page(dst)[:, :, :r, :] = self.page(src)[:, :, :r, :]

    def write_token(self, page, slot, k_row, v_row):
        pg = self.page(page)
        pg[0, :, slot, :] = k_row
        pg[1, :, slot, :] = v_row

    def swap_out(self, evictions):
        """Carry out KVFSModel.kv_offload: page contents to host slots."""
        if not hasattr(self, "host"):
            self.host = {}
        for p, s in evictions:
            self.host[s] = self.page(p).copy()

    def swap_in(self, loads):
        """Carry out KVFSModel.kv_restore: host slots back into pages."""
        for s, q in loads:
            self.data[q] = self.host.pop(s)

    def move_tokens(self, moves):
        """Carry out the copies of KVFSModel.kv_gather: rows of (src page, slot) into (dst page, slot)."""
        for sp, ss, dp, ds in moves:
            self.page(dp)[:, :, ds, :] = self.page(sp)[:, :, ss, :]

    def apply(self, cow, slots, k_new, v_new):
        """Carry out a plan from KVFSModel.append: copies first, then the token rows
        k_new/v_new [T, Hkv, D] in batch order."""
        for src, dst, r in cow:
            self.copy_slots(src, dst, r)
        t = 0
        for mine in slots:
            for page, slot in mine:
                self.write_token(page, slot, k_new[t], v_new[t])
                t += 1
        assert t == len(k_new)

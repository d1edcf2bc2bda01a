"""CPU tests of the C-ABI library's host half: symbols, file-system state against the oracle's
model (bit-exact), and the batch descriptor's structure.  No GPU, no device calls."""
import os
import re

import numpy as np
import pytest

from oracle.kvfs_model import KVFSModel, KVError
from paper_2510_25412_amd import binding
from trace_util import load_trace, parse_expect


def host_ctx(n_pages, free_order=None, Hq=32, Hkv=8, D=128, dtype="bf16", decode_waves=0, tuning=None):
    cfg = binding.make_config(Hq, Hkv, D, 16, dtype, n_pages, device=-1, free_order=free_order, decode_waves=decode_waves,
                              tuning=tuning)
    return binding.Context(cfg)


def test_library_exports_every_declared_symbol(repo_root):
    hdr = open(os.path.join(repo_root, "include", "symphony_kv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sym_[a-z0-9_]+)\s*\(", hdr))
    assert len(declared) >= 20
    lib = binding.load()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(binding._SIGNATURES), declared ^ set(binding._SIGNATURES)


def test_shapes_supported_and_rejected():
    ok = binding.make_config(32, 8, 128, 16, "bf16", 8)
    assert binding.page_bytes(ok) == 8 * 2 * 16 * 256
    assert binding.page_bytes(binding.make_config(8, 8, 64, 16, "f32", 8)) == 65536
    assert binding.page_bytes(binding.make_config(8, 8, 128, 16, "f32", 8)) == 0      # row != 256 bytes
    assert binding.page_bytes(binding.make_config(32, 8, 128, 32, "bf16", 8)) == 0     # page != 16 tokens
    assert binding.page_bytes(binding.make_config(24, 8, 128, 16, "bf16", 8)) == 0     # group of 3
    with pytest.raises(binding.SymError):
        binding.Context(binding.make_config(32, 8, 128, 16, "bf16", 8, device=-1, free_order=[0, 1, 2, 3, 4, 5, 6, 6]))


def test_planner_settings_defaults_overrides_and_clamping():
    """sym_tuning: the defaults depend on the shape only (matrix-core decode and one token per row of heads at 8 query
    heads per kv head; no draft rows in fp32); a caller's struct replaces them; values out of range are clamped, which
    the tile count of a descriptor shows (tile_rows 7 acts as 256, prefill_min -5 as 2)."""
    import ctypes as C
    lib = binding.load()

    def defaults(*shape):
        t = binding.SymTuning()
        assert lib.sym_tuning_defaults(C.byref(binding.make_config(*shape, 8)), C.byref(t)) == 0
        return {n: getattr(t, n) for n in binding.TUNING_FIELDS}

    d4 = defaults(32, 8, 128, 16, "bf16")
    assert d4 == dict(decode_mfma=0, min_units=4, prefill_min=16, share_min_lips=4, share_min_pages=8, tile_rows=256,
                      row_tokens=4, range_cost=3, bin_tolerance=3, bin_waves=8, fuse_append=1, mix_lead=0, mix_spread=50, share_tiles=512)
    d8 = defaults(64, 8, 128, 16, "bf16")
    assert d8["decode_mfma"] == 1 and d8["row_tokens"] == 2
    assert defaults(8, 8, 64, 16, "f32")["row_tokens"] == 1 and defaults(8, 8, 64, 16, "f32")["decode_mfma"] == 0
    t = binding.SymTuning()
    assert lib.sym_tuning_defaults(C.byref(binding.make_config(24, 8, 128, 16, "bf16", 8)), C.byref(t)) == binding.SYM_EINVAL
    assert lib.sym_tuning_defaults(C.byref(binding.make_config(32, 8, 128, 16, "bf16", 8)), None) == binding.SYM_EINVAL
    with pytest.raises(KeyError):
        binding.make_config(32, 8, 128, 16, "bf16", 8, tuning={"no_such_setting": 1})

    def n_tiles(tuning):
        c = host_ctx(64, tuning=tuning)
        words = c.build_desc([64], np.arange(4, dtype=np.int32), [0, 4], [64])
        return int(words[4])
    assert n_tiles(None) == 8 and n_tiles({"tile_rows": 128}) == 16 and n_tiles({"tile_rows": 7}) == 8
    assert n_tiles({"prefill_min": 65}) == 0 and n_tiles({"prefill_min": -5}) == 8


def test_fig1_hand_trace_library():
    """Same hand-derived trace of the paper's Fig. 1 program that pins the oracle's model.
    (The library's pages hold 16 tokens, the trace uses 4: token counts are scaled by 4 and
    slot indices compared after dividing by 4.)"""
    c = host_ctx(8)
    for op, args, exp in load_trace("fig1_state_trace.txt"):
        e = parse_expect(exp)
        if op == "open":
            assert c.kv_open(args[0]) == e["h"]
        elif op == "fork":
            assert c.kv_fork(int(args[0])) == e["h"]
        elif op == "append":
            h, n = int(args[0]), int(args[1]) * 4
            cow, slots = c.plan_append([h], [n])
            assert [(s, d, r // 4) for s, d, r in cow] == e["cow"]
            got = [(int(x) // 16, int(x) % 16 // 4) for x in slots[::4]]
            assert got == e["slots"]
            assert c.kv_pages(h) == e["pages"]
        elif op == "remove":
            c.kv_remove(int(args[0]))
        elif op == "close":
            c.kv_close(int(args[0]))
        elif op == "len":
            assert c.kv_len(int(args[0])) == e["len"] * 4
        if "rc" in e:
            assert [c.page_refcount(p) for p in range(8)] == e["rc"], (op, args)
        if "free" in e:
            assert c.free_pages() == e["free"]


def test_random_ops_with_names_handles_and_bad_batches_match_oracle_model():
    """Names, second handles, close, remove through any handle, stale handles and batches that name a
    file twice (also through two handles): every call returns the same handle or the same error on both
    sides, and after every step every handle number answers kv_len alike."""
    rng = np.random.default_rng(77)
    m = KVFSModel(256, 16)
    c = host_ctx(256)
    names = ["doc%d" % i for i in range(5)]
    top = 0                                              # handle numbers 0 .. top have been seen

    def both(call_m, call_c):
        try:
            a = call_m()
        except KVError as e:
            with pytest.raises(binding.SymError) as ce:
                call_c()
            assert ce.value.code == e.code
            return None
        b = call_c()
        return a, b

    n_busy = n_stale = 0
    for step in range(1200):
        r = rng.random()
        h = int(rng.integers(0, top + 2))                # any number: live, closed, never issued
        if r < 0.15:
            res = both(lambda: m.kv_open(None), lambda: c.kv_open(None))
        elif r < 0.35:
            nm = names[int(rng.integers(len(names)))]
            res = both(lambda: m.kv_open(nm), lambda: c.kv_open(nm))
        elif r < 0.45:
            res = both(lambda: m.kv_fork(h), lambda: c.kv_fork(h))
        elif r < 0.60:
            res = both(lambda: m.kv_close(h), lambda: c.kv_close(h))
            n_stale += res is None
            res = None
        elif r < 0.68:
            both(lambda: m.kv_remove(h), lambda: c.kv_remove(h))
            res = None
        else:
            k = int(rng.integers(1, 5))
            hs = [int(x) for x in rng.integers(0, top + 1, size=k)]        # repeats and two handles of one file happen
            ns = [int(rng.integers(1, 30)) for _ in hs]
            try:
                cow, slots = m.append(list(zip(hs, ns)))
            except KVError as e:
                with pytest.raises(binding.SymError) as ce:
                    c.plan_append(hs, ns)
                assert ce.value.code == e.code
                n_busy += e.code == binding.SYM_EBUSY
            else:
                ccow, cslots = c.plan_append(hs, ns)
                assert ccow == cow and cslots.tolist() == [p * 16 + s for mine in slots for p, s in mine]
            res = None
        if res is not None:
            assert res[0] == res[1]
            top = max(top, res[0])
        for hh in range(top + 2):
            lens = both(lambda: m.kv_len(hh), lambda: c.kv_len(hh))
            if lens is not None:
                assert lens[0] == lens[1]
                if step % 40 == 0:
                    assert c.kv_pages(hh) == m.kv_pages(hh)
        if step % 40 == 0:
            assert c.free_pages() == m.free_pages()
            assert [c.page_refcount(p) for p in range(256)] == m.refcount.tolist()
    assert n_busy > 10 and n_stale > 10                  # the program did name files twice and did use stale handles
    m.audit()


def test_random_ops_match_oracle_model_bit_exact():
    rng = np.random.default_rng(2024)
    order = rng.permutation(512).astype(np.int32)
    m = KVFSModel(512, 16, order)
    c = host_ctx(512, order)
    live = []
    for step in range(1500):
        r = rng.random()
        if r < 0.12 or not live:
            a, b = m.kv_open(), c.kv_open()
            assert a == b
            live.append(a)
        elif r < 0.30:
            p = live[rng.integers(len(live))]
            a, b = m.kv_fork(p), c.kv_fork(p)
            assert a == b
            live.append(a)
        elif r < 0.40:
            h = int(live[rng.integers(len(live))])
            n = int(rng.integers(0, m.kv_len(h) + 1))
            m.kv_truncate(h, n)
            c.kv_truncate([h], [n])
        elif r < 0.52:                       # extract / merge: a new file out of existing tokens
            src = int(live[rng.integers(len(live))])
            L = m.kv_len(src)
            kind = int(rng.integers(5))
            try:
                if kind == 0:
                    srcs = [int(live[i]) for i in rng.integers(len(live), size=int(rng.integers(0, 4)))]
                    a, moves = m.kv_merge(srcs)
                    b = None
                else:
                    idx = {1: np.arange(L)[:int(rng.integers(0, L + 1))],                               # a prefix: all shared
                           2: np.flatnonzero(rng.random(L) < 0.8),                                      # pruned, in order
                           3: np.r_[np.arange(min(L, 16)), np.arange(max(L - 40, min(L, 16)), L)],      # first page + recent window
                           4: rng.integers(0, max(L, 1), size=int(rng.integers(0, 50))) if L else np.zeros(0, np.int64)}[kind]
                    a, moves = m.kv_extract(src, [int(i) for i in idx])
                    b = c.kv_extract(src, idx)
            except KVError as e:
                with pytest.raises(binding.SymError) as ce:
                    c.kv_merge(srcs) if kind == 0 else c.kv_extract(src, idx)
                assert ce.value.code == e.code == binding.SYM_ENOSPC
            else:
                if b is None:
                    b = c.kv_merge(srcs)
                assert a == b
                assert c.last_moves().tolist() == [[sp * 16 + ss, dp * 16 + ds] for sp, ss, dp, ds in moves]
                live.append(a)
        elif r < 0.85:
            k = min(len(live), int(rng.integers(1, 6)))
            hs = [int(x) for x in rng.choice(live, size=k, replace=False)]
            ns = [int(rng.integers(1, 40)) for _ in hs]
            try:
                cow, slots = m.append(list(zip(hs, ns)))
            except KVError as e:
                with pytest.raises(binding.SymError) as ce:
                    c.plan_append(hs, ns)
                assert ce.value.code == e.code
            else:
                ccow, cslots = c.plan_append(hs, ns)
                assert ccow == cow
                assert cslots.tolist() == [p * 16 + s for mine in slots for p, s in mine]
        else:
            h = live.pop(rng.integers(len(live)))
            m.kv_remove(h)
            c.kv_remove(h)
        if step % 50 == 0 or step == 1499:
            assert c.free_pages() == m.free_pages()
            assert [c.page_refcount(p) for p in range(512)] == m.refcount.tolist()
            for h in live:
                assert c.kv_pages(h) == m.kv_pages(h) and c.kv_len(h) == m.kv_len(h)
    st = c.get_stats()
    assert st["cow_copies"] == m.cow_copies and st["pages_free"] == m.free_pages()
    assert st["pages_shared"] == int((m.refcount > 1).sum())
    assert st["tokens_moved"] > 0 and st["pages_referenced"] > 0


def test_extract_merge_hand_trace_library():
    """The hand-worked page-size-16 twin of the model's extract / merge trace, on the library."""
    c = host_ctx(16)
    a = c.kv_open()
    c.plan_append([a], [40])                              # pages 0,1,2 (16, 16, 8 tokens)
    b = c.kv_extract(a, list(range(16)) + [32, 33, 16])   # page 0 referenced; (32, 33, 16) assembled in page 3
    assert c.kv_pages(b) == [0, 3] and c.kv_len(b) == 19
    assert c.last_moves().tolist() == [[32, 48], [33, 49], [16, 50]]
    assert [c.page_refcount(p) for p in range(5)] == [2, 1, 1, 1, 0]
    d = c.kv_extract(a, [32, 33])                         # slots 0, 1 of page 2: a shared, partly used page
    assert c.kv_pages(d) == [2] and len(c.last_moves()) == 0 and c.page_refcount(2) == 2
    cow, slots = c.plan_append([d], [1])                  # the next append copies it first
    assert cow == [(2, 4, 2)] and slots.tolist() == [4 * 16 + 2]
    e = c.kv_merge([a, b])                                # 40 + 19 tokens: pages 0, 1 referenced, the rest assembled
    assert c.kv_len(e) == 59 and c.kv_pages(e) == [0, 1, 5, 6]
    mv = c.last_moves().tolist()
    assert mv[:8] == [[32 + k, 80 + k] for k in range(8)] and mv[8:16] == [[k, 88 + k] for k in range(8)]
    assert mv[16:24] == [[8 + k, 96 + k] for k in range(8)] and mv[24:] == [[48, 104], [49, 105], [50, 106]]
    z = c.kv_extract(a, [])
    assert c.kv_len(z) == 0 and c.kv_pages(z) == []
    assert c.kv_merge([]) >= 0
    # several files in one call: all or none, same result as one call each
    snap = ([c.page_refcount(p) for p in range(16)], c.free_pages())
    with pytest.raises(binding.SymError) as err:
        c.kv_extract_batch([a, b, a], [[1, 2], [18, 0], [0, 40]])
    assert err.value.code == binding.SYM_EINVAL and snap == ([c.page_refcount(p) for p in range(16)], c.free_pages())
    x, y = c.kv_extract_batch([a, b], [[1, 2], list(range(19))])
    assert c.kv_pages(x) == [7] and c.kv_pages(y) == [0, 3] and c.last_moves().tolist() == [[1, 112], [2, 113]]
    c.kv_remove(x)
    c.kv_remove(y)
    snap = ([c.page_refcount(p) for p in range(16)], c.free_pages())
    for call, code in ((lambda: c.kv_extract(a, [40]), binding.SYM_EINVAL), (lambda: c.kv_extract(a, [-1]), binding.SYM_EINVAL),
                       (lambda: c.kv_extract(77, [0]), binding.SYM_EBADF), (lambda: c.kv_merge([a, 77]), binding.SYM_EBADF),
                       (lambda: c.kv_extract(a, np.tile(np.arange(39, -1, -1), 4)), binding.SYM_ENOSPC)):   # 10 fresh pages, 9 free
        with pytest.raises(binding.SymError) as err:
            call()
        assert err.value.code == code
        assert snap == ([c.page_refcount(p) for p in range(16)], c.free_pages())


def test_error_codes_and_all_or_nothing():
    c = host_ctx(4)
    a = c.kv_open()
    c.plan_append([a], [9 * 16 // 4])          # 36 tokens -> 3 pages
    b = c.kv_fork(a)
    snap = ([c.page_refcount(p) for p in range(4)], c.kv_pages(a), c.kv_pages(b), c.free_pages(), c.kv_len(a))
    for kv, n, code in (([a, b], [1, 64], binding.SYM_ENOSPC), ([a, a], [1, 1], binding.SYM_EBUSY),
                        ([a], [0], binding.SYM_EINVAL), ([99], [1], binding.SYM_EBADF)):
        with pytest.raises(binding.SymError) as e:
            c.plan_append(kv, n)
        assert e.value.code == code
        assert snap == ([c.page_refcount(p) for p in range(4)], c.kv_pages(a), c.kv_pages(b), c.free_pages(), c.kv_len(a))
    c.kv_remove(b)
    with pytest.raises(binding.SymError) as e:
        c.kv_fork(b)
    assert e.value.code == binding.SYM_EBADF
    # named files persist across close; anonymous ones vanish with their last handle
    n1 = c.kv_open("sys_msg.kv")
    c.plan_append([n1], [5])
    c.kv_close(n1)
    assert c.free_pages() == 0
    n2 = c.kv_open("sys_msg.kv")
    assert c.kv_len(n2) == 5
    c.kv_close(a)
    assert c.free_pages() == 3
    # a host-only context refuses device calls instead of touching the GPU
    with pytest.raises(binding.SymError):
        c.kv_append(n2, 1, 1, 1)


def test_extract_of_no_tokens_same_codes_as_the_model():
    """An extract of no tokens makes an empty file from a usable source and is refused, with the model's
    code and without a new file, from a stale handle (EBADF) or a waiting file (EBUSY)."""
    m, c = KVFSModel(32, 16), host_ctx(32)
    a, b = c.kv_open(), c.kv_open()
    ma, mb = m.kv_open(), m.kv_open()
    c.plan_append([a, b], [20, 5])
    m.append([(ma, 20), (mb, 5)])
    assert c.kv_extract(a, []) == m.kv_extract(ma, [])[0]
    c.kv_offload([b])
    m.kv_offload([mb])
    files = c.get_stats()["files"]
    for h in (b, 99, -1):
        with pytest.raises(KVError) as em:
            m.kv_extract(h, [])
        with pytest.raises(binding.SymError) as ec:
            c.kv_extract(h, [])
        assert ec.value.code == em.value.code
    assert c.get_stats()["files"] == files and c.free_pages() == m.free_pages()


def _state(c, handles, n_pages):
    return ([c.page_refcount(p) for p in range(n_pages)], [(c.kv_len(h), c.kv_pages(h), c.kv_waiting(h)) for h in handles],
            c.free_pages(), c.get_stats()["files"], c.get_stats()["host_slots"])


def test_a_failed_staging_reservation_changes_nothing():
    """Calls that change file-system state reserve their pinned staging memory first: when that
    reservation fails (forced by the test hook), the call returns SYM_EHIP and page tables, lengths,
    reference counts, free pages, file count and host slots are what they were; the same call then
    succeeds and leaves the state the model predicts."""
    m = KVFSModel(32, 16)
    c = host_ctx(32)
    a, b = c.kv_open(), c.kv_open()
    ma, mb = m.kv_open(), m.kv_open()
    c.plan_append([a, b], [40, 21])
    m.append([(ma, 40), (mb, 21)])
    f = c.kv_fork(a)
    mf = m.kv_fork(ma)
    hs = [a, b, f]

    def failing(call):
        snap = _state(c, hs, 32)
        c.test_fail_staging(1)
        with pytest.raises(binding.SymError) as e:
            call()
        assert e.value.code == binding.SYM_EHIP
        assert _state(c, hs, 32) == snap
        # the hook was used up by the failed call: it does not linger
        return call()

    x = failing(lambda: c.kv_extract(a, [0, 1, 2, 17, 39]))
    mx, _ = m.kv_extract(ma, [0, 1, 2, 17, 39])
    assert c.kv_pages(x) == m.kv_pages(mx)
    y = failing(lambda: c.kv_merge([b, a]))
    my, _ = m.kv_merge([mb, ma])
    assert c.kv_pages(y) == m.kv_pages(my)
    failing(lambda: c.kv_offload([b]))
    m.kv_offload([mb])
    assert c.kv_pages(b) == m.kv_pages(mb) and c.kv_waiting(b)
    failing(lambda: c.kv_restore([b]))
    m.kv_restore([mb])
    assert c.kv_pages(b) == m.kv_pages(mb) and not c.kv_waiting(b)
    assert [c.page_refcount(p) for p in range(32)] == [int(r) for r in m.refcount]
    assert c.free_pages() == m.free_pages()


def _walk_desc(words, Hkv, P=16):
    hdr = words[:20]
    n_rows, n_waves, n_partials, n_lips = (int(x) for x in hdr[:4])
    rows = words[hdr[5]:hdr[5] + 4 * n_rows].reshape(n_rows, 4)
    waves = words[hdr[6]:hdr[6] + 8 * n_waves].reshape(n_waves, 8)
    merge = words[hdr[7]:hdr[7] + 8 * int(hdr[14])].reshape(int(hdr[14]), 8)
    pt = words[hdr[8]:hdr[9]]
    ptoff = words[hdr[9]:hdr[9] + n_lips + 1]
    return n_rows, n_waves, n_partials, rows, waves, merge, pt, ptoff


@pytest.mark.parametrize("lengths,n_tok,waves", [([38, 81, 130, 201], [1, 1, 1, 1], 64), ([700, 16, 17, 1, 4096], [1, 1, 1, 1, 1], 2048),
                                                 ([40, 300], [8, 1], 32), ([5], [5], 8), ([1030, 64, 333, 2000], [3, 2, 1, 7], 96)])
@pytest.mark.parametrize("range_cost", [0, 3])
@pytest.mark.parametrize("row_tokens", [1, 4])
def test_descriptor_covers_every_unit_once_and_is_balanced(lengths, n_tok, waves, range_cost, row_tokens):
    """Rows (up to row_tokens new tokens of one LIP each, a short draft sharing one pass over the
    file), wave ranges, partial numbering and merge entries of the descriptor, walked the way the
    decode kernel walks them."""
    Hkv = 8
    # decode_mfma: the global cut of the matrix-core decode kernel (else: bins, below)
    c = host_ctx(4096, decode_waves=waves, tuning={"range_cost": range_cost, "row_tokens": row_tokens, "decode_mfma": 1})
    rng = np.random.default_rng(1)
    np_l = [-(-L // 16) for L in lengths]
    flat = rng.permutation(4096)[:sum(np_l)].astype(np.int32)
    off = np.concatenate([[0], np.cumsum(np_l)]).astype(np.int64)
    words = c.build_desc(n_tok, flat, off, lengths)
    n_rows, n_waves, n_partials, rows, wv, merge, pt, ptoff = _walk_desc(words, Hkv)
    assert np.array_equal(pt, flat) and np.array_equal(ptoff, off)
    # rows: page-table offset, tokens the first token sees, its q row, (tokens - 1) << 28 | first own page
    exp_rows, q0 = [], 0
    for b, (L, n) in enumerate(zip(lengths, n_tok)):
        for i in range(0, n, row_tokens):
            exp_rows.append((int(off[b]), L - n + i + 1, q0 + i, min(row_tokens, n - i)))
        q0 += n
    assert n_rows == len(exp_rows)
    assert [(int(r[0]), int(r[1]), int(r[2]), (int(r[3]) >> 28) + 1) for r in rows] == exp_rows
    assert not (rows[:, 3] & 0x0fffffff).any()
    nts = [e[3] for e in exp_rows]
    npgs = [-(-(e[1] + e[3] - 1) // 16) for e in exp_rows]        # pages the row's last token sees
    # walk every wave's range exactly as the kernel does; record coverage and partial numbering
    cover = {}
    units, starts = [], []
    pieces = {}
    for k in range(n_waves):
        row, g, p, rem, part = (int(x) for x in wv[k, :5])
        # ids of the first range's first three pages travel with the wave record
        assert wv[k, 5:8].tolist() == [int(pt[int(rows[row, 0]) + min(p + i, npgs[row] - 1)]) for i in range(3)]
        units.append(rem)
        starts.append(0)
        while rem > 0:
            starts[-1] += p == 0
            npg = npgs[row]
            cnt = min(rem, npg - p)
            for x in range(p, p + cnt):
                assert (row, g, x) not in cover
                cover[(row, g, x)] = k
            whole = p == 0 and cnt == npg
            pieces.setdefault((row, g), []).append(None if whole else part)
            if not whole:
                part += nts[row]
            rem -= cnt
            p += cnt
            if p == npg:
                p, g = 0, g + 1
                if g == Hkv:
                    g, row = 0, row + 1
    total = sum(npgs) * Hkv
    assert len(cover) == total and sum(units) == total
    # equal cost whatever the raggedness: units + range_cost per (row, head) begun in the range
    # (a cut that falls into the overhead part of a (row, head) snaps to its first page, which
    # can move one range_cost from one side of the cut to the other)
    cost = [u + range_cost * s for u, s in zip(units, starts)]
    assert max(cost) - min(cost) <= 1 + 2 * range_cost
    assert n_waves <= waves
    items = {}
    for first, cnt, out_idx, xf, xs, xc, stride, _ in merge.tolist():
        assert xc == 0 and out_idx not in items
        items[out_idx] = (first, cnt, stride)
    seen_parts = []
    for (row, g), ps in sorted(pieces.items()):
        for t in range(nts[row]):
            out_idx = (int(rows[row, 2]) + t) * 32 + g * 4          # q row * Hq + first query head of the group
            if ps == [None]:
                assert out_idx not in items                       # whole range: final output, no partial
            else:
                first, cnt, stride = items.pop(out_idx)
                assert None not in ps and stride == nts[row] and cnt == len(ps)
                assert [x + t for x in ps] == [first + i * stride for i in range(cnt)]
                seen_parts += [x + t for x in ps]
    assert not items
    assert sorted(seen_parts) == list(range(n_partials)) and n_partials <= 2 * n_waves * row_tokens


def _walk_bins(words, P=16):
    """Walks the bins of a descriptor the way the vector-unit decode kernel does.  Returns per bin the cost, and
    checks on the way: every wavefront's pieces, the LDS slots they use, the in-bin merge lists."""
    hdr = words[:48]
    n_segs, off_segs, n_bins, W, off_lm = (int(hdr[i]) for i in (32, 33, 34, 35, 36))
    segs = words[off_segs:off_segs + 8 * n_segs].reshape(n_segs, 8)
    assert not words[off_segs + 8 * n_segs:off_segs + 8 * (n_segs + 2)].any()       # the spare records the kernel may read ahead
    waves = words[hdr[6]:hdr[6] + 8 * n_bins * W].reshape(n_bins, W, 8)
    lmerge = words[off_lm:off_lm + 32 * n_bins].reshape(n_bins, 32)
    pt = words[hdr[8]:hdr[9]]
    assert int(hdr[1]) == n_bins * W
    cover = {}                                                     # (segment, page) -> (bin, wavefront)
    seg_bin = {}
    loads = []
    for b in range(n_bins):
        cut = {}                                                   # segment -> [(wavefront, slot)] of its pieces in LDS
        units_b = 0
        for k in range(W):
            seg, p, rem = (int(x) for x in waves[b, k, :3])
            if rem == 0:
                continue
            assert waves[b, k, 4:7].tolist() == [int(pt[int(segs[seg, 0]) + min(p + i, int(segs[seg, 3]) - 1)]) for i in range(3)]
            piece = 0
            while rem > 0:
                pb, pe = int(segs[seg, 2]), int(segs[seg, 3])
                assert pb <= p < pe
                cnt = min(rem, pe - p)
                for x in range(p, p + cnt):
                    assert (seg, x) not in cover
                    cover[(seg, x)] = (b, k)
                assert seg_bin.setdefault(seg, b) == b             # a segment lives in one bin
                if not (p == pb and cnt == pe - pb):
                    cut.setdefault(seg, []).append((k, 2 * k if piece == 0 else 2 * k + 1))
                piece += 1
                units_b += cnt
                rem -= cnt
                seg, p = seg + 1, (int(segs[seg + 1, 2]) if seg + 1 < n_segs else 0)
        # the in-bin merge list names exactly the cut segments, each with the slot of its first piece, that piece's
        # wavefront and the count; later pieces are first pieces of the following wavefronts (slot 2 * wavefront)
        cnt = int(lmerge[b, 0])
        assert cnt <= W - 1 and cnt == len(cut)
        listed = {}
        for e in lmerge[b, 4:4 + 4 * cnt].reshape(cnt, 4).tolist():
            listed[e[0]] = e[1:]
        for seg, ps in cut.items():
            s0, w0, n = listed[seg]
            assert n == len(ps) >= 2 and ps[0] == (w0, s0)
            assert [q for q in ps[1:]] == [(w0 + i, 2 * (w0 + i)) for i in range(1, n)]
        assert len({s for ps in cut.values() for _, s in ps}) == sum(len(ps) for ps in cut.values())   # no slot used twice
        loads.append(units_b)
    return segs, cover, seg_bin, loads, n_bins, W


@pytest.mark.parametrize("lengths,n_tok,waves,range_cost", [
    ([38, 81, 130, 201], [1, 1, 1, 1], 64, 3), ([700, 16, 17, 1, 4096], [1, 1, 1, 1, 1], 2048, 3), ([5], [1], 8, 0),
    ([1030, 64, 333, 2000], [1, 1, 1, 1], 96, 3), ([70000, 33], [1, 1], 2048, 3), ([300] * 40, [1] * 40, 256, 0),
    (list(range(20, 2000, 37)), [1] * 54, 2048, 3)])
def test_descriptor_bins_cover_every_unit_once_and_are_balanced(lengths, n_tok, waves, range_cost):
    """The bins of the vector-unit decode kernel: segments are whole (row, kv head) ranges, or the parts of a range that a
    bin boundary divides; every (row, head, page) is covered by exactly one wavefront; a range in one segment writes the
    output, the segments of a divided range number their partials consecutively and share a merge entry; the bins
    carry equal cost."""
    Hkv, G = 8, 4
    c = host_ctx(1 << 15, decode_waves=waves, tuning={"range_cost": range_cost})
    rng = np.random.default_rng(2)
    np_l = [-(-L // 16) for L in lengths]
    flat = rng.permutation(1 << 15)[:sum(np_l)].astype(np.int32)
    off = np.concatenate([[0], np.cumsum(np_l)]).astype(np.int64)
    words = c.build_desc(n_tok, flat, off, lengths)
    n_rows, n_waves, n_partials, rows, _, merge, pt, ptoff = _walk_desc(words, Hkv)
    assert n_rows == len(lengths) and np.array_equal(pt, flat)
    segs, cover, seg_bin, loads, n_bins, W = _walk_bins(words)
    assert W == 8 and n_bins * W <= max(waves, W)
    # segments against the rows: per (row, head) consecutive pieces that tile [0, pages)
    by_range = {}
    for i, (tbl, g, pb, pe, vis, qh, dest, app) in enumerate(segs.tolist()):
        assert app == -1                                            # build_desc alone appends nothing
        qrow = qh // 32
        assert qh == qrow * 32 + g * G                              # q row * Hq + first query head of the kv head
        by_range.setdefault((qrow, g), []).append((pb, pe, dest, i))
        assert tbl == int(off[qrow]) and vis == lengths[qrow]
    assert sorted(by_range) == [(r, g) for r in range(n_rows) for g in range(Hkv)]
    parts = []
    items = {int(m[2]): m for m in merge.tolist()}
    for (row, g), ps in by_range.items():
        ps.sort()
        assert ps[0][0] == 0 and ps[-1][1] == np_l[row] and all(a[1] == b[0] for a, b in zip(ps, ps[1:]))
        for pb, pe, dest, i in ps:
            assert all((i, x) in cover for x in range(pb, pe))
        key = row * 32 + g * G
        if len(ps) == 1:
            assert ps[0][2] == -1 and key not in items              # whole range in one segment: the final output
        else:
            first, cnt, _, xf, xs, xc, stride, _ = items.pop(key)
            assert cnt == len(ps) and stride == 1 and xc == 0 and [p[2] for p in ps] == list(range(first, first + cnt))
            parts += [p[2] for p in ps]
    assert not items and sorted(parts) == list(range(n_partials))
    assert len(cover) == sum(np_l) * Hkv == sum(loads)
    # balance.  Whole ranges handed out longest first (several ranges per bin): nothing is split and the fullest bin is within
    # 3 % of the mean; otherwise contiguous shares of equal cost: at most n_bins - 1 ranges are cut, and the bins differ by no
    # more than a boundary snapped across one range start
    cost = [0] * n_bins
    for i, (tbl, g, pb, pe, *_rest) in enumerate(segs.tolist()):
        cost[seg_bin[i]] += pe - pb + range_cost
    mean = sum(cost) / n_bins
    if n_partials == 0 and n_bins > 1:
        assert len(segs) >= 3 * n_bins and max(cost) <= 1.03 * mean + 1
    else:
        assert len(parts) - len({k for k, ps in by_range.items() if len(ps) > 1}) <= n_bins - 1       # one extra segment per boundary
        assert max(cost) - min(cost) <= 1 + 2 * range_cost
        assert [seg_bin[i] for i in range(len(segs))] == sorted(seg_bin[i] for i in range(len(segs)))   # contiguous shares


def test_descriptor_rejects_bad_tables():
    c = host_ctx(64)
    with pytest.raises(binding.SymError):
        c.build_desc([1], np.array([1, 2], np.int32), [0, 2], [40])       # needs 3 pages
    with pytest.raises(binding.SymError):
        c.build_desc([1], np.array([1, 2, 64], np.int32), [0, 3], [40])   # page id out of range
    with pytest.raises(binding.SymError):
        c.build_desc([0], np.array([1], np.int32), [0, 1], [4])


@pytest.mark.parametrize("lead,spread", [(0, 50), (100, 0), (0, 0), (0, 100), (30, 40), (99, 1)])
def test_descriptor_order_table_names_every_group_once(lead, spread):
    """A launch with tiles and bins: the order table lists every tile group and every decode group exactly once, tile
    groups in increasing order (tiles come longest first), decode groups too; `mix_lead` percent of the tile groups
    precede the first decode group and all decode groups lie before the end of the next `mix_spread` percent."""
    c = host_ctx(1 << 14, tuning={"mix_lead": lead, "mix_spread": spread})
    lengths = [600, 40, 1000, 333, 64, 2000, 90, 2100] * 5
    n_tok = [64, 1, 128, 1, 16, 1, 1, 1] * 5
    np_l = [-(-L // 16) for L in lengths]
    flat = np.arange(sum(np_l), dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(np_l)]).astype(np.int64)
    words = c.build_desc(n_tok, flat, off, lengths)
    hdr = words[:48]
    n_groups, off_groups, tile_blocks, n_bins = int(hdr[37]), int(hdr[38]), int(hdr[18]), int(hdr[34])
    T, D = tile_blocks // 8, -(-n_bins // 8)
    assert T > 8 and D > 1 and n_groups == T + D
    order = words[off_groups:off_groups + n_groups].tolist()
    assert [g for g in order if g >= 0] == list(range(T))
    assert [~g for g in order if g < 0] == list(range(D))
    first_dec = next(i for i, g in enumerate(order) if g < 0)
    last_dec = max(i for i, g in enumerate(order) if g < 0)
    n_lead = T * lead // 100
    n_spread = min(T - n_lead, -(-T * spread // 100))
    assert first_dec >= n_lead and sum(g >= 0 for g in order[:first_dec]) <= n_lead + max(1, -(-n_spread // D))
    assert sum(g >= 0 for g in order[:last_dec]) <= n_lead + n_spread
    # a batch without tiles, and one without bins, carry no table
    w2 = c.build_desc([1, 1], flat[:100], [0, 40, 100], [630, 950])
    assert int(w2[37]) == 0
    w3 = c.build_desc([64], flat[:40], [0, 40], [600])
    assert int(w3[37]) == 0 and int(w3[4]) > 0


@pytest.mark.parametrize("tile_rows", [128, 256])
def test_descriptor_tiles_for_prefill_chunks(tile_rows):
    """LIPs with 16+ new tokens become tiles (one per kv head and tile_rows / 4 new tokens at 4 heads
    per group); the others stay decode rows; q rows keep the batch's token order."""
    TQ = tile_rows // 4
    c = host_ctx(4096, tuning={"tile_rows": tile_rows})
    lengths, n_tok = [100, 77, 40, 16], [70, 1, 3, 16]
    np_l = [-(-L // 16) for L in lengths]
    flat = np.arange(sum(np_l), dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(np_l)]).astype(np.int64)
    words = c.build_desc(n_tok, flat, off, lengths)
    hdr = words[:20]
    n_rows, n_tiles = int(hdr[0]), int(hdr[4])
    starts = list(range(0, 70, TQ))
    assert n_rows == 2 and n_tiles == (len(starts) + 1) * 8      # the 3-token LIP is one row of three tokens
    rows = words[hdr[5]:hdr[5] + 4 * n_rows].reshape(n_rows, 4)
    assert rows[:, 2].tolist() == [70, 71] and rows[:, 0].tolist() == [int(off[1]), int(off[2])]
    assert rows[:, 1].tolist() == [77, 38] and rows[:, 3].tolist() == [0, 2 << 28]
    tiles = words[hdr[10]:hdr[10] + 12 * n_tiles].reshape(n_tiles, 12)
    exp = [(int(off[0]), 30, t0, min(TQ, 70 - t0), g, t0, 0) for g in range(8) for t0 in starts]
    exp += [(int(off[3]), 0, 74, 16, g, 0, 0) for g in range(8)]
    assert sorted(tuple(int(x) for x in t[:7]) for t in tiles) == sorted(exp)
    # the list comes in 8 shares (one per XCD), tiles of one (file, kv head) together in one share, costs balanced
    xo = words[20:29].tolist()
    assert xo[0] == 0 and xo[8] == n_tiles and all(a <= b for a, b in zip(xo, xo[1:]))
    assert int(words[18]) == 8 * max(b - a for a, b in zip(xo, xo[1:]))
    cost = lambda t: -(-(int(t[1]) + int(t[5]) + int(t[3])) // 32) + 1
    loads, where = [], {}
    for x in range(8):
        share = tiles[xo[x]:xo[x + 1]]
        loads.append(sum(cost(t) for t in share))
        for t in share:
            where.setdefault((int(t[0]), int(t[4])), set()).add(x)
    assert all(len(v) == 1 for v in where.values())
    group_cost = max(sum(cost(t) for t in tiles if (int(t[0]), int(t[4])) == k) for k in where)
    assert max(loads) - min(loads) <= group_cost
    # fp32 storage has no tile kernel: everything is a row
    c32 = host_ctx(4096, Hq=8, Hkv=8, D=64, dtype="f32")
    w32 = c32.build_desc(n_tok, flat, off, lengths)
    assert int(w32[0]) == sum(n_tok) and int(w32[4]) == 0


def test_truncate_errors_change_nothing():
    c = host_ctx(8)
    a, b = c.kv_open(), c.kv_open()
    c.plan_append([a, b], [40, 20])
    for kv, ln, code in (([a, b], [10, 21], binding.SYM_EINVAL), ([a, 77], [1, 1], binding.SYM_EBADF), ([a], [-1], binding.SYM_EINVAL)):
        with pytest.raises(binding.SymError) as e:
            c.kv_truncate(kv, ln)
        assert e.value.code == code and c.kv_len(a) == 40 and c.kv_len(b) == 20
    c.kv_truncate([a, b], [17, 0])
    assert c.kv_len(a) == 17 and len(c.kv_pages(a)) == 2 and c.kv_pages(b) == [] and c.free_pages() == 6


def test_descriptor_shared_prefix_groups():
    """Single-token LIPs whose page lists start with the same ids form a group: the common full
    pages become shared tiles (members x kv heads x key chunks), the members' rows start after
    them, and every (member row, head) gets a merge entry that points at the tiles' partials."""
    c = host_ctx(4096, decode_waves=64)
    prefix = list(range(100, 140))                      # 40 shared pages
    # 6 forks of the prefix with private tails, one unrelated file, one fork that shares only 3 pages
    tables, lengths = [], []
    for i in range(6):
        tail = list(range(1000 + 10 * i, 1000 + 10 * i + 1 + i % 3))
        tables.append(prefix + tail)
        lengths.append(16 * 40 + 16 * (len(tail) - 1) + 1 + i)
    tables.append(list(range(2000, 2020)))
    lengths.append(16 * 20 - 3)
    tables.append(prefix[:3] + list(range(3000, 3030)))
    lengths.append(16 * 33 - 1)
    flat = np.concatenate(tables).astype(np.int32)
    off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int64)
    words = c.build_desc([1] * 8, flat, off, lengths)
    hdr = words[:20]
    n_rows, n_tiles, n_merge, n_members, n_shared = int(hdr[0]), int(hdr[4]), int(hdr[14]), int(hdr[16]), int(hdr[17])
    assert n_rows == 8 and n_members == 6 and n_tiles == n_shared and n_shared % 8 == 0
    nc = n_shared // 8
    rows = words[hdr[5]:hdr[5] + 4 * n_rows].reshape(n_rows, 4)
    assert rows[:, 3].tolist() == [40] * 6 + [0, 0]       # members start after the 40 common pages
    members = words[hdr[15]:hdr[15] + n_members].tolist()
    assert members == [0, 1, 2, 3, 4, 5]
    # page-table section: the first member keeps its whole table (the tiles read the common pages
    # through it); the other five leave the 40 common pages out, and their offsets are moved back by
    # 40 so that page i of the file is still entry offset + i for every page of their own range
    pt = words[hdr[8]:hdr[9]]
    assert len(pt) == len(flat) - 5 * 40
    for b in range(8):
        first = int(rows[b, 3]) & 0x0fffffff if b in (1, 2, 3, 4, 5) else 0
        for i in range(first, len(tables[b])):
            assert int(pt[int(rows[b, 0]) + i]) == tables[b][i], (b, i)
    ptoff = words[hdr[9]:hdr[9] + 9]
    assert ptoff[:8].tolist() == rows[:, 0].tolist() and int(ptoff[8]) == len(pt)
    tiles = words[hdr[10]:hdr[10] + 12 * n_tiles].reshape(n_tiles, 12)
    assert all(int(t[6]) == 1 and int(t[3]) == 6 and int(t[0]) == int(off[0]) for t in tiles)
    covered = {}
    for t in tiles:
        covered.setdefault(int(t[4]), []).append((int(t[7]), int(t[8])))
        assert int(t[7]) % 2 == 0 and int(t[8]) % 2 == 0
    for g in range(8):                                   # every head: the chunks tile [0, 40) exactly
        spans = sorted(covered[g])
        assert spans[0][0] == 0 and spans[-1][1] == 40 and all(a[1] == b[0] for a, b in zip(spans, spans[1:]))
    merge = words[hdr[7]:hdr[7] + 8 * n_merge].reshape(n_merge, 8)
    by_out = {int(m[2]): m for m in merge}
    n_partials = int(hdr[2])
    used = set()
    for r in range(6):
        for g in range(8):
            m = by_out[r * 32 + g * 4]
            assert int(m[1]) >= 1 and int(m[5]) == nc and int(m[4]) == 6
            slots = [int(m[3]) + i * int(m[4]) for i in range(nc)]
            tile_first = sorted(int(t[5]) for t in tiles if int(t[4]) == g)
            assert slots == [f + r for f in tile_first]      # member r of each chunk tile of head g
            used.update(slots)
            used.update(range(int(m[0]), int(m[0]) + int(m[1])))
    assert max(used) < n_partials
    # the unrelated file and the 3-page sharer are ordinary rows
    assert all(int(by_out[k][5]) == 0 for k in by_out if k // 32 >= 6)


def test_descriptor_shared_prefix_chunks_are_never_empty():
    """Common prefixes of 16 .. 200 pages, few and many members: every shared tile covers at least one page, and per kv
    head the key chunks cover the common pages exactly once, in order (pages per chunk are rounded up to whole
    32-token blocks, which must shorten the list of chunks, not leave empty ones at its end)."""
    c = host_ctx(1 << 16)
    for members in (4, 16):
        for C in range(16, 201, 2):
            tables = [list(range(100, 100 + C)) + [5000 + 8 * i, 5001 + 8 * i] for i in range(members)]
            lengths = [16 * C + 17 + i for i in range(members)]
            flat = np.concatenate(tables).astype(np.int32)
            off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int64)
            words = c.build_desc([1] * members, flat, off, lengths)
            hdr = words[:20]
            n_tiles, n_shared = int(hdr[4]), int(hdr[17])
            assert n_tiles == n_shared and n_shared % 8 == 0 and n_shared > 0
            tiles = words[hdr[10]:hdr[10] + 12 * n_tiles].reshape(n_tiles, 12)
            spans = {}
            for t in tiles:
                assert int(t[7]) < int(t[8]), (members, C, t[:9].tolist())
                spans.setdefault(int(t[4]), []).append((int(t[7]), int(t[8])))
            for g in range(8):
                sp = sorted(spans[g])
                assert sp[0][0] == 0 and sp[-1][1] == C and all(a[1] == b[0] for a, b in zip(sp, sp[1:])), (members, C, sp)
            # the members' merge entries count exactly the chunks that exist
            merge = words[hdr[7]:hdr[7] + 8 * int(hdr[14])].reshape(int(hdr[14]), 8)
            assert set(merge[:, 5].tolist()) == {n_shared // 8}


def test_descriptor_shares_the_partial_slots_between_groups():
    """Every member of a shared-prefix group leaves one partial per kv head and key chunk.  When the
    wanted number of key chunks does not fit into the partial slots for all groups, all groups get fewer
    chunks; the first groups must not take what they want and leave the last ones to read their whole
    prefix member by member."""
    c = host_ctx(8192, decode_waves=64)                  # few wave slots: few partial slots
    tables, lengths = [], []
    for gidx in range(5):                                # five groups of six forks of a 64-page prefix
        prefix = list(range(1000 * gidx + 100, 1000 * gidx + 164))
        for i in range(6):
            tables.append(prefix + [1000 * gidx + 500 + i])
            lengths.append(16 * 64 + 1 + i)
    flat = np.concatenate(tables).astype(np.int32)
    off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int64)
    words = c.build_desc([1] * 30, flat, off, lengths)
    hdr = words[:20]
    n_rows, n_tiles, n_members, n_shared = int(hdr[0]), int(hdr[4]), int(hdr[16]), int(hdr[17])
    rows = words[hdr[5]:hdr[5] + 4 * n_rows].reshape(n_rows, 4)
    assert n_members == 30, "every group is shared"
    assert (rows[:, 3] & 0x0fffffff).tolist() == [64] * 30   # every member's own range starts after the prefix
    tiles = words[hdr[10]:hdr[10] + 12 * n_tiles].reshape(n_tiles, 12)
    per_group = {}
    for t in tiles:
        per_group[int(t[0])] = per_group.get(int(t[0]), 0) + 1
    assert len(per_group) == 5 and len(set(per_group.values())) == 1     # the same number of tiles (chunks x heads) for every group


def test_copies_before_appends_only_when_they_overlap():
    """A batch's page copies and appends may run in any order on the device unless an append lands
    in a slot that a copy of the same batch reads: a fork that was truncated (or an extract of a
    leading part) sees fewer tokens of the shared last page than its source; when the source comes
    first in the batch, copies the page and leaves, the other appends in place from its own end."""
    def scenario(how):
        c = host_ctx(64)
        a = c.kv_open()
        c.plan_append([a], [39])                       # 2 full pages + 7 tokens in page 2
        if how == "fork":
            b = c.kv_fork(a)
        elif how == "truncate":
            b = c.kv_fork(a)
            c.kv_truncate([b], [35])                   # sees 3 tokens of page 2
        else:
            b = c.kv_extract(a, np.arange(35))         # page 2 referenced, 3 tokens seen
        assert c.kv_pages(b)[-1] == c.kv_pages(a)[-1] == 2
        return c, a, b

    for how in ("truncate", "extract"):
        c, a, b = scenario(how)
        cow, slots = c.plan_append([a, b], [1, 2])     # a copies slots 0..6 of page 2; b, then alone, writes slots 3 and 4 of it
        assert cow == [(2, 3, 7)] and slots.tolist() == [3 * 16 + 7, 2 * 16 + 3, 2 * 16 + 4]
        assert c.plan_copies_first()
        c, a, b = scenario(how)
        cow, slots = c.plan_append([b, a], [2, 1])     # b copies slots 0..2; a, then alone, writes slot 7: disjoint
        assert cow == [(2, 3, 3)] and slots.tolist() == [3 * 16 + 3, 3 * 16 + 4, 2 * 16 + 7]
        assert not c.plan_copies_first()
    c, a, b = scenario("fork")
    cow, slots = c.plan_append([a, b], [1, 2])         # both see 7 tokens: copy takes slots 0..6, the append slots 7 and 8
    assert cow == [(2, 3, 7)] and slots.tolist() == [3 * 16 + 7, 2 * 16 + 7, 2 * 16 + 8]
    assert not c.plan_copies_first()
    cow, slots = c.plan_append([a], [5])               # the flag belongs to the last plan
    assert cow == [] and not c.plan_copies_first()


def test_offload_restore_hand_trace_library():
    """The model's hand-worked offload / restore trace at page size 16, on the library."""
    c = host_ctx(16)
    a = c.kv_open()
    c.plan_append([a], [40])                              # a: pages 0,1,2
    b = c.kv_fork(a)
    c.plan_append([b], [12])                              # b: 0,1,3,4 (page 2 copied into 3)
    assert c.kv_pages(b) == [0, 1, 3, 4]
    c.kv_offload([a])
    assert c.last_swaps().tolist() == [[2, 0]] and c.kv_pages(a) == [0, 1, -1] and c.free_pages() == 12 and c.kv_waiting(a)
    for call in (lambda: c.plan_append([b, a], [1, 1]), lambda: c.kv_fork(a), lambda: c.kv_truncate([a], [3]),
                 lambda: c.kv_extract(a, [0]), lambda: c.kv_merge([b, a]), lambda: c.kv_offload([a]), lambda: c.kv_restore([b]),
                 lambda: c.kv_offload([b, b])):
        with pytest.raises(binding.SymError) as e:
            call()
        assert e.value.code == binding.SYM_EBUSY
    assert c.kv_len(b) == 52 and c.kv_len(a) == 40 and not c.kv_waiting(b)
    c.kv_offload([b])
    assert c.last_swaps().tolist() == [[0, 1], [1, 2], [3, 3], [4, 4]]
    assert c.kv_pages(a) == [-2, -3, -1] and c.kv_pages(b) == [-2, -3, -4, -5] and c.free_pages() == 16
    c.kv_restore([b])
    assert c.last_swaps().tolist() == [[1, 0], [2, 1], [3, 2], [4, 3]]
    assert c.kv_pages(b) == [0, 1, 2, 3] and c.kv_pages(a) == [0, 1, -1]
    assert [c.page_refcount(p) for p in range(5)] == [2, 2, 1, 1, 0]
    c.kv_restore([a])
    assert c.last_swaps().tolist() == [[0, 4]] and c.kv_pages(a) == [0, 1, 4]
    c.kv_offload([a])
    assert c.kv_pages(a) == [0, 1, -1]
    c.kv_remove(a)                                        # a waiting file can be removed: its slot is released
    st = c.get_stats()
    assert [c.page_refcount(p) for p in range(5)] == [1, 1, 1, 1, 0] and st["host_slots"] == 5
    assert st["pages_offloaded"] == 6 and st["pages_restored"] == 5
    c.kv_offload([b])
    assert c.last_swaps().tolist() == [[0, 0], [1, 1], [2, 2], [3, 3]]       # lowest free slots again


def test_random_ops_with_offload_match_oracle_model_bit_exact():
    rng = np.random.default_rng(77)
    order = rng.permutation(384).astype(np.int32)
    m = KVFSModel(384, 16, order)
    c = host_ctx(384, order)
    live = []

    def both(fm, fc):
        """Same call on model and library: same result or the same error code."""
        try:
            a = fm()
        except KVError as e:
            with pytest.raises(binding.SymError) as ce:
                fc()
            assert ce.value.code == e.code
            return None, None
        return a, fc()

    for step in range(1500):
        r = rng.random()
        h = int(live[rng.integers(len(live))]) if live else None
        if r < 0.1 or not live:
            a, b = m.kv_open(), c.kv_open()
            assert a == b
            live.append(a)
        elif r < 0.2:
            a, b = both(lambda: m.kv_fork(h), lambda: c.kv_fork(h))
            assert a == b
            if a is not None:
                live.append(a)
        elif r < 0.28:
            n = int(rng.integers(0, m.kv_len(h) + 1))
            both(lambda: m.kv_truncate(h, n), lambda: c.kv_truncate([h], [n]))
        elif r < 0.36:
            L = m.kv_len(h)
            idx = np.flatnonzero(rng.random(L) < 0.8)
            a, b = both(lambda: m.kv_extract(h, [int(i) for i in idx]), lambda: c.kv_extract(h, idx))
            if a is not None:
                assert a[0] == b
                live.append(b)
        elif r < 0.62:
            k = min(len(live), int(rng.integers(1, 5)))
            hs = [int(x) for x in rng.choice(live, size=k, replace=False)]
            ns = [int(rng.integers(1, 40)) for _ in hs]
            a, b = both(lambda: m.append(list(zip(hs, ns))), lambda: c.plan_append(hs, ns))
            if a is not None:
                assert b[0] == a[0] and b[1].tolist() == [p * 16 + s for mine in a[1] for p, s in mine]
                # copies before appends exactly when an append of the batch lands in a slot that a copy reads
                overlap = any(p == src and s < cnt for src, _, cnt in a[0] for mine in a[1] for p, s in mine)
                assert c.plan_copies_first() == overlap
        elif r < 0.78:
            k = min(len(live), int(rng.integers(1, 4)))
            hs = [int(x) for x in rng.choice(live, size=k, replace=False)]
            a, _ = both(lambda: m.kv_offload(hs), lambda: c.kv_offload(hs))
            if a is not None:
                assert c.last_swaps().tolist() == [list(x) for x in a]
        elif r < 0.92:
            k = min(len(live), int(rng.integers(1, 4)))
            hs = [int(x) for x in rng.choice(live, size=k, replace=False)]
            a, _ = both(lambda: m.kv_restore(hs), lambda: c.kv_restore(hs))
            if a is not None:
                assert c.last_swaps().tolist() == [list(x) for x in a]
        else:
            live.remove(h)
            m.kv_remove(h)
            c.kv_remove(h)
        if step % 40 == 0 or step == 1499:
            m.audit()
            assert c.free_pages() == m.free_pages()
            assert [c.page_refcount(p) for p in range(384)] == m.refcount.tolist()
            for x in live:
                assert c.kv_pages(x) == m.kv_pages(x) and c.kv_len(x) == m.kv_len(x) and c.kv_waiting(x) == m.is_waiting(x)
    st = c.get_stats()
    assert st["pages_offloaded"] > 100 and st["pages_restored"] > 50 and st["host_slots"] == m.n_slots


@pytest.mark.parametrize("lam,a,c,max_wait", [(1e-4, 100.0, 2.0, 200.0), (0.05, 100.0, 2.0, 200.0), (0.2, 60.0, 1.5, 50.0),
                                               (1.0, 100.0, 2.0, 200.0), (0.02, 400.0, 9.0, 1000.0)])
def test_batch_timer_matches_oracle_decision_by_decision(lam, a, c, max_wait):
    """The library's firing controller against the oracle's on the same Poisson trace: every decision
    at every event time, the waits, and the estimates (identical doubles: same operations in the
    same order)."""
    from oracle.scheduler import BatchTimer as OracleTimer
    from sched_sim import simulate, poisson_arrivals
    arr = poisson_arrivals(lam, 6000, seed=int(lam * 1e5) + 1)
    o, l = OracleTimer(64, max_wait, 0.125, 50.0, 1.0), binding.BatchTimer(64, max_wait, 0.125, 50.0, 1.0)
    lo, ll = [], []
    ro = simulate(o, arr, a, c, log=lo)
    rl = simulate(l, arr, a, c, log=ll)
    assert lo == ll and len(lo) > 90
    assert np.array_equal(ro["waits"], rl["waits"]) and np.array_equal(ro["batches"], rl["batches"])
    st = l.state()
    assert (st["rate"], st["target"], st["a"], st["c"], st["pending"]) == (o.rate(), o.target(), o.a, o.c, len(o.pending))
    l.close()


def test_batch_timer_rejects_bad_arguments():
    for args in ((0, 100.0, 0.1, 1.0, 1.0), (8, -1.0, 0.1, 1.0, 1.0), (8, 100.0, 0.0, 1.0, 1.0), (8, 100.0, 1.5, 1.0, 1.0),
                 (8, 100.0, 0.1, -1.0, 1.0), (8, float("nan"), 0.1, 1.0, 1.0)):
        with pytest.raises(binding.SymError):
            binding.BatchTimer(*args)
    t = binding.BatchTimer(8, 100.0)
    assert t.decide(0.0) == 0 and t.next_deadline() == float("inf")
    t.arrive(5.0)
    assert t.decide(5.0) == 1 and t.decide(5.0, gpu_idle=False) == 0 and t.next_deadline() == 105.0
    t.close()


def test_one_context_from_four_threads():
    """The header promises one mutex per context: four threads work on files of their own in ONE
    context at the same time (ctypes releases the interpreter lock during a call).  Afterwards every
    page is free again, no count is off, and each thread has seen exactly its own tokens."""
    import threading
    c = host_ctx(4096)
    errors = []

    def work(seed):
        try:
            rng = np.random.default_rng(seed)
            mine = {}                                    # handle -> tokens
            for _ in range(1500):
                r = rng.random()
                if r < 0.25 or not mine:
                    mine[c.kv_open()] = 0
                elif r < 0.45:
                    p = int(rng.choice(list(mine)))
                    mine[c.kv_fork(p)] = mine[p]
                elif r < 0.85:
                    hs = [int(h) for h in rng.choice(list(mine), size=min(len(mine), 3), replace=False)]
                    ns = [int(rng.integers(1, 20)) for _ in hs]
                    c.plan_append(hs, ns)
                    for h, n in zip(hs, ns):
                        mine[h] += n
                else:
                    h = int(rng.choice(list(mine)))
                    c.kv_remove(h)
                    del mine[h]
                if len(mine) > 12:
                    h = next(iter(mine))
                    c.kv_remove(h)
                    del mine[h]
            for h, n in mine.items():
                assert c.kv_len(h) == n and len(c.kv_pages(h)) == -(-n // 16)
            for h in list(mine):
                c.kv_remove(h)
        except Exception as e:
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=(s,)) for s in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=60)
    assert not any(t.is_alive() for t in threads) and not errors, errors
    st = c.get_stats()
    assert c.free_pages() == 4096 and st["files"] == 0 and st["handles"] == 0 and st["pages_shared"] == 0
    assert all(c.page_refcount(p) == 0 for p in range(0, 4096, 7))


# ---- do the comparisons above notice when library and model differ? -----------------------------
@pytest.mark.parametrize("module_file,what,edits", [
    ("kvfs_model.py", "highest rank first", [("heapq.heappop(self.free_ranks)", "self.free_ranks.pop(self.free_ranks.index(max(self.free_ranks)))")]),
    ("kvfs_model.py", "shared partial page written in place", [("if r != 0 and self.refcount[f.pages[-1]] > 1:", "if False:")]),
    ("kvfs_model.py", "copy takes one slot too few", [("cow.append((src, dst, r))", "cow.append((src, dst, r - 1))")]),
    ("kvfs_model.py", "truncate keeps one page too few", [("keep=-(-new_len // self.P))", "keep=new_len // self.P)")]),
    ("kvfs_model.py", "extract: nothing is ever shared", [("same = all(pg == toks[0][0] and sl == k for k, (pg, sl) in enumerate(toks))", "same = False")]),
    ("kvfs_model.py", "extract: destination slots shifted", [("moves.append((pg, sl, dst, k))", "moves.append((pg, sl, dst, (k + 1) % P))")]),
    ("kvfs_model.py", "offload: a page leaves as soon as one reader waits", [("if len(self.waiters[p]) == self.refcount[p]:", "if True:")]),
    ("kvfs_model.py", "offload: host slots never reused", [("                    if self.free_slots:\n", "                    if False:\n")]),
    ("kvfs_model.py", "restore: count of the new page is 1", [("self.refcount[q] = len(refs)", "self.refcount[q] = 1")]),
    ("kvfs_model.py", "same file twice in a batch allowed", [("            if any(f is g for g in files):\n                raise KVError(EBUSY, \"same file twice in a batch\")\n", "")]),
    ("kvfs_model.py", "close of the last handle keeps an anonymous file", [("if f.name is None and not f.handles:", "if False:")]),
    ("kvfs_model.py", "second open of a name makes a new file", [("if name is not None and name in self.names:", "if False:")]),
    ("scheduler.py", "target ignores the per-call cost", [("t = lam * self.a / (1.0 - load)", "t = lam * self.a")]),
    ("scheduler.py", "new gaps ignored", [("self.mean_gap = self.mean_gap + self.w * (gap - self.mean_gap)", "pass")]),
    ("scheduler.py", "fires while the GPU is busy", [("if not gpu_idle or not self.pending:", "if not self.pending:")]),
])
def test_library_against_model_tests_notice_a_wrong_model(module_file, what, edits):
    """The library's host state is pinned by comparing it with the oracle's model; here the model is
    made wrong on purpose (in a copy of its source) and the comparisons in this file must fail."""
    from test_oracle_pins_have_teeth import _failing_pins
    me = "test_library_against_model_tests_notice_a_wrong_model"
    assert _failing_pins(module_file, edits, ["test_host_lib.py"], first=True, skip=(me,)), f"no test notices a model with: {what}"

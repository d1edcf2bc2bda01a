"""GPU parity tests: the HIP path through the C ABI against the CPU oracle, element by element
on the same seeded inputs.  Bars: page tables / reference counts bit-exact; attention outputs
within |gpu - ref| <= 2e-3 * max(1, |ref|) (bf16 inputs, fp32 accumulation)."""

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle.driver import run_workload as run_oracle, OracleSession, widen
from paper_2510_25412_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _hip():
    from paper_2510_25412_amd import driver
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return driver


def check_outputs(got, ref, rows=None, tol=TOL):
    if rows is not None:
        got, ref = got[rows], ref[rows]
    n_bad = int((~np.isfinite(got)).sum())
    assert n_bad == 0, f"{n_bad} non-finite outputs"
    worst = float((np.abs(got - ref) / np.maximum(1.0, np.abs(ref))).max())
    assert worst <= tol, f"max scaled error {worst:.3e} > {tol}"
    return worst


def check_state(wl, sess, osess):
    for f in wl.lengths:
        if f in sess.h:
            assert sess.pages(f) == osess.model.kv_pages(osess.h[f]), f
            assert sess.ctx.kv_len(sess.h[f]) == osess.model.kv_len(osess.h[f])
    assert sess.ctx.free_pages() == osess.model.free_pages()
    used = sorted({p for f in sess.h for p in sess.pages(f)})
    assert [sess.ctx.page_refcount(p) for p in used] == [int(osess.model.refcount[p]) for p in used]


def run_both(wl, only=None, **kw):
    print(f"[case] {wl.name} lips={len(wl.batch_files)} tokens={sum(wl.batch_n)}", flush=True)
    got, sess = _hip().run_workload(wl, poison=True, **kw)
    ref, osess = run_oracle(wl, dtype=np.float64, only=only)
    return got, sess, ref, osess


def test_append_read_roundtrip_and_cow_bytes():
    """kv_append then kv_read returns the appended rows bit for bit, across page boundaries,
    for both storage types, and after a copy-on-write of a partly filled shared page."""
    drv = _hip()
    for shape in (synth.Shape(8, 8, 64, 16, synth.F32), synth.Shape(32, 8, 128, 16, synth.BF16)):
        wl = synth.custom("rt", shape, [("new", 45), ("fork", 0, 7), ("fork", 0, 0)], [(0, 1)], 32, seed=5)
        sess = drv.HipSession(shape, 32)
        ops = list(wl.setup_ops())
        sess.setup(ops)
        K0, V0 = ops[1][2], ops[1][3]
        K1, V1 = ops[3][2], ops[3][3]
        tdt = torch.float32 if shape.dtype == synth.F32 else torch.bfloat16
        for fid, Kx, Vx in ((0, K0, V0), (1, np.concatenate([K0, K1]), np.concatenate([V0, V1])), (2, K0, V0)):
            n = len(Kx)
            k = torch.empty((n, shape.n_kv_heads, shape.head_dim), dtype=tdt, device="cuda")
            v = torch.empty_like(k)
            sess.ctx.kv_read(sess.h[fid], 0, n, k, v, sess.stream)
            torch.cuda.synchronize()
            assert np.array_equal(k.float().cpu().numpy(), widen(Kx)) and np.array_equal(v.float().cpu().numpy(), widen(Vx))
        assert sess.ctx.get_stats()["cow_copies"] == 1
        sess.close()


def test_config1_tiny_fp32_all_outputs():
    wl = synth.config1()
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref, tol=1e-5)          # fp32 storage: far inside the bar
    check_state(wl, sess, osess)
    sess.close()


def test_config2_decode_batch_full_size():
    wl = synth.config2()
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


def test_config3_fork_tree_full_size():
    """The fork tree at its full size (16 roots x 16 forks, shared 2048-token prefixes): every output of all
    256 LIPs against the fp64 oracle, state bit for bit."""
    wl = synth.config3()
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    st = sess.ctx.get_stats()
    assert st["cow_copies"] == 0 and st["pages_shared"] == 16 * 128     # aligned prefix: shared, never copied
    sess.close()


def test_config4_mixed_reduced():
    """Mixed prefill + decode at reduced size (chunks of 48 tokens on files of 0..600 tokens,
    plus decode LIPs): every output checked."""
    wl = synth.config4(n_prefill=4, chunk=48, pre_hi=600, n_decode=12, dec_lo=100, dec_hi=500, slack_pages=64)
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


def test_config4_mixed_full_size():
    """The mixed batch at its full size, in the launch configuration the benchmark times (256-row
    tiles on eight-wavefront workgroups, XCD shares, decode ranges in the same grid): every output of the
    32 x 512 prefill tokens and of the 224 decode LIPs against the fp64 oracle, state bit for bit."""
    wl = synth.config4()
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


def test_config5_long_context_full_size():
    """The long-context batch at its full size (16 LIPs of 32k..131k tokens, 64Q/8KV, pages scattered
    by a random allocation ranking over a 3,000,000-page = 196 GB pool: byte offsets beyond 2^32,
    8 query heads per kv head on the matrix cores): every output of all 16 LIPs against the fp64 oracle."""
    wl = synth.config5()
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


@pytest.mark.parametrize("dtype", [synth.F32, synth.BF16])
def test_edge_cases(dtype):
    """Empty file + one token (output = the new V row), page-boundary lengths, a single-token
    file, small multi-token calls, unaligned forks that force copies, parent appending after
    its children, 8:1 and 1:1 head groups."""
    D = 64 if dtype == synth.F32 else 128
    for Hq, Hkv in ((8, 8), (16, 8), (32, 8), (64, 8), (4, 1)):
        shape = synth.Shape(Hq, Hkv, D, 16, dtype)
        files = [("new", 0), ("new", 1), ("new", 15), ("new", 16), ("new", 17), ("new", 31), ("new", 250),
                 ("fork", 6, 0), ("fork", 6, 9), ("fork", 4, 3), ("fork", 9, 0)]
        batch = [(0, 1), (1, 1), (2, 1), (3, 1), (4, 2), (5, 5), (7, 1), (8, 3), (10, 1), (9, 1), (6, 1)]
        wl = synth.custom(f"edge_{dtype}_{Hq}_{Hkv}", shape, files, batch, 128, seed=99 + Hq)
        got, sess, ref, osess = run_both(wl)
        check_outputs(got, ref)
        check_state(wl, sess, osess)
        assert sess.ctx.get_stats()["cow_copies"] == osess.model.cow_copies > 0
        # empty file + one new token: exactly the new V row of the matching kv head
        b = wl.batch()
        v0 = widen(b["v_new"])[0]
        G = Hq // Hkv
        assert np.array_equal(got[0], np.repeat(v0, G, axis=0))
        sess.close()


def test_chunk_equals_sequential_on_gpu():
    """One 6-token pred (draft rows on the matrix cores, softmax weights rounded to fp16) equals
    six 1-token preds (same appended rows; the VALU decode kernel)."""
    drv = _hip()
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    wl = synth.custom("chunk", shape, [("new", 70)], [(0, 6)], 32, seed=123)
    got, sess = drv.run_workload(wl)
    sess.close()
    sess2 = drv.HipSession(shape, 32)
    sess2.setup(wl.setup_ops())
    b = wl.batch()
    outs = []
    for i in range(6):
        one = dict(files=[0], n_tokens=[1], q=b["q"][i:i + 1], k_new=b["k_new"][i:i + 1], v_new=b["v_new"][i:i + 1])
        outs.append(sess2.pred(sess2.upload_batch(one)).cpu().numpy())
    check_outputs(got, np.concatenate(outs), tol=1e-3)
    sess2.close()


def test_enospc_leaves_device_context_unchanged():
    drv = _hip()
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    wl = synth.custom("full", shape, [("new", 40), ("new", 16)], [(0, 1), (1, 1)], 5, seed=3)   # 3 + 1 pages of 5
    sess = drv.HipSession(shape, 5)
    sess.setup(wl.setup_ops())
    from paper_2510_25412_amd import binding
    b = wl.batch()
    big = dict(files=[0, 1], n_tokens=[10, 1], q=np.repeat(b["q"][:1], 11, 0), k_new=np.repeat(b["k_new"][:1], 11, 0),
               v_new=np.repeat(b["v_new"][:1], 11, 0))
    snap = (sess.pages(0), sess.pages(1), sess.ctx.free_pages())
    with pytest.raises(binding.SymError) as e:
        sess.pred(sess.upload_batch(big))
    assert e.value.code == binding.SYM_ENOSPC
    assert snap == (sess.pages(0), sess.pages(1), sess.ctx.free_pages())
    ref, osess = run_oracle(wl, dtype=np.float64)
    got = sess.pred(sess.upload_batch(b)).cpu().numpy()
    check_outputs(got, ref)
    sess.close()


def test_failed_staging_reservation_leaves_device_context_unchanged():
    """pred_batch and kv_append reserve their pinned staging memory before they commit the append: with the
    reservation forced to fail they return SYM_EHIP, files and pool are as before, and the same batch then
    runs and matches the oracle (a half-committed append would show as a file one token longer than its data)."""
    drv = _hip()
    from paper_2510_25412_amd import binding
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    wl = synth.custom("stagefail", shape, [("new", 40), ("fork", 0, 3), ("new", 16)], [(0, 1), (1, 2), (2, 1)], 12, seed=4)
    sess = drv.HipSession(shape, 12, poison=True)
    sess.setup(wl.setup_ops())
    b = wl.batch()
    db = sess.upload_batch(b)
    snap = ([sess.pages(f) for f in (0, 1, 2)], [sess.ctx.kv_len(sess.h[f]) for f in (0, 1, 2)], sess.ctx.free_pages(),
            [sess.ctx.page_refcount(p) for p in range(12)])
    for call in (lambda: sess.pred(db), lambda: sess.ctx.kv_append(sess.h[0], 2, db["k_new"], db["v_new"], sess.stream),
                 lambda: sess.ctx.pred_batch_static(db["kv"], db["n_tokens"], db["q"], db["k_new"], db["v_new"], db["out"], sess.stream)):
        sess.ctx.test_fail_staging(1)
        with pytest.raises(binding.SymError) as e:
            call()
        assert e.value.code == binding.SYM_EHIP
        assert snap == ([sess.pages(f) for f in (0, 1, 2)], [sess.ctx.kv_len(sess.h[f]) for f in (0, 1, 2)], sess.ctx.free_pages(),
                        [sess.ctx.page_refcount(p) for p in range(12)])
    ref, osess = run_oracle(wl, dtype=np.float64)
    got = sess.pred(db).cpu().numpy()
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


def test_raw_entry_matches_allocator_entry():
    """pred_batch_raw over the page tables that pred_batch built gives the same outputs."""
    wl = synth.config2(n_lips=8, lo=100, hi=900, slack_pages=32)
    got, sess = _hip().run_workload(wl)
    b = wl.batch()
    tables = [sess.pages(f) for f in wl.batch_files]
    flat = np.concatenate(tables).astype(np.int32)
    off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int64)
    lengths = [sess.ctx.kv_len(sess.h[f]) for f in wl.batch_files]
    from paper_2510_25412_amd.driver import to_device
    q = to_device(b["q"], sess.device)
    out = torch.empty((len(lengths), 32, 128), dtype=torch.float32, device=sess.device)
    sess.ctx.pred_batch_raw(wl.batch_n, flat, off, lengths, q, out, sess.stream)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), got)
    sess.close()


def test_split_invariance_many_launches():
    """The same batch cut into 2048 wave ranges (many partial results, combined by the merge kernel that follows
    the attention launch) and into 12 ranges gives the same outputs, launch after launch with fresh queries: a
    stale or half-written partial from another XCD would show up here."""
    drv = _hip()
    wl = synth.config2(n_lips=24, lo=60, hi=2500, slack_pages=32)
    sa = drv.HipSession(wl.shape, wl.n_pages, decode_waves=2048)
    sb = drv.HipSession(wl.shape, wl.n_pages, decode_waves=12)
    ops = list(wl.setup_ops())
    sa.setup(ops)
    sb.setup(ops)
    tables = [sa.pages(f) for f in wl.batch_files]
    assert tables == [sb.pages(f) for f in wl.batch_files]
    flat = np.concatenate(tables).astype(np.int32)
    off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int64)
    lengths = [wl.lengths[f] for f in wl.batch_files]
    n = len(lengths)
    g = torch.Generator(device="cuda").manual_seed(7)
    oa = torch.empty((n, 32, 128), dtype=torch.float32, device="cuda")
    ob = torch.empty_like(oa)
    worst = 0.0
    split_tol = 2e-5        # the VALU kernel keeps fp32 weights: different cuts differ by the order of sums only
    for it in range(60):
        q = torch.randn((n, 32, 128), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        oa.fill_(float("nan"))
        ob.fill_(float("nan"))
        sa.ctx.pred_batch_raw([1] * n, flat, off, lengths, q, oa, sa.stream)
        sb.ctx.pred_batch_raw([1] * n, flat, off, lengths, q, ob, sb.stream)
        torch.cuda.synchronize()
        d = ((oa - ob).abs() / ob.abs().clamp(min=1.0)).max().item()
        assert d == d and d <= split_tol, f"launch {it}: split results differ by {d}"
        worst = max(worst, d)
    sa.close()
    sb.close()


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8), (8, 8), (16, 8)])
def test_prefill_chunks_on_matrix_cores(Hq, Hkv):
    """Multi-token pred calls of 16+ tokens (the MFMA tile kernel): chunk lengths around the
    tile and block sizes, on empty, tiny, page-aligned and long files, mixed with decode rows
    and short multi-token calls in one batch; every output checked."""
    shape = synth.Shape(Hq, Hkv, 128, 16, synth.BF16)
    files = [("new", 0), ("new", 0), ("new", 5), ("new", 16), ("new", 31), ("new", 100), ("new", 1000), ("new", 333),
             ("fork", 6, 0), ("new", 64), ("new", 777)]
    batch = [(0, 16), (1, 129), (2, 17), (3, 33), (4, 100), (5, 64), (6, 200), (7, 1), (8, 48), (9, 5), (10, 31)]
    wl = synth.custom(f"prefill_{Hq}_{Hkv}", shape, files, batch, 256, seed=4242 + Hq)
    got, sess, ref, osess = run_both(wl)
    worst = check_outputs(got, ref)
    check_state(wl, sess, osess)
    print(f"prefill {Hq}/{Hkv}: worst scaled error {worst:.2e}")
    sess.close()


def test_prefill_chunk_equals_sequential():
    """A 40-token chunk through the tile kernel equals 40 single-token preds through the decode
    kernel (two different kernels, same appended rows)."""
    drv = _hip()
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    wl = synth.custom("chunk40", shape, [("new", 90)], [(0, 40)], 32, seed=321)
    got, sess = drv.run_workload(wl, poison=True)
    sess.close()
    sess2 = drv.HipSession(shape, 32, poison=True)
    sess2.setup(wl.setup_ops())
    b = wl.batch()
    outs = []
    for i in range(40):
        one = dict(files=[0], n_tokens=[1], q=b["q"][i:i + 1], k_new=b["k_new"][i:i + 1], v_new=b["v_new"][i:i + 1])
        outs.append(sess2.pred(sess2.upload_batch(one)).cpu().numpy())
    check_outputs(got, np.concatenate(outs), tol=1e-3)
    sess2.close()


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8), (8, 8)])
def test_shared_prefix_groups(Hq, Hkv):
    """Forks of a prefix decode through the shared-prefix tiles (prefix pages read once per
    group) + their own rows + the merge: groups larger than a tile, an unaligned prefix, members
    with no private tokens, a fork of a fork, an unrelated file, in one batch.  Outputs must
    match the oracle, and match the run with grouping switched off."""
    shape = synth.Shape(Hq, Hkv, 128, 16, synth.BF16)
    files = [("new", 600), ("new", 205), ("new", 333)]                       # two prefixes, one loner
    files += [("fork", 0, int(s)) for s in (0, 1, 15, 16, 17, 40, 100, 3)]    # 8 forks of file 0
    files += [("fork", 1, 2 * i) for i in range(40)]                         # 40 forks of file 1 (unaligned prefix)
    files += [("fork", 5, 0), ("fork", 5, 9)]                                # forks of a fork
    batch = [(f, 1) for f in range(2, len(files))] + [(0, 1)]
    wl = synth.custom(f"share_{Hq}_{Hkv}", shape, files, batch, 512, seed=77 + Hq)
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()
    plain, sess2 = _hip().run_workload(wl, poison=True, tuning={"share_min_lips": 0})
    sess2.close()
    check_outputs(got, plain, tol=1e-3)     # the tile kernel rounds softmax weights to fp16, the decode kernel does not


@pytest.mark.parametrize("Hq,Hkv,D,dtype", [(32, 8, 128, synth.BF16), (64, 8, 128, synth.BF16), (8, 8, 64, synth.F32)])
def test_very_wide_batch_of_tiny_files(Hq, Hkv, D, dtype):
    """4096 LIPs in one batch, files of 0..40 tokens (empty ones among them), one new token each: 32 768 ranges of one to
    three pages, over a hundred per workgroup, most wavefronts switching range after every page; every output and every
    page table against the oracle."""
    shape = synth.Shape(Hq, Hkv, D, 16, dtype)
    rng = np.random.default_rng(11)
    lengths = rng.integers(0, 41, size=4096)
    lengths[:7] = [0, 1, 15, 16, 17, 31, 32]
    files = [("new", int(L)) for L in lengths]
    batch = [(f, 1) for f in range(len(files))]
    wl = synth.custom(f"wide_{Hq}_{Hkv}", shape, files, batch, 3 * 4096 + 64, seed=606 + Hq)
    got, sess, ref, osess = run_both(wl)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


def test_many_sharing_members_use_the_slots_the_workspace_holds():
    """1600 LIPs in 100 forked groups (9 shared pages each): more sharing members than the partial slots a context
    needs at the least (1280 at 8 kv heads) would hold.  The slots are counted from what the caller's workspace holds
    behind the batch's descriptor, so every group is still read through tiles; all outputs against the oracle, and
    against the run that shares nothing."""
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    n_groups, fan = 100, 16
    files = [("new", 16 * 9 + 3) for _ in range(n_groups)]
    files += [("fork", g, 1 + (7 * g + 3 * i) % 30) for g in range(n_groups) for i in range(fan)]
    batch = [(f, 1) for f in range(n_groups, len(files))]
    wl = synth.custom("many_members", shape, files, batch, 8192, seed=4242)
    got, sess, ref, osess = run_both(wl)
    st = sess.ctx.get_stats()
    assert st["last_batch_shared_rows"] == n_groups * fan and st["last_batch_tiles"] >= n_groups * 8
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()
    plain, sess2 = _hip().run_workload(wl, poison=True, tuning={"share_min_lips": 0})
    sess2.close()
    check_outputs(got, plain, tol=1e-3)


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8), (8, 8), (16, 8)])
@pytest.mark.parametrize("prefix_pages", [1, 2, 3, 4, 5, 7, 9, 16, 41])
def test_small_shared_prefix_tiles_split_by_key_block(Hq, Hkv, prefix_pages):
    """Batches whose shared-prefix tiles all have at most 64 rows run the kernel that splits a tile by
    key block over its two pairs of wavefronts: prefixes of one block (the second pair gets nothing),
    of an odd and an even number of blocks, with a half block at the end (odd page counts), groups of
    fewer than 32 rows (one wavefront per pair) and of exactly 64, members with and without tokens of
    their own.  The sharing thresholds are turned down so that even a one-page prefix is shared."""
    tuning = {"share_min_lips": 2, "share_min_pages": 1}     # (the library raises the page threshold to its minimum, 2)
    G = Hq // Hkv
    shape = synth.Shape(Hq, Hkv, 128, 16, synth.BF16)
    n_big = 64 // G                                      # members of a 64-row group
    files = [("new", 16 * prefix_pages + 5), ("new", 16 * prefix_pages)]
    files += [("fork", 0, int(s)) for s in (0, 1, 17)]                                  # 3 members: 3 * G rows
    files += [("fork", 1, (7 * i) % 40) for i in range(n_big)]                           # exactly 64 rows
    batch = [(f, 1) for f in range(2, len(files))]
    wl = synth.custom(f"split_{Hq}_{Hkv}_{prefix_pages}", shape, files, batch, 1024, seed=300 + prefix_pages + Hq)
    got, sess, ref, osess = run_both(wl, tuning=tuning)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()
    plain, sess2 = _hip().run_workload(wl, poison=True, tuning={"share_min_lips": 0})
    sess2.close()
    check_outputs(got, plain, tol=1e-3)


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8), (8, 8), (16, 8)])
@pytest.mark.parametrize("waves", [0, 24])
def test_draft_verify_rows(Hq, Hkv, waves):
    """Short multi-token pred calls (2..15 new tokens: a draft being verified, paper section 4.1)
    share one pass over the file per row of up to four tokens.  Drafts that straddle page
    boundaries, start on an empty file, sit on long files cut over many wave ranges (partials per
    token, merged), mixed with single-token LIPs and a fork that forces a copy; all outputs
    against the oracle and against the run with one row per token."""
    shape = synth.Shape(Hq, Hkv, 128, 16, synth.BF16)
    files = [("new", 0), ("new", 13), ("new", 14), ("new", 15), ("new", 16), ("new", 29), ("new", 1000), ("new", 2047),
             ("new", 777), ("fork", 8, 5), ("new", 300), ("new", 3000)]
    batch = [(0, 3), (1, 4), (2, 2), (3, 8), (4, 5), (5, 7), (6, 4), (7, 6), (8, 1), (9, 3), (10, 15), (11, 2)]
    wl = synth.custom(f"draft_{Hq}_{Hkv}", shape, files, batch, 512, seed=909 + Hq)
    kw = dict(decode_waves=waves) if waves else {}
    got, sess, ref, osess = run_both(wl, **kw)
    worst = check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()
    plain, sess2 = _hip().run_workload(wl, poison=True, tuning={"row_tokens": 1}, **kw)
    sess2.close()
    check_outputs(got, plain, tol=1e-3)
    print(f"draft rows {Hq}/{Hkv} waves={waves}: worst scaled error {worst:.2e}")


@pytest.mark.parametrize("Hq,Hkv,D,dtype", [(32, 8, 128, synth.BF16), (8, 8, 64, synth.F32), (4, 1, 128, synth.BF16)])
def test_extract_merge_bytes_state_and_pred(Hq, Hkv, D, dtype):
    """kv_extract / kv_merge (section 4.2) on the GPU: page tables and reference counts equal the
    oracle model's bit for bit, every file reads back (kv_read) exactly the oracle's rows, and a
    pred over the new files (and their sources) matches the oracle.  Extracts: pruned subset, first
    page + recent window (unaligned shift), reversed order with repeats, identity, empty; merges:
    unaligned concatenation, a file with itself, of extracts."""
    from oracle.attention import gather_file
    shape = synth.Shape(Hq, Hkv, D, 16, dtype)
    rng = np.random.default_rng(31)
    keep = np.flatnonzero(rng.random(1000) < 0.6)
    files = [("new", 1000), ("new", 77), ("new", 160),
             ("extract", 0, keep),                                            # 3 pruned context
             ("extract", 0, np.r_[np.arange(16), np.arange(700, 1000)]),      # 4 first page + recent window
             ("extract", 1, np.r_[np.arange(76, -1, -1), [5, 5, 5]]),         # 5 reversed, repeats
             ("extract", 2, np.arange(160)),                                  # 6 identity: all pages shared
             ("extract", 2, []),                                              # 7 empty
             ("merge", [1, 2]),                                               # 8 unaligned: 77 + 160
             ("merge", [2, 2, 1]),                                            # 9 aligned start, itself twice
             ("merge", [4, 7, 5]),                                            # 10 of extracts, with an empty one
             ("fork", 6, 3)]                                                  # 11 fork of an extract + private tokens
    batch = [(3, 1), (4, 2), (5, 1), (6, 1), (7, 3), (8, 1), (9, 1), (10, 5), (11, 1), (0, 1), (2, 1)]
    wl = synth.custom(f"xm_{Hq}_{Hkv}_{dtype}", shape, files, batch, 512, seed=1234 + Hq)
    print(f"[case] {wl.name}", flush=True)
    drv = _hip()
    sess = drv.HipSession(shape, wl.n_pages, poison=True)
    sess.setup(wl.setup_ops())
    osess = OracleSession(shape, wl.n_pages)
    osess.setup(wl.setup_ops())
    check_state(wl, sess, osess)
    tdt = torch.float32 if dtype == synth.F32 else torch.bfloat16
    for fid in range(len(files)):
        n = osess.model.kv_len(osess.h[fid])
        assert sess.ctx.kv_len(sess.h[fid]) == n
        if n == 0:
            continue
        k = torch.empty((n, Hkv, D), dtype=tdt, device="cuda")
        v = torch.empty_like(k)
        sess.ctx.kv_read(sess.h[fid], 0, n, k, v, sess.stream)
        torch.cuda.synchronize()
        Ko, Vo = gather_file(osess.pool, osess.model.kv_pages(osess.h[fid]), n)
        assert np.array_equal(k.float().cpu().numpy(), Ko) and np.array_equal(v.float().cpu().numpy(), Vo), fid
    st = sess.ctx.get_stats()
    assert st["tokens_moved"] > 0 and st["pages_referenced"] >= 10 + 1 + 10      # identity extract, first page, merge 9's first file
    b = wl.batch()
    got = sess.pred(sess.upload_batch(b)).cpu().numpy()
    ref = osess.pred(b, dtype=np.float64)
    check_outputs(got, ref)
    check_state(wl, sess, osess)
    sess.close()


@pytest.mark.parametrize("Hq,Hkv,D,dtype", [(32, 8, 128, synth.BF16), (8, 8, 64, synth.F32)])
def test_offload_restore_bytes_state_and_pred(Hq, Hkv, D, dtype):
    """kv_offload / kv_restore (section 4.3) on the GPU: files leave for pinned host memory and come
    back while other files keep appending into the pages they freed (so a copy that ran late, or
    into the wrong slot, would read overwritten bytes).  Page tables, reference counts and host
    slots equal the oracle model's bit for bit; every file reads back exactly the oracle's rows;
    a pred over all files matches the oracle."""
    from oracle.attention import gather_file
    shape = synth.Shape(Hq, Hkv, D, 16, dtype)
    files = [("new", 300), ("fork", 0, 20), ("new", 77), ("new", 1000), ("fork", 3, 0), ("extract", 3, np.arange(0, 1000, 3))]
    then = [("offload", [0]), ("append", 2, 100),            # file 1 still reads file 0's first pages: only the last one leaves
            ("offload", [1, 3]), ("append", 2, 700),         # 0 and 1 all out; 3's pages stay (4 reads them); 2 grows into freed pages
            ("offload", [4]), ("append", 5, 40),             # now 3 and 4 both wait: their pages leave
            ("restore", [1]), ("append", 1, 5),              # back for 0 and 1 at once; 1 copies the shared last page
            ("restore", [4, 0]), ("append", 2, 30), ("restore", [3])]
    batch = [(0, 1), (1, 2), (2, 1), (3, 1), (4, 3), (5, 1)]
    wl = synth.custom(f"swap_{Hq}_{Hkv}_{dtype}", shape, files, batch, 256, seed=555 + Hq, then=then)
    print(f"[case] {wl.name}", flush=True)
    drv = _hip()
    sess = drv.HipSession(shape, wl.n_pages, poison=True)
    osess = OracleSession(shape, wl.n_pages)
    for op in wl.setup_ops():                              # step by step: the state is compared after every operation
        sess.setup([op])
        osess.setup([op])
        for fid in sess.h:
            assert sess.pages(fid) == osess.model.kv_pages(osess.h[fid]), (op[0], fid)
        assert sess.ctx.free_pages() == osess.model.free_pages()
    torch.cuda.synchronize()
    check_state(wl, sess, osess)
    st = sess.ctx.get_stats()
    assert st["pages_offloaded"] == st["pages_restored"] > 80 and st["host_slots"] == osess.model.n_slots
    tdt = torch.float32 if dtype == synth.F32 else torch.bfloat16
    for fid in range(len(files)):
        n = osess.model.kv_len(osess.h[fid])
        k = torch.empty((n, Hkv, D), dtype=tdt, device="cuda")
        v = torch.empty_like(k)
        sess.ctx.kv_read(sess.h[fid], 0, n, k, v, sess.stream)
        torch.cuda.synchronize()
        Ko, Vo = gather_file(osess.pool, osess.model.kv_pages(osess.h[fid]), n)
        assert np.array_equal(k.float().cpu().numpy(), Ko) and np.array_equal(v.float().cpu().numpy(), Vo), fid
    b = wl.batch()
    got = sess.pred(sess.upload_batch(b)).cpu().numpy()
    ref = osess.pred(b, dtype=np.float64)
    check_outputs(got, ref)
    # a waiting file refuses work and leaves the batch untouched
    from paper_2510_25412_amd import binding
    sess.ctx.kv_offload([sess.h[2]], sess.stream)
    before = sess.ctx.kv_len(sess.h[0])
    with pytest.raises(binding.SymError) as e:
        sess.pred(sess.upload_batch(b))
    assert e.value.code == binding.SYM_EBUSY and sess.ctx.kv_len(sess.h[0]) == before
    sess.close()


@pytest.mark.parametrize("pareto_index", [0.6, 3.0])
def test_rag_driver_replayed_on_the_oracle(pareto_index):
    """The RAG workload of the paper's section 5 in miniature (8 documents of 150 tokens, the 3 most
    requested retained, 40 Poisson requests, batches fired by the library's controller): the run is
    recorded, then replayed operation by operation on the CPU model.  Every batch's outputs must
    match the oracle's and the final page tables / reference counts must be identical: prefill
    chunks, decode rows, forks of cached documents, evictions and removals under allocator churn."""
    from paper_2510_25412_amd import rag
    drv = _hip()
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    cfg = rag.RagConfig(n_docs=8, doc_tokens=150, answer_tokens=5, retain=3, pareto_index=pareto_index, rate_per_s=20000.0,
                        n_requests=40, prefill_chunk=64, max_batch=8, max_wait_us=200.0, seed=17)
    n_pages = 1024
    sess = drv.HipSession(shape, n_pages, max_lips=cfg.max_batch, max_tokens=cfg.max_batch * cfg.prefill_chunk + 64,
                          max_entries=cfg.max_batch * 16 + 64, poison=True)
    print(f"[case] rag pareto={pareto_index}", flush=True)
    d = rag.RagDriver(sess, cfg, trace=True)
    res = d.run()
    assert res["requests"] == 40 and res["cached_topics"] <= 3 and 0 < res["mean_batch"] <= 8
    assert res["pred_calls"] == 40 * 5 + (40 - round(res["hit_rate"] * 40)) * 3
    osess = OracleSession(shape, n_pages)
    it = iter(d.outputs)
    worst = 0.0
    for op in d.trace:
        if op[0] == "pred":
            T = sum(op[2])
            ref = osess.pred(dict(files=op[1], n_tokens=op[2], q=d.q_host[:T], k_new=d.k_host[:T], v_new=d.v_host[:T]), dtype=np.float64)
            worst = max(worst, check_outputs(next(it), ref))
        else:
            osess.setup([op])
    assert set(d.h) == set(osess.h)
    for fid in d.h:
        assert sess.ctx.kv_pages(d.h[fid]) == osess.model.kv_pages(osess.h[fid])
    assert sess.ctx.free_pages() == osess.model.free_pages()
    osess.model.audit()
    print(f"rag pareto {pareto_index}: {len(d.outputs)} batches, hit rate {res['hit_rate']:.2f}, worst scaled error {worst:.2e}")
    d.close()
    assert sess.ctx.free_pages() == n_pages
    sess.close()


@pytest.mark.parametrize("Hq,Hkv,D,dtype,seed", [(32, 8, 128, synth.BF16, 1), (64, 8, 128, synth.BF16, 2), (8, 8, 64, synth.F32, 3),
                                                 (16, 8, 128, synth.BF16, 4), (8, 8, 128, synth.BF16, 5), (32, 8, 128, synth.BF16, 6),
                                                 (32, 8, 64, synth.F32, 7), (4, 1, 128, synth.BF16, 8),
                                                 (16, 8, 128, synth.BF16, 123), (32, 8, 128, synth.BF16, 126)])
def test_random_program_against_oracle(Hq, Hkv, D, dtype, seed):
    _random_program(Hq, Hkv, D, dtype, seed, big=False)


@pytest.mark.parametrize("Hq,Hkv,D,dtype,seed", [(32, 8, 128, synth.BF16, 4), (64, 8, 128, synth.BF16, 1)])
def test_random_program_large(Hq, Hkv, D, dtype, seed):
    """The same at sizes where prefill chunks span several tiles, prefixes of up to 3000 tokens are
    shared by twelve files and batches hold up to 48 LIPs."""
    _random_program(Hq, Hkv, D, dtype, seed, big=True)


def _random_program(Hq, Hkv, D, dtype, seed, big):
    """A seeded random program over the whole API (open, append, fork, extract, merge, truncate,
    offload, restore, remove, pred batches that mix single tokens, drafts and prefill chunks) run
    step by step on the library and on the oracle: same error codes, every pred's outputs within the
    bar, page tables / reference counts / free pages equal after every step.  What a fixed scenario
    does not think of (a fork of an extract that waits while its source is truncated, ...) shows up here."""
    from oracle.kvfs_model import KVError
    from paper_2510_25412_amd import binding
    drv = _hip()
    shape = synth.Shape(Hq, Hkv, D, 16, dtype)
    # sizes: steps, pool pages, LIPs per batch, tokens per batch, forks of a long prefix, its length, file and append lengths, chunk sizes
    if big:
        n_steps, n_pages, max_lips, max_tok, n_forks, pre_lo, pre_hi, new_hi, app_hi, keep = 110, 16384, 48, 8192, 11, 600, 3000, 1500, 400, 40
        chunks = [1, 1, 1, 1, 1, 1, 2, 3, 5, 8, 17, 40, 130, 300]
    else:
        n_steps, n_pages, max_lips, max_tok, n_forks, pre_lo, pre_hi, new_hi, app_hi, keep = 260, 1536, 16, 1024, 5, 140, 400, 70, 50, 6
        chunks = [1, 1, 1, 1, 2, 3, 5, 8, 17, 40]
    sess = drv.HipSession(shape, n_pages, max_lips=max_lips, max_tokens=max_tok, max_entries=1 << 18, poison=True)
    osess = OracleSession(shape, n_pages)
    rng = np.random.default_rng(1000 + seed)
    print(f"[case] random program {Hq}/{Hkv} {dtype} seed {seed}", flush=True)

    def data(n, heads):
        x = rng.standard_normal((n, heads, D), dtype=np.float32)
        return synth.bf16_round(x) if dtype == synth.BF16 else x

    def both(op):
        """The same setup operation on both sides: both succeed or both fail with the same code."""
        try:
            osess.setup([op])
        except KVError as e:
            with pytest.raises(binding.SymError) as ce:
                sess.setup([op])
            assert ce.value.code == e.code, op[0]
            return False
        sess.setup([op])
        return True

    next_fid, n_pred, worst = 0, 0, 0.0
    for step in range(n_steps):
        fids = sorted(osess.h)
        live = [f for f in fids if not osess.model.is_waiting(osess.h[f])]
        r = rng.random()
        if step % 60 == 5:                  # a long prefix forked five times: decode through shared-prefix tiles
            both(("open", next_fid))
            both(("append", next_fid, data(n := int(rng.integers(pre_lo, pre_hi)), Hkv), data(n, Hkv)))
            for i in range(1, n_forks + 1):
                both(("fork", next_fid + i, next_fid))
            next_fid += n_forks + 1
        elif r < 0.08 or len(fids) < 3:
            both(("open", next_fid))
            both(("append", next_fid, data(n := int(rng.integers(1, new_hi)), Hkv), data(n, Hkv)))
            next_fid += 1
        elif r < 0.2 and live:
            f = int(rng.choice(live))
            both(("append", f, data(n := int(rng.integers(1, app_hi)), Hkv), data(n, Hkv)))
        elif r < 0.3 and fids:
            if both(("fork", next_fid, int(rng.choice(fids)))):
                next_fid += 1
        elif r < 0.37 and fids:
            f = int(rng.choice(fids))
            L = osess.model.kv_len(osess.h[f])
            idx = np.flatnonzero(rng.random(L) < 0.7) if rng.random() < 0.7 else np.arange(L)[:int(rng.integers(0, L + 1))]
            if both(("extract", next_fid, f, [int(i) for i in idx])):
                next_fid += 1
        elif r < 0.42 and len(fids) >= 2:
            if both(("merge", next_fid, [int(x) for x in rng.choice(fids, size=2)])):
                next_fid += 1
        elif r < 0.47 and live:
            f = int(rng.choice(live))
            n = int(rng.integers(0, osess.model.kv_len(osess.h[f]) + 1))
            osess.model.kv_truncate(osess.h[f], n)
            sess.ctx.kv_truncate([sess.h[f]], [n])
        elif r < 0.55 and fids:
            both(("offload", [int(x) for x in rng.choice(fids, size=min(len(fids), int(rng.integers(1, 3))), replace=False)]))
        elif r < 0.63 and fids:
            both(("restore", [int(x) for x in rng.choice(fids, size=min(len(fids), int(rng.integers(1, 3))), replace=False)]))
        elif r < 0.7 and len(fids) > keep:
            f = int(rng.choice(fids))
            osess.setup([("remove", f)])
            sess.setup([("remove", f)])
        elif live:
            k = int(rng.integers(1, min(len(live), max_lips) + 1))
            files = [int(x) for x in rng.choice(live, size=k, replace=False)]
            nt = [int(rng.choice(chunks)) for _ in files]
            T = sum(nt)
            b = dict(files=files, n_tokens=nt, q=data(T, Hq), k_new=data(T, Hkv), v_new=data(T, Hkv))
            try:
                ref = osess.pred(b, dtype=np.float64)
            except KVError as e:
                with pytest.raises(binding.SymError) as ce:
                    sess.pred(sess.upload_batch(b))
                assert ce.value.code == e.code
            else:
                got = sess.pred(sess.upload_batch(b)).cpu().numpy()
                worst = max(worst, check_outputs(got, ref))
                n_pred += 1
        for f in osess.h:
            assert sess.ctx.kv_pages(sess.h[f]) == osess.model.kv_pages(osess.h[f]), (step, f)
        assert sess.ctx.free_pages() == osess.model.free_pages(), step
    torch.cuda.synchronize()
    used = sorted({p for f in osess.h for p in osess.model.kv_pages(osess.h[f]) if p >= 0})
    assert [sess.ctx.page_refcount(p) for p in used] == [int(osess.model.refcount[p]) for p in used]
    osess.model.audit()
    assert n_pred > (10 if big else 40)
    print(f"random program: {n_pred} pred batches, worst scaled error {worst:.2e}")
    sess.close()


def test_calibration_kernels():
    """The kernels that bench.py calibrates against do the work they are priced at: the copy copies
    every byte, the streaming read leaves its checksum slot alone, and the MFMA loop's accumulators
    hold the products of its operands (checked through a sum that needs only the MFMA operand layout:
    lane l supplies row or column l % 32 and the 8 consecutive k from 8 * (l / 32))."""
    from paper_2510_25412_amd import binding
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    n = (1 << 20) + 48
    src = torch.randint(0, 255, (n,), dtype=torch.uint8, device=dev)
    dst = torch.zeros_like(src)
    binding.calib_copy(dst, src, n)
    out8 = torch.zeros(1, dtype=torch.int64, device=dev)
    binding.calib_read(src, n, out8)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert int(out8.item()) in (0, 1)

    blocks, iters = 3, 2
    sink = torch.full((blocks * 512,), float("nan"), dtype=torch.float32, device=dev)
    flops = binding.calib_mfma(sink, blocks, iters)
    torch.cuda.synchronize()
    assert flops == blocks * 8 * iters * 16 * 32768
    got = sink.cpu().numpy().astype(np.float64).reshape(blocks, 8, 64)
    tid = np.arange(512, dtype=np.uint64).reshape(8, 64, 1, 1)
    e = np.arange(8, dtype=np.uint64).reshape(1, 1, 1, 8)
    i = np.arange(4, dtype=np.uint64).reshape(1, 1, 4, 1)
    for b in range(blocks):
        hsh = ((tid * 8 + e + 131 * i + 977 * b) * 2654435761) & 0xFFFFFFFF          # [wave][lane][reg][elem]
        x = ((hsh >> 20).astype(np.int64) - 2048) / 2048.0
        y = (((hsh >> 8) & 4095).astype(np.int64) - 2048) / 2048.0
        bf = lambda a: torch.tensor(a, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
        x, y = bf(x), bf(y)
        # column sums of A and row sums of B over the 32 lanes that hold the same k: k = 8 * (lane / 32) + elem
        sa = x.reshape(8, 2, 32, 4, 8).sum(axis=2).transpose(0, 2, 1, 3).reshape(8, 4, 16)   # [wave][reg][k]
        sb = y.reshape(8, 2, 32, 4, 8).sum(axis=2).transpose(0, 2, 1, 3).reshape(8, 4, 16)
        for w in range(8):
            want = iters * sum(float(sa[w, (a + r) & 3] @ sb[w, a]) for a in range(4) for r in range(4))
            have = got[b, w].sum() - 2016.0              # every thread adds its lane index
            assert abs(have - want) <= 2e-2 + 1e-3 * abs(want), (b, w, have, want)     # fp32 sums of ~1e3 terms


@pytest.mark.parametrize("Hq,Hkv", [(32, 8), (64, 8)])
def test_every_kind_of_work_in_one_batch(Hq, Hkv):
    """Two fork groups (their members' page tables travel without the common pages), a prefill
    chunk, plain single-token LIPs and drafts of 3 and 6 tokens in ONE batch: prefill and shared-prefix
    tiles in one grid with the decode work, and, because of the drafts, every decode range (the
    members' own ranges included) on the matrix-core decode kernel.  Few waves, so that ranges are
    cut inside the members' rows too."""
    shape = synth.Shape(Hq, Hkv, 128, 16, synth.BF16)
    files = [("new", 700), ("new", 330), ("new", 1500), ("new", 64), ("new", 909)]
    files += [("fork", 0, int(s)) for s in (5, 40, 0, 17, 90, 33)]          # files 5..10: forks of file 0
    files += [("fork", 1, int(s)) for s in (1, 2, 3, 60, 7)]                # files 11..15: forks of file 1
    batch = [(f, 1) for f in range(5, 16)] + [(2, 1), (3, 100), (4, 3), (0, 6), (1, 1)]
    wl = synth.custom(f"allkinds_{Hq}_{Hkv}", shape, files, batch, 1024, seed=4242 + Hq)
    for waves in (0, 40):
        kw = dict(decode_waves=waves) if waves else {}
        got, sess, ref, osess = run_both(wl, **kw)
        worst = check_outputs(got, ref)
        check_state(wl, sess, osess)
        sess.close()
        print(f"all kinds {Hq}/{Hkv} waves={waves}: worst scaled error {worst:.2e}")


_SETTINGS = [{"bin_waves": 4}, {"fuse_append": 0}, {"bin_tolerance": 0}, {"bin_tolerance": 1000}, {"min_units": 1, "range_cost": 0},
             {"mix_lead": 100, "mix_spread": 0}, {"mix_lead": 0, "mix_spread": 0}, {"mix_lead": 0, "mix_spread": 100}, {"mix_lead": 40, "mix_spread": 30},
             {"share_tiles": 16}, {"share_tiles": 4096}, {"share_min_lips": 2, "share_min_pages": 2}, {"tile_rows": 128}, {"prefill_min": 2},
             {"prefill_min": 200}, {"row_tokens": 1}, {"decode_mfma": 1}, {"decode_mfma": 1, "row_tokens": 2}]


@pytest.mark.parametrize("with_chunk", [False, True])
def test_every_planner_setting_gives_the_oracles_outputs(with_chunk):
    """sym_tuning decides where work runs, never what is computed: one batch (two fork groups, plain LIPs of very
    different lengths, a short draft; with or without a prefill chunk, i.e. as `attn_kernel` with its order table or as
    `decode_only_kernel`) under every setting in turn, few wavefront slots so that ranges are cut; each run against the
    oracle (computed once) and the final page tables against the model."""
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    files = [("new", 700), ("new", 330), ("new", 1500), ("new", 64), ("new", 909), ("new", 15), ("new", 2300)]
    files += [("fork", 0, int(x)) for x in (5, 40, 0, 17, 90, 33)]          # forks of file 0
    files += [("fork", 1, int(x)) for x in (1, 2, 3, 60, 7)]                # forks of file 1
    batch = [(f, 1) for f in range(7, 18)] + [(2, 1), (4, 1), (5, 1), (6, 1), (0, 3)]
    if with_chunk:
        batch += [(3, 100)]
    else:
        batch.remove((0, 3))             # a plain decode batch: one new token everywhere
    wl = synth.custom(f"settings_{int(with_chunk)}", shape, files, batch, 1024, seed=777 + int(with_chunk))
    ref, osess = run_oracle(wl, dtype=np.float64)
    for tuning in [None] + _SETTINGS:
        print(f"[case] {wl.name} tuning={tuning}", flush=True)
        got, sess = _hip().run_workload(wl, poison=True, tuning=tuning, decode_waves=48)
        worst = check_outputs(got, ref)
        check_state(wl, sess, osess)
        sess.close()
        print(f"  worst scaled error {worst:.2e}")


@pytest.mark.parametrize("Hq,Hkv,D,dtype,multi", [(32, 8, 128, synth.BF16, 1), (32, 8, 128, synth.BF16, 3), (8, 8, 64, synth.F32, 3),
                                                  (64, 8, 128, synth.BF16, 1), (16, 8, 128, synth.BF16, 1)])
def test_layered_pred_layer_by_layer_against_the_oracle(Hq, Hkv, D, dtype, multi):
    """A context with three layers: one page table, three layers of every page.  The files are built with different rows
    in every layer (forks, a copy-on-write, an extract, an offload and restore: every layer must move), then one batch
    (decode LIPs, forks of one prefix, a LIP with several new tokens, a prefill chunk where tiles exist) runs as
    sym_pred_begin + one sym_pred_layer per layer, in shuffled layer order.  Per layer: outputs against an oracle that
    was given that layer's rows; afterwards every file of every layer is read back and compared bit for bit with the
    oracle's pages (the appends that ride in the attention kernel included); the state calls refused while layers are
    left are checked on the way."""
    drv = _hip()
    from paper_2510_25412_amd import binding
    L = 3
    shape = synth.Shape(Hq, Hkv, D, 16, dtype)
    files = [("new", 45), ("fork", 0, 7), ("fork", 0, 0), ("new", 300), ("new", 16), ("extract", 3, list(range(0, 300, 3))),
             ("new", 700)] + [("fork", 6, int(x)) for x in (3, 0, 18, 40, 1)]
    # (a bf16 batch with a LIP of 2..15 new tokens runs all its decode rows on the matrix cores; without one, the vector-unit
    # kernel runs them in bins and appends the single tokens itself)
    batch = [(0, 1), (1, 1), (2, multi), (3, 1), (4, 40 if dtype == synth.BF16 else 5), (5, 1)] + [(f, 1) for f in range(7, 12)]
    wls = [synth.custom(f"layered{l}", shape, files, batch, 256, seed=900 + 17 * l, then=[("offload", [3, 5]), ("restore", [3, 5])])
           for l in range(L)]
    sess = drv.HipSession(shape, 256, device="cuda:0", max_lips=len(batch), max_tokens=1024, max_entries=4096, poison=True,
                          n_layers=L, decode_waves=24)
    # the same program on every layer's rows: append ops carry [L, n, Hkv, D]
    for ops in zip(*[list(w.setup_ops()) for w in wls]):
        op = ops[0]
        if op[0] == "append":
            op = ("append", op[1], np.stack([o[2] for o in ops]), np.stack([o[3] for o in ops]))
        sess.setup([op])
    refs, osessions = zip(*[run_oracle(w, dtype=np.float64) for w in wls])
    bs = [w.batch() for w in wls]
    dbs = [sess.upload_batch(b) for b in bs]
    kv, nt = dbs[0]["kv"], dbs[0]["n_tokens"]
    with pytest.raises(binding.SymError) as e:                 # no batch is open yet
        sess.ctx.pred_layer(0, dbs[0]["q"], dbs[0]["k_new"], dbs[0]["v_new"], dbs[0]["out"], sess.stream)
    assert e.value.code == binding.SYM_EINVAL
    sess.ctx.pred_begin(kv, nt, sess.stream)
    for l in (2, 0):
        sess.ctx.pred_layer(l, dbs[l]["q"], dbs[l]["k_new"], dbs[l]["v_new"], dbs[l]["out"], sess.stream)
    for call in (lambda: sess.ctx.kv_fork(kv[0]), lambda: sess.ctx.kv_remove(kv[0]), lambda: sess.ctx.pred_begin(kv, nt, sess.stream),
                 lambda: sess.ctx.kv_truncate([kv[0]], [3]), lambda: sess.ctx.kv_offload([kv[0]], sess.stream),
                 lambda: sess.ctx.pred_layer(2, dbs[2]["q"], dbs[2]["k_new"], dbs[2]["v_new"], dbs[2]["out"], sess.stream)):
        with pytest.raises(binding.SymError) as e:             # one layer is left: nothing may change the files
            call()
        assert e.value.code == binding.SYM_EBUSY
    sess.ctx.pred_layer(1, dbs[1]["q"], dbs[1]["k_new"], dbs[1]["v_new"], dbs[1]["out"], sess.stream)
    torch.cuda.synchronize()
    for l in range(L):
        worst = check_outputs(dbs[l]["out"].cpu().numpy(), refs[l])
        print(f"layer {l}: worst scaled error {worst:.2e}")
    check_state(wls[0], sess, osessions[0])
    from oracle.attention import gather_file
    tdt = torch.float32 if dtype == synth.F32 else torch.bfloat16
    for l in range(L):
        for f in range(len(files)):
            n = sess.ctx.kv_len(sess.h[f])
            k = torch.empty((n, Hkv, D), dtype=tdt, device="cuda")
            v = torch.empty_like(k)
            sess.ctx.kv_read(sess.h[f], 0, n, k, v, sess.stream, layer=l)
            torch.cuda.synchronize()
            K, V = gather_file(osessions[l].pool, osessions[l].model.kv_pages(osessions[l].h[f]), n)
            assert np.array_equal(k.float().cpu().numpy(), K) and np.array_equal(v.float().cpu().numpy(), V), (l, f)
    sess.ctx.kv_fork(kv[0])                                       # the batch is complete: the files can change again
    sess.close()


@pytest.mark.parametrize("how", ["truncate", "extract"])
def test_copy_and_in_place_append_on_one_page_in_one_batch(how):
    """Two files share a partly filled page but see different numbers of its tokens (a fork that
    was truncated, or an extract of a leading part).  In one batch the file that sees more comes
    first and copies the page; the other is then the only owner and appends in place, into slots
    that the first one's copy must still read: the copies have to run before the appends.  (With
    forks alone both see the same number of tokens and copies and appends are disjoint.)"""
    drv = _hip()
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    sess = drv.HipSession(shape, 256, max_lips=8, max_tokens=256, max_entries=4096, poison=True)
    osess = OracleSession(shape, 256)
    rng = np.random.default_rng(31 + len(how))

    def data(n, heads):
        return synth.bf16_round(rng.standard_normal((n, heads, 128), dtype=np.float32))

    def both(op):
        osess.setup([op])
        sess.setup([op])

    both(("open", 0))
    both(("append", 0, data(239, 8), data(239, 8)))          # 14 full pages + 15 tokens
    if how == "truncate":
        both(("fork", 1, 0))
        osess.model.kv_truncate(osess.h[1], 232)             # the fork sees 8 tokens of the shared last page
        sess.ctx.kv_truncate([sess.h[1]], [232])
    else:
        both(("extract", 1, 0, list(range(232))))
    assert sess.ctx.kv_pages(sess.h[1])[-1] == sess.ctx.kv_pages(sess.h[0])[-1]      # the last page is shared
    for files, nt in (([0, 1], [2, 8]), ([1, 0], [3, 1])):
        T = sum(nt)
        b = dict(files=files, n_tokens=nt, q=data(T, 32), k_new=data(T, 8), v_new=data(T, 8))
        ref = osess.pred(b, dtype=np.float64)
        got = sess.pred(sess.upload_batch(b)).cpu().numpy()
        check_outputs(got, ref)
        for f in (0, 1):
            assert sess.ctx.kv_pages(sess.h[f]) == osess.model.kv_pages(osess.h[f])
    # every stored token of both files, bit for bit
    from oracle.attention import gather_file
    for f in (0, 1):
        n = osess.model.kv_len(osess.h[f])
        k = torch.empty((n, 8, 128), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        sess.ctx.kv_read(sess.h[f], 0, n, k, v, sess.stream)
        torch.cuda.synchronize()
        Ko, Vo = gather_file(osess.pool, osess.model.kv_pages(osess.h[f]), n)
        assert np.array_equal(k.float().cpu().numpy(), Ko) and np.array_equal(v.float().cpu().numpy(), Vo), f
    sess.close()


@pytest.mark.parametrize("n_moved", [1, 2, 3, 5])
def test_extract_of_very_few_tokens(n_moved):
    """An extract or merge that has to copy one, two or three tokens: the list of moves is shorter than
    one 16-byte unit of the copy that brings it to the device.  The new file and every other file
    read back bit for bit (a move list that did not arrive would move whatever the workspace held)."""
    from oracle.attention import gather_file
    drv = _hip()
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    sess = drv.HipSession(shape, 128, max_lips=8, max_tokens=256, max_entries=4096, poison=True)
    osess = OracleSession(shape, 128)
    rng = np.random.default_rng(900 + n_moved)

    def data(n, heads):
        return synth.bf16_round(rng.standard_normal((n, heads, 128), dtype=np.float32))

    def both(op):
        osess.setup([op])
        sess.setup([op])

    for f, n in ((0, 70), (1, 33), (2, 5)):
        both(("open", f))
        both(("append", f, data(n, 8), data(n, 8)))
    # a pred first, so that the workspace holds a descriptor when the move list is due
    b = dict(files=[0, 1, 2], n_tokens=[1, 1, 1], q=data(3, 32), k_new=data(3, 8), v_new=data(3, 8))
    check_outputs(sess.pred(sess.upload_batch(b)).cpu().numpy(), osess.pred(b, dtype=np.float64))
    both(("extract", 3, 0, [int(i) for i in rng.choice(71, size=n_moved, replace=False)]))
    both(("extract", 4, 2, [1 + i for i in range(min(n_moved, 5))]))
    for f in range(5):
        n = osess.model.kv_len(osess.h[f])
        k = torch.empty((n, 8, 128), dtype=torch.bfloat16, device="cuda")
        v = torch.empty_like(k)
        sess.ctx.kv_read(sess.h[f], 0, n, k, v, sess.stream)
        torch.cuda.synchronize()
        Ko, Vo = gather_file(osess.pool, osess.model.kv_pages(osess.h[f]), n)
        assert np.array_equal(k.float().cpu().numpy(), Ko) and np.array_equal(v.float().cpu().numpy(), Vo), f
        assert sess.ctx.kv_pages(sess.h[f]) == osess.model.kv_pages(osess.h[f])
    sess.close()


@pytest.mark.parametrize("Hq,Hkv,D,dtype,seed", [(32, 8, 128, synth.BF16, 3), (64, 8, 128, synth.BF16, 4), (8, 8, 64, synth.F32, 5)])
def test_raw_entry_on_arbitrary_page_tables(Hq, Hkv, D, dtype, seed):
    """sym_pred_batch_raw with page tables that no allocator would produce: pages repeated within a
    table, identical tables, prefixes shared in whole or in part by some LIPs, ragged last pages,
    single tokens, drafts and chunks, against dense attention over the gathered pages."""
    from oracle.attention import gather_file, dense_attention
    from paper_2510_25412_amd.driver import to_device
    drv = _hip()
    shape = synth.Shape(Hq, Hkv, D, 16, dtype)
    NP = 400
    sess = drv.HipSession(shape, NP, max_lips=40, max_tokens=4096, max_entries=1 << 16, poison=True)
    osess = OracleSession(shape, NP)
    rng = np.random.default_rng(7000 + seed)

    def data(n, heads):
        x = rng.standard_normal((n, heads, D), dtype=np.float32)
        return synth.bf16_round(x) if dtype == synth.BF16 else x

    fill = ("append", 0, data(NP * 16, Hkv), data(NP * 16, Hkv))     # defined data in every page, on both sides
    for s in (sess, osess):
        s.setup([("open", 0)])
        s.setup([fill])
    assert sess.ctx.kv_pages(sess.h[0]) == list(range(NP))
    worst = 0.0
    for it in range(12):
        n_lips = int(rng.integers(1, 33))
        tables, lengths, nts = [], [], []
        prefixes = [rng.permutation(NP)[:int(rng.integers(2, 60))].tolist() for _ in range(3)]
        for b in range(n_lips):
            kind = rng.random()
            if kind < 0.45:                # one of the prefixes, whole or in part, then private pages (or none)
                pre = prefixes[int(rng.integers(3))]
                pre = pre[:int(rng.integers(1, len(pre) + 1))] if rng.random() < 0.3 else pre
                t = pre + rng.permutation(NP)[:int(rng.integers(0, 12))].tolist()
            elif kind < 0.55 and tables:   # the same table as another LIP
                t = list(tables[int(rng.integers(len(tables)))])
            else:                          # any pages, repeats allowed
                t = rng.integers(0, NP, size=int(rng.integers(1, 70))).tolist()
            nt = int(rng.choice([1, 1, 1, 1, 1, 2, 3, 4, 6, 17, 40]))
            if nt > len(t) * 16:
                nt = 1
            tables.append(t)
            lengths.append(int(rng.integers(max(nt, (len(t) - 1) * 16 + 1), len(t) * 16 + 1)))
            nts.append(nt)
        T = sum(nts)
        q = data(T, Hq)
        flat = np.concatenate(tables).astype(np.int32)
        off = np.concatenate([[0], np.cumsum([len(t) for t in tables])]).astype(np.int64)
        out = torch.empty((T, Hq, D), dtype=torch.float32, device=sess.device)
        sess.ctx.pred_batch_raw(nts, flat, off, lengths, to_device(q, sess.device), out, sess.stream)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        ref = np.empty_like(got, dtype=np.float64)
        row = 0
        for t, L, nt in zip(tables, lengths, nts):
            K, V = gather_file(osess.pool, t, L)
            ref[row:row + nt] = dense_attention(widen(q[row:row + nt]).astype(np.float64), widen(K).astype(np.float64),
                                                widen(V).astype(np.float64), L - nt, dtype=np.float64)
            row += nt
        worst = max(worst, check_outputs(got, ref))
    sess.close()
    print(f"raw entry, arbitrary tables {Hq}/{Hkv}: worst scaled error {worst:.2e}")


def test_two_contexts_on_two_threads_and_streams():
    """Two contexts driven at the same time from two host threads, each on a stream of its own
    (default priority): the library keeps no state outside a context, so both must produce what they
    produce alone (ctypes releases the interpreter lock during the calls, so the calls do overlap)."""
    import threading
    drv = _hip()
    wls = [synth.config2(n_lips=24, lo=100, hi=900, slack_pages=64),
           synth.config3(n_roots=3, n_children=6, prefix=400, suffix_hi=60, slack_pages=64)]
    refs = [run_oracle(wl, dtype=np.float64) for wl in wls]
    results, errors = [None, None], []

    def work(i):
        try:
            st = torch.cuda.Stream(device="cuda:0")
            with torch.cuda.stream(st):
                for rep in range(4):
                    got, sess = drv.run_workload(wls[i], poison=True)
                    results[i] = (got, [sess.pages(f) for f in sorted(sess.h)], sess.ctx.free_pages())
                    sess.close()
        except Exception as e:                      # reported by the main thread
            errors.append((i, repr(e)))

    print("[case] two contexts, two threads, two streams", flush=True)
    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
    assert not any(t.is_alive() for t in threads), "a worker thread did not finish"
    assert not errors, errors
    for i, (wl, (ref, osess)) in enumerate(zip(wls, refs)):
        got, pages, free = results[i]
        check_outputs(got, ref)
        assert pages == [osess.model.kv_pages(osess.h[f]) for f in sorted(osess.h)]
        assert free == osess.model.free_pages()


# ---- do these parity tests notice when the two sides differ? ------------------------------------
# A mistake is written into a COPY of the oracle's source (on the CPU; the kernels run unchanged),
# a few quick parity tests above are run against the copy, and at least one must fail: the
# comparisons are real ones, with a bar tight enough for a wrong scale, head mapping, mask, page
# choice or copy.
_QUICK = ["test_config1_tiny_fp32_all_outputs", "test_edge_cases", "test_chunk_equals_sequential_on_gpu", "test_prefill_chunk_equals_sequential",
          "test_copy_and_in_place_append_on_one_page_in_one_batch", "test_extract_of_very_few_tokens", "test_config4_mixed_reduced"]


def test_quick_parity_tests_pass_under_the_harness_without_a_mistake():
    from test_oracle_pins_have_teeth import _failing_pins
    assert _failing_pins("attention.py", [], ["test_gpu_parity.py"], only=_QUICK) == []


@pytest.mark.parametrize("module_file,what,edits", [
    ("attention.py", "scale dropped", [("@ K[:, g, :].T) * scale", "@ K[:, g, :].T)")]),
    ("attention.py", "heads interleaved instead of grouped", [("g = h // G", "g = h % Hkv")]),
    ("attention.py", "a token does not see itself", [("<= (len_before + np.arange(n))", "< (len_before + np.arange(n))")]),
    ("attention.py", "a token sees one token too many", [("<= (len_before + np.arange(n))", "<= (len_before + 1 + np.arange(n))")]),
    ("attention.py", "K and V swapped in the gather", [("K[lo:lo + n] = pg[0,", "K[lo:lo + n] = pg[1,"), ("V[lo:lo + n] = pg[1,", "V[lo:lo + n] = pg[0,")]),
    ("attention.py", "weighted sum of K", [("out[:, h, :] = p @ V[:, g, :]", "out[:, h, :] = p @ K[:, g, :]")]),
    ("kvfs_model.py", "highest rank first", [("heapq.heappop(self.free_ranks)", "self.free_ranks.pop(self.free_ranks.index(max(self.free_ranks)))")]),
    ("kvfs_model.py", "shared partial page written in place", [("if r != 0 and self.refcount[f.pages[-1]] > 1:", "if False:")]),
    ("kvfs_model.py", "copy takes one slot too few", [("cow.append((src, dst, r))", "cow.append((src, dst, r - 1))")]),
    ("kvfs_model.py", "copies after the appends", [("        for src, dst, r in cow:\n            self.copy_slots(src, dst, r)\n        t = 0\n", "        t = 0\n"),
                                                   ("        assert t == len(k_new)\n", "        assert t == len(k_new)\n        for src, dst, r in cow:\n            self.copy_slots(src, dst, r)\n")]),
    ("kvfs_model.py", "extract: nothing is ever shared", [("same = all(pg == toks[0][0] and sl == k for k, (pg, sl) in enumerate(toks))", "same = False")]),
    ("kvfs_model.py", "extract: destination slots shifted", [("moves.append((pg, sl, dst, k))", "moves.append((pg, sl, dst, (k + 1) % P))")]),
])
@pytest.mark.filterwarnings("ignore::RuntimeWarning")
def test_parity_tests_notice_a_wrong_oracle(module_file, what, edits):
    from test_oracle_pins_have_teeth import _failing_pins
    print(f"[case] oracle with a planted mistake: {what}", flush=True)
    failed = _failing_pins(module_file, edits, ["test_gpu_parity.py"], only=_QUICK, first=True)
    assert failed, f"no parity test notices an oracle with: {what}"

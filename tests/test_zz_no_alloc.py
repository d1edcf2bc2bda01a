"""The entry point that allocates nothing (sym_pred_batch_static) against sym_pred_batch, through
the C ABI: same outputs (to the parity bar; bit for bit where both build the same descriptor),
same page tables, on two calls in a row on one context, the second with a smaller input."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2510_25412_amd import synth

pytestmark = pytest.mark.gpu

TOL = 2e-3


def _session(wl):
    from paper_2510_25412_amd import driver
    entries = sum(wl.pages_after_batch().values()) + 64 * len(wl.batch_files)
    sess = driver.HipSession(wl.shape, wl.n_pages, wl.free_order, "cuda:0", max_lips=len(wl.batch_files),
                             max_tokens=max(int(sum(wl.batch_n)), max(wl.lengths.values())) + 64, max_entries=entries, poison=True)
    sess.setup(wl.setup_ops())
    return sess


def _sub_batch(batch, lips):
    """The pred calls of the LIPs `lips` of a batch, as a batch of their own."""
    starts = np.concatenate([[0], np.cumsum(batch["n_tokens"])])
    rows = np.concatenate([np.arange(starts[b], starts[b + 1]) for b in lips])
    return dict(files=[batch["files"][b] for b in lips], n_tokens=[batch["n_tokens"][b] for b in lips],
                q=batch["q"][rows], k_new=batch["k_new"][rows], v_new=batch["v_new"][rows])


def _pred(sess, batch, static):
    db = sess.upload_batch(batch)
    fn = sess.ctx.pred_batch_static if static else sess.ctx.pred_batch
    fn(db["kv"], db["n_tokens"], db["q"], db["k_new"], db["v_new"], db["out"], sess.stream)
    torch.cuda.synchronize()
    return db["out"].cpu().numpy()


def _compare(wl, calls, exact):
    """Two sessions with the same files; each call of `calls` (lists of LIP indices of the workload's batch) runs
    on one through sym_pred_batch and on the other through sym_pred_batch_static."""
    print(f"[case] no-alloc {wl.name} lips={len(wl.batch_files)} calls={[len(c) for c in calls]}", flush=True)
    ref_s, got_s = _session(wl), _session(wl)
    batch = wl.batch()
    for lips in calls:
        sub = _sub_batch(batch, lips)
        ref = _pred(ref_s, sub, False)
        got = _pred(got_s, sub, True)
        assert np.isfinite(got).all()
        if exact:
            assert np.array_equal(got, ref)
        err = float((np.abs(got - ref) / np.maximum(1.0, np.abs(ref))).max())
        assert err <= TOL, err
        for f in wl.batch_files:
            assert got_s.pages(f) == ref_s.pages(f)
            assert got_s.ctx.kv_len(got_s.h[f]) == ref_s.ctx.kv_len(ref_s.h[f])
        assert got_s.ctx.free_pages() == ref_s.ctx.free_pages()
    ref_s.close()
    got_s.close()


def test_static_entry_point_matches_pred_batch_twice_second_smaller():
    from paper_2510_25412_amd import binding
    assert binding.load().sym_static_scratch_bytes() == 64 << 20
    # forks that share a prefix (shared-prefix tiles + members' partials + merge): all 18 LIPs, then 7 of them
    # (the key chunks of the tiles depend on the partial slots at hand: equal to the bar, not bit for bit)
    wl = synth.config3(n_roots=3, n_children=6, prefix=640, slack_pages=64)
    _compare(wl, [list(range(18)), [0, 1, 2, 3, 4, 5, 9]], exact=False)
    # plain decode rows cut into ranges (partials + merge): 24 LIPs, then 5; the same descriptor on both paths
    wl = synth.config2(n_lips=24, lo=40, hi=2000, slack_pages=64)
    _compare(wl, [list(range(24)), [3, 4, 11, 17, 23]], exact=True)
    # a prefill chunk + decode rows, then the decode rows alone
    wl = synth.config4(n_prefill=2, n_decode=6, chunk=48, pre_hi=300, dec_lo=30, dec_hi=200, slack_pages=64)
    _compare(wl, [list(range(8)), [2, 3, 4]], exact=True)


def test_static_entry_point_refuses_what_does_not_fit_and_changes_nothing():
    from paper_2510_25412_amd import driver, binding
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    wl = synth.config2(n_lips=2, lo=20, hi=60, slack_pages=4200)
    sess = driver.HipSession(shape, wl.n_pages, None, "cuda:0", max_lips=2, max_tokens=1 << 20, max_entries=1 << 17)
    sess.setup(wl.setup_ops())
    h = sess.h[wl.batch_files[0]]
    before = (sess.ctx.kv_len(h), sess.ctx.kv_pages(h), sess.ctx.free_pages())
    T = 60000            # 21 words per new token: beyond the 1 Mi-word descriptor limit
    q = torch.zeros((T, 32, 128), dtype=torch.bfloat16, device="cuda")
    kn = torch.zeros((T, 8, 128), dtype=torch.bfloat16, device="cuda")
    out = torch.empty((T, 32, 128), dtype=torch.float32, device="cuda")
    with pytest.raises(binding.SymError) as ei:
        sess.ctx.pred_batch_static([h], [T], q, kn, kn, out, sess.stream)
    assert ei.value.code == binding.SYM_ENOSPC
    assert (sess.ctx.kv_len(h), sess.ctx.kv_pages(h), sess.ctx.free_pages()) == before
    sess.close()

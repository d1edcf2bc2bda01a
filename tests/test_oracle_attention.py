"""Pins for the oracle's attention (CPU only): brute force, closed forms, invariants and a
library routine, chosen so that a dropped term, a wrong sign/index or a transposed operand
in the oracle fails at least one of them."""
import math

import numpy as np
import pytest
import torch

from oracle.attention import dense_attention, gather_file, pred_batch
from oracle.kvfs_model import KVFSModel, PagePool
from oracle.driver import OracleSession, run_workload, widen
from paper_2510_25412_amd import synth


def _rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float32)


def brute_force(q, K, V, len_before):
    """Triple-loop float64 evaluation of the definition, written independently."""
    n, Hq, D = q.shape
    N, Hkv, _ = K.shape
    G = Hq // Hkv
    out = np.zeros((n, Hq, D))
    for i in range(n):
        vis = len_before + i + 1
        for h in range(Hq):
            g = h // G
            s = [sum(float(q[i, h, d]) * float(K[j, g, d]) for d in range(D)) / math.sqrt(D) for j in range(vis)]
            mx = max(s)
            w = [math.exp(x - mx) for x in s]
            z = sum(w)
            for d in range(D):
                out[i, h, d] = sum(w[j] * float(V[j, g, d]) for j in range(vis)) / z
    return out


@pytest.mark.parametrize("n,L,Hq,Hkv,D", [(1, 0, 2, 2, 4), (1, 39, 4, 2, 8), (3, 17, 6, 3, 8), (5, 0, 4, 1, 4)])
def test_brute_force(n, L, Hq, Hkv, D):
    rng = np.random.default_rng(n * 100 + L)
    q, K, V = _rand(rng, n, Hq, D), _rand(rng, L + n, Hkv, D), _rand(rng, L + n, Hkv, D)
    ref = brute_force(q, K, V, L)
    assert np.abs(dense_attention(q, K, V, L, dtype=np.float64) - ref).max() <= 1e-12
    assert np.abs(dense_attention(q, K, V, L, dtype=np.float32) - ref).max() <= 1e-6


def test_rows_sum_to_one_and_causal_zeroes():
    rng = np.random.default_rng(3)
    q, K, V = _rand(rng, 4, 8, 16), _rand(rng, 24, 2, 16), _rand(rng, 24, 2, 16)
    _, p = dense_attention(q, K, V, 20, return_probs=True)
    assert np.abs(p.sum(axis=-1) - 1).max() <= 1e-6
    for i in range(4):
        assert np.all(p[i, :, 20 + i + 1:] == 0) and np.all(p[i, :, :20 + i + 1] > 0)


def test_closed_forms():
    rng = np.random.default_rng(11)
    Hq, Hkv, D, N = 8, 2, 16, 50
    q, K, V = _rand(rng, 1, Hq, D), _rand(rng, N, Hkv, D), _rand(rng, N, Hkv, D)
    G = Hq // Hkv
    # (i) zero query -> plain mean of V per kv head
    o = dense_attention(np.zeros_like(q), K, V, N - 1, dtype=np.float64)
    for h in range(Hq):
        assert np.abs(o[0, h] - V[:, h // G].astype(np.float64).mean(axis=0)).max() <= 1e-12
    # (i') all K rows equal -> mean again
    o = dense_attention(q, np.repeat(K[:1], N, axis=0), V, N - 1, dtype=np.float64)
    assert np.abs(o[0, 3] - V[:, 3 // G].astype(np.float64).mean(axis=0)).max() <= 1e-12
    # (ii) constant V -> that constant
    c = _rand(rng, 1, Hkv, D)
    o = dense_attention(q, K, np.repeat(c, N, axis=0), N - 1, dtype=np.float64)
    for h in range(Hq):
        assert np.abs(o[0, h] - c[0, h // G]).max() <= 1e-12
    # (iii) single visible token -> its V row (empty file + one new token)
    o = dense_attention(q, K[:1], V[:1], 0)
    for h in range(Hq):
        assert np.array_equal(o[0, h], V[0, h // G])
    # (iv) one key aligned with q and scaled huge -> that token's V row
    K2 = K.copy()
    for g in range(Hkv):
        K2[7, g] = 1e4 * q[0, g * G] / np.linalg.norm(q[0, g * G])
    o = dense_attention(q, K2, V, N - 1, dtype=np.float64)
    assert np.abs(o[0, 0] - V[7, 0]).max() <= 1e-9 and np.abs(o[0, G] - V[7, 1]).max() <= 1e-9
    # (v) shifting every key by u changes all scores by q.u, which softmax ignores
    u = _rand(rng, 1, Hkv, D)
    a = dense_attention(q, K, V, N - 1, dtype=np.float64)
    b = dense_attention(q, K.astype(np.float64) + u, V, N - 1, dtype=np.float64)   # shift applied exactly
    assert np.abs(a - b).max() <= 1e-9
    # (vi) two tokens, known logits: weights are the logistic function of the score gap
    q1 = np.zeros((1, 1, 4), np.float32); q1[0, 0, 0] = 2.0
    K1 = np.zeros((2, 1, 4), np.float32); K1[0, 0, 0] = 1.0; K1[1, 0, 0] = -1.0
    V1 = np.zeros((2, 1, 4), np.float32); V1[0, 0, 1] = 1.0; V1[1, 0, 2] = 1.0
    o = dense_attention(q1, K1, V1, 1, dtype=np.float64)      # scores +1, -1 after the 1/sqrt(4) scale
    w0 = 1 / (1 + math.exp(-2.0))
    assert abs(o[0, 0, 1] - w0) <= 1e-12 and abs(o[0, 0, 2] - (1 - w0)) <= 1e-12


def test_gqa_mapping_is_consecutive_groups():
    """Query head h reads kv head h // G: making kv head 1 special must move heads G..2G-1 only."""
    rng = np.random.default_rng(5)
    Hq, Hkv, D, N = 8, 4, 8, 12
    q, K, V = _rand(rng, 1, Hq, D), _rand(rng, N, Hkv, D), _rand(rng, N, Hkv, D)
    a = dense_attention(q, K, V, N - 1)
    V2 = V.copy(); V2[:, 1] += 1.0
    b = dense_attention(q, K, V2, N - 1)
    changed = [h for h in range(Hq) if not np.array_equal(a[0, h], b[0, h])]
    assert changed == [2, 3]
    assert np.abs((b - a)[0, 2:4] - 1.0).max() <= 1e-5


def test_library_special_case_sdpa():
    """torch's scaled_dot_product_attention with KV heads repeated and an explicit mask."""
    rng = np.random.default_rng(9)
    n, L, Hq, Hkv, D = 6, 45, 8, 2, 32
    q, K, V = _rand(rng, n, Hq, D), _rand(rng, L + n, Hkv, D), _rand(rng, L + n, Hkv, D)
    G = Hq // Hkv
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)[None]
    mask = torch.arange(L + n)[None, :] <= (L + torch.arange(n))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    assert np.abs(dense_attention(q, K, V, L) - ref).max() <= 1e-5


def test_contiguous_equals_paged_bit_identical():
    """Gathering a file's pages gives back exactly the rows that were appended, so attention
    on the gathered arrays is bit-identical to attention on the original contiguous arrays,
    for any page placement."""
    rng = np.random.default_rng(21)
    Hq, Hkv, D, P = 4, 2, 8, 4
    for order in (None, rng.permutation(32)):
        m = KVFSModel(32, P, order)
        pool = PagePool(Hkv, P, D)
        h = m.kv_open()
        K, V = _rand(rng, 23, Hkv, D), _rand(rng, 23, Hkv, D)
        for lo, hi in ((0, 5), (5, 6), (6, 23)):          # appended in ragged pieces
            cow, slots = m.append([(h, hi - lo)])
            pool.apply(cow, slots, K[lo:hi], V[lo:hi])
        Kg, Vg = gather_file(pool, m.kv_pages(h), 23)
        assert np.array_equal(Kg, K) and np.array_equal(Vg, V)
        q = _rand(rng, 1, Hq, D)
        assert np.array_equal(dense_attention(q, Kg, Vg, 22), dense_attention(q, K, V, 22))


def test_fork_cow_append_invariance():
    """Outputs of forked files equal those of deep-copied unforked files, bit for bit; the
    parent is unchanged by child activity.  Prefix 22 on pages of 4 forces a page copy."""
    shape = synth.Shape(4, 2, 8, 4, synth.F32)
    forked = synth.custom("forked", shape, [("new", 22), ("fork", 0, 0), ("fork", 0, 5), ("fork", 0, 9)],
                          [(1, 1), (2, 1), (3, 2), (0, 1)], 64, seed=77)
    out_f, s_f = run_workload(forked)
    assert s_f.model.cow_copies == 3
    # unforked twin: every child is its own file holding prefix + private suffix
    ops = list(forked.setup_ops())
    prefixKV = ops[1][2], ops[1][3]
    s_u = OracleSession(shape, 64)
    app = {op[1]: (op[2], op[3]) for op in ops if op[0] == "append"}
    for fid in range(4):
        s_u.setup([("open", fid), ("append", fid, prefixKV[0], prefixKV[1])])
        if fid != 0 and fid in app:
            s_u.setup([("append", fid, app[fid][0], app[fid][1])])
    out_u = s_u.pred(forked.batch())
    assert np.array_equal(out_f, out_u)
    assert s_u.model.cow_copies == 0
    # parent content untouched by the children: its gathered prefix is still the original
    Kp, _ = gather_file(s_f.pool, s_f.model.kv_pages(s_f.h[0]), 22)
    assert np.array_equal(Kp, prefixKV[0])
    s_f.model.audit()


@pytest.mark.parametrize("how", ["truncate", "extract"])
def test_a_copy_takes_the_page_as_it_was_before_the_batch(how):
    """One batch in which a page is both copied and appended to in place: file A (6 tokens, pages of
    4) shares its partly filled page with a file B that sees only ONE token of it (a fork truncated
    to 5 tokens, or an extract of the first 5).  A appends first and copies slots 0 and 1 away; B, now
    alone on the page, appends into slot 1.  A must keep ITS token 5 in slot 1 of the copy, whatever B
    wrote there: every file reads back exactly the rows that were appended to it (section 4.2: a fork
    shares tensors, it never lets one file's writes show in another)."""
    rng = np.random.default_rng(21)
    Hkv, D, P = 2, 4, 4
    m, pool = KVFSModel(16, P), PagePool(Hkv, P, D)
    rows = {}                                           # file handle -> the K rows it must hold

    def append(items):
        k = [_rand(rng, n, Hkv, D) for _, n in items]
        v = [_rand(rng, n, Hkv, D) for _, n in items]
        cow, slots = m.append(items)
        pool.apply(cow, slots, np.concatenate(k), np.concatenate(v))
        for (h, _), kk in zip(items, k):
            rows[h] = np.concatenate([rows[h], kk]) if h in rows else kk
        return cow

    a = m.kv_open()
    append([(a, 6)])
    if how == "truncate":
        b = m.kv_fork(a)
        m.kv_truncate(b, 5)
    else:
        b, moves = m.kv_extract(a, list(range(5)))
        assert moves == []                              # slots 0.. of existing pages: referenced, not copied
    rows[b] = rows[a][:5]
    assert m.kv_pages(a) == m.kv_pages(b) and m.refcount[m.kv_pages(a)[1]] == 2
    shared = m.kv_pages(a)[1]
    cow = append([(a, 1), (b, 2)])
    assert cow == [(shared, m.kv_pages(a)[1], 2)] and m.kv_pages(b)[1] == shared    # A copied two slots, B stayed
    for h in (a, b):
        K, _ = gather_file(pool, m.kv_pages(h), m.kv_len(h))
        assert np.array_equal(K, rows[h]), "file %d does not read back what was appended to it" % h
    m.audit()


def test_sampled_outputs_equal_the_full_run():
    """The full-size GPU tests ask the oracle for the outputs of a few LIPs of a batch only: those
    rows must be the rows of the full run, bit for bit, every other row NaN, and the file-system state
    the same (the append is carried out for every LIP either way)."""
    shape = synth.Shape(4, 2, 8, 4, synth.BF16)
    wl = synth.custom("sampled", shape, [("new", 9), ("new", 0), ("fork", 0, 3), ("new", 30), ("fork", 3, 0)],
                      [(0, 1), (1, 5), (2, 2), (3, 1), (4, 7)], 64, seed=5)
    full, s_full = run_workload(wl)
    part, s_part = run_workload(wl, only=[1, 4, 2])
    starts = np.concatenate([[0], np.cumsum([1, 5, 2, 1, 7])])
    for b in range(5):
        rows = slice(starts[b], starts[b + 1])
        if b in (1, 2, 4):
            assert np.array_equal(part[rows], full[rows]), b
        else:
            assert np.isnan(part[rows]).all(), b
    assert not np.isnan(full).any()
    for f in range(5):
        assert s_part.model.kv_pages(s_part.h[f]) == s_full.model.kv_pages(s_full.h[f])
    assert np.array_equal(s_part.model.refcount, s_full.model.refcount)


def test_chunk_equals_sequential():
    """One n-token pred equals n one-token preds (pins the in-chunk causal mask and the
    append order)."""
    rng = np.random.default_rng(31)
    Hq, Hkv, D, P, L, n = 4, 2, 8, 4, 10, 7
    K0, V0 = _rand(rng, L, Hkv, D), _rand(rng, L, Hkv, D)
    q, kn, vn = _rand(rng, n, Hq, D), _rand(rng, n, Hkv, D), _rand(rng, n, Hkv, D)

    def fresh():
        m, pool = KVFSModel(16, P), PagePool(Hkv, P, D)
        h = m.kv_open()
        cow, slots = m.append([(h, L)])
        pool.apply(cow, slots, K0, V0)
        return m, pool, h
    m, pool, h = fresh()
    chunk = pred_batch(m, pool, [h], [n], q, kn, vn)
    m2, pool2, h2 = fresh()
    seq = np.concatenate([pred_batch(m2, pool2, [h2], [1], q[i:i + 1], kn[i:i + 1], vn[i:i + 1]) for i in range(n)])
    assert np.abs(chunk - seq).max() <= 1e-6
    assert m.kv_pages(h) == m2.kv_pages(h2) and m.kv_len(h) == L + n


def test_token_permutation_invariance():
    rng = np.random.default_rng(41)
    q, K, V = _rand(rng, 1, 4, 8), _rand(rng, 30, 2, 8), _rand(rng, 30, 2, 8)
    perm = rng.permutation(30)
    a = dense_attention(q, K, V, 29, dtype=np.float64)
    b = dense_attention(q, K[perm], V[perm], 29, dtype=np.float64)
    assert np.abs(a - b).max() <= 1e-12


def test_split_merge_identity():
    """Log-sum-exp merge of partial results over any partition of the keys equals the
    unsplit result (the identity the GPU's split over pages relies on)."""
    rng = np.random.default_rng(51)
    D, N = 8, 57
    q, K, V = _rand(rng, 1, 1, D), _rand(rng, N, 1, D), _rand(rng, N, 1, D)
    full = dense_attention(q, K, V, N - 1, dtype=np.float64)[0, 0]
    cuts = [0, 3, 4, 30, 57]
    m_i, l_i, acc_i = [], [], []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        s = (K[lo:hi, 0].astype(np.float64) @ q[0, 0].astype(np.float64)) / math.sqrt(D)
        m_i.append(s.max()); e = np.exp(s - s.max()); l_i.append(e.sum()); acc_i.append(e @ V[lo:hi, 0].astype(np.float64))
    M = max(m_i)
    l = sum(li * math.exp(mi - M) for li, mi in zip(l_i, m_i))
    o = sum(ai * math.exp(mi - M) for ai, mi in zip(acc_i, m_i)) / l
    assert np.abs(o - full).max() <= 1e-12


def test_fp32_oracle_close_to_fp64():
    wl = synth.config1()
    a, _ = run_workload(wl, dtype=np.float32)
    b, _ = run_workload(wl, dtype=np.float64)
    assert np.abs(a - b).max() <= 2e-6


def test_bf16_rounding_matches_torch():
    x = np.random.default_rng(1).standard_normal(100000).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -0.0, 3.0e-39]      # exact ties (round to even) and tiny values
    ours = synth.bf16_round(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, ref)
    assert np.array_equal(widen(ours), torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    assert np.array_equal(synth.to_f32(ours), widen(ours))


def test_workload_shapes():
    wl = synth.config1()
    assert [wl.lengths[f] for f in wl.batch_files] == [37, 80, 129, 200]
    wl2 = synth.config2()
    L = np.array([wl2.lengths[f] for f in wl2.batch_files])
    assert len(L) == 64 and L.min() >= 512 and L.max() <= 4096
    b1, b2 = synth.config1().batch(), synth.config1().batch()
    assert np.array_equal(b1["q"], b2["q"]) and np.array_equal(b1["k_new"], b2["k_new"])


def test_pred_on_extracted_and_merged_files_equals_dense_on_indexed_arrays():
    """extract / merge (section 4.2) defined on plain arrays: the new file's K/V are the source
    rows indexed (or concatenated) with numpy, and a pred on the new file is dense attention on
    those arrays plus the new row, bit for bit; the sources still read as before."""
    rng = np.random.default_rng(5)
    Hq, Hkv, D, P = 4, 2, 8, 4
    sess = OracleSession(synth.Shape(Hq, Hkv, D, P, synth.F32), 64, rng.permutation(64))
    Ka, Va = _rand(rng, 23, Hkv, D), _rand(rng, 23, Hkv, D)
    Kb, Vb = _rand(rng, 10, Hkv, D), _rand(rng, 10, Hkv, D)
    idx = [0, 1, 2, 3, 9, 8, 20, 21, 22, 5, 5]
    sess.setup([("open", 0), ("append", 0, Ka, Va), ("open", 1), ("append", 1, Kb, Vb),
                ("extract", 2, 0, idx), ("merge", 3, [1, 0, 1]), ("extract", 4, 0, list(range(23)))])
    expect = {2: (Ka[idx], Va[idx]), 3: (np.concatenate([Kb, Ka, Kb]), np.concatenate([Vb, Va, Vb])), 4: (Ka, Va),
              0: (Ka, Va), 1: (Kb, Vb)}
    for fid, (K, V) in expect.items():
        Kg, Vg = gather_file(sess.pool, sess.model.kv_pages(sess.h[fid]), len(K))
        assert np.array_equal(Kg, K) and np.array_equal(Vg, V), fid
    files = [2, 3, 4, 0]
    q, kn, vn = _rand(rng, 4, Hq, D), _rand(rng, 4, Hkv, D), _rand(rng, 4, Hkv, D)
    out = sess.pred(dict(files=files, n_tokens=[1] * 4, q=q, k_new=kn, v_new=vn))
    for i, fid in enumerate(files):
        K, V = expect[fid]
        ref = dense_attention(q[i:i + 1], np.concatenate([K, kn[i:i + 1]]), np.concatenate([V, vn[i:i + 1]]), len(K))
        assert np.array_equal(out[i:i + 1], ref), fid
    # file 4 shared every page with file 0: both appended into the partly filled last page, one of them a copy
    assert sess.model.cow_copies == 1
    Kg, _ = gather_file(sess.pool, sess.model.kv_pages(sess.h[0]), 24)
    assert np.array_equal(Kg[:23], Ka) and np.array_equal(Kg[23], kn[3])
    sess.model.audit()

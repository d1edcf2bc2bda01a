"""Attention of one layer over paged KV files (test infrastructure, CPU only).

What `pred` (paper section 4.1) computes on this path: after the call's new tokens are
appended to the file, every new token i of LIP b gets, for every query head h,
    O[b,i,h,:] = softmax_j(scale * q[b,i,h,:] . K_b[j,g,:]) . V_b[j,g,:],  j = 0 .. L_b+i,
with g = h // (Hq/Hkv) and scale = 1/sqrt(D): the token sees the whole existing file and
the new tokens up to itself.  The pages of the file are first gathered into contiguous
[N, Hkv, D] arrays (KVFS keeps token-level K/V in pages, section 4.2); then the formula
is evaluated as written: all scores, max, exponentials, sum, divide, weighted sum.  No
running softmax, no splitting of the key range, no blocking.
"""
import numpy as np


def gather_file(pool, page_ids, length):
    """Contiguous K, V [length, Hkv, D] of a file from its page list."""
    P = pool.shape[2]
    K = np.empty((length, pool.shape[1], pool.shape[3]), pool.dtype)
    V = np.empty_like(K)
    for idx, p in enumerate(page_ids):
        lo = idx * P
        n = min(P, length - lo)
        if n <= 0:
            break
        pg = pool.page(p)
        K[lo:lo + n] = pg[0, :, :n, :].transpose(1, 0, 2)
        V[lo:lo + n] = pg[1, :, :n, :].transpose(1, 0, 2)
    return K, V


def dense_attention(q, K, V, len_before, scale=None, dtype=np.float32, return_probs=False):
    """q [n, Hq, D]; K, V [N, Hkv, D] with N = len_before + n (new tokens included).
    Returns O [n, Hq, D] in `dtype`; row i attends to tokens 0 .. len_before+i."""
    n, Hq, D = q.shape
    N, Hkv, _ = K.shape
    assert N == len_before + n and Hq % Hkv == 0
    G = Hq // Hkv
    scale = dtype(1.0 / np.sqrt(D)) if scale is None else dtype(scale)
    q = q.astype(dtype)
    K = K.astype(dtype)
    V = V.astype(dtype)
    out = np.empty((n, Hq, D), dtype)
    probs = []
    for h in range(Hq):
        g = h // G
        s = (q[:, h, :] @ K[:, g, :].T) * scale                       # [n, N]
        visible = np.arange(N)[None, :] <= (len_before + np.arange(n))[:, None]
        s = np.where(visible, s, dtype(-np.inf))
        e = np.exp(s - s.max(axis=1, keepdims=True))
        p = e / e.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ V[:, g, :]
        if return_probs:
            probs.append(p)
    if return_probs:
        return out, np.stack(probs, axis=1)                            # [n, Hq, N]
    return out


def pred_batch(model, pool, handles, n_tokens, q, k_new, v_new, dtype=np.float32):
    """The attention part of one batched `pred`: append every LIP's new K/V rows to its
    file (allocation and copy-on-write per the state model), then attend.
    q [T, Hq, D], k_new/v_new [T, Hkv, D] with T = sum(n_tokens), LIPs in batch order.
    Returns O [T, Hq, D]."""
    items = [(h, int(n)) for h, n in zip(handles, n_tokens)]
    before = [model.kv_len(h) for h, _ in items]
    cow, slots = model.append(items)
    pool.apply(cow, slots, k_new, v_new)
    out = np.empty(q.shape, dtype)
    t = 0
    for (h, n), L in zip(items, before):
        K, V = gather_file(pool, model.kv_pages(h), L + n)
        out[t:t + n] = dense_attention(q[t:t + n], K, V, L, dtype=dtype)
        t += n
    return out

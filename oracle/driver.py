"""Runs a synthetic workload (any object with .shape, .n_pages, .free_order, .setup_ops()
and .batch()) through the oracle.  Test infrastructure, CPU only."""
import numpy as np

from .kvfs_model import KVFSModel, PagePool
from .attention import pred_batch


def widen(a):
    """Stored patterns -> float32 values: bf16 bit patterns (uint16) become the high half
    of a float32 word, which is exact; float32 passes through."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return np.asarray(a, np.float32)


class OracleSession:
    """File ids of the workload -> handles of a KVFSModel plus the page contents."""

    def __init__(self, shape, n_pages, free_order=None):
        self.model = KVFSModel(n_pages, shape.page_tokens, free_order)
        self.pool = PagePool(shape.n_kv_heads, shape.page_tokens, shape.head_dim)
        self.h = {}

    def setup(self, ops):
        for op in ops:
            if op[0] == "open":
                self.h[op[1]] = self.model.kv_open(None)
            elif op[0] == "fork":
                self.h[op[1]] = self.model.kv_fork(self.h[op[2]])
            elif op[0] == "append":
                _, fid, K, V = op
                cow, slots = self.model.append([(self.h[fid], len(K))])
                self.pool.apply(cow, slots, widen(K), widen(V))
            elif op[0] == "remove":
                self.model.kv_remove(self.h.pop(op[1]))
            elif op[0] == "extract":                      # ("extract", new fid, source fid, token indices)
                self.h[op[1]], moves = self.model.kv_extract(self.h[op[2]], op[3])
                self.pool.move_tokens(moves)
            elif op[0] == "merge":                        # ("merge", new fid, [source fids])
                self.h[op[1]], moves = self.model.kv_merge([self.h[f] for f in op[2]])
                self.pool.move_tokens(moves)
            elif op[0] == "offload":                      # ("offload", [fids]) / ("restore", [fids])
                self.pool.swap_out(self.model.kv_offload([self.h[f] for f in op[1]]))
            elif op[0] == "restore":
                self.pool.swap_in(self.model.kv_restore([self.h[f] for f in op[1]]))
            else:
                raise ValueError(op[0])

    def pred(self, batch, dtype=np.float32, only=None):
        """Runs the batch.  `only` = indices of batch entries whose outputs are wanted
        (the append is always carried out for all); others are returned as NaN rows."""
        handles = [self.h[f] for f in batch["files"]]
        q, k, v = widen(batch["q"]), widen(batch["k_new"]), widen(batch["v_new"])
        if only is None:
            return pred_batch(self.model, self.pool, handles, batch["n_tokens"], q, k, v, dtype=dtype)
        from .attention import gather_file, dense_attention
        items = [(h, int(n)) for h, n in zip(handles, batch["n_tokens"])]
        before = [self.model.kv_len(h) for h, _ in items]
        cow, slots = self.model.append(items)
        self.pool.apply(cow, slots, k, v)
        out = np.full(q.shape, np.nan, dtype)
        starts = np.concatenate([[0], np.cumsum(batch["n_tokens"])])
        for b in only:
            h, n = items[b]
            K, V = gather_file(self.pool, self.model.kv_pages(h), before[b] + n)
            out[starts[b]:starts[b] + n] = dense_attention(q[starts[b]:starts[b] + n], K, V, before[b], dtype=dtype)
        return out


def run_workload(wl, dtype=np.float32, only=None):
    s = OracleSession(wl.shape, wl.n_pages, wl.free_order)
    s.setup(wl.setup_ops())
    out = s.pred(wl.batch(), dtype=dtype, only=only)
    return out, s

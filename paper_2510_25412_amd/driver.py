"""Runs a synthetic workload (synth.Workload) through the HIP library on one GPU.  torch is
used for device memory and the stream only; every step of the path runs in the library."""
import numpy as np
import torch

from . import binding, synth


def to_device(a, device):
    """Stored patterns (uint16 bf16 bits or float32) -> device tensor of the storage dtype."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)


class HipSession:
    """Device pool + workspace + library context for one workload shape.  n_layers > 1: the pool holds that many
    layers of every page; setup() appends the same rows to every layer unless an op carries rows per layer."""

    def __init__(self, shape, n_pages, free_order=None, device="cuda:0", max_lips=4096, max_tokens=1 << 16,
                 max_entries=1 << 21, decode_waves=0, poison=False, n_layers=1, tuning=None):
        self.shape = shape
        self.n_layers = n_layers
        self.device = torch.device(device)
        cfg = binding.make_config(shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.page_tokens, shape.dtype, n_pages,
                                  device=self.device.index or 0, free_order=free_order, decode_waves=decode_waves, n_layers=n_layers,
                                  tuning=tuning)
        pb = binding.page_bytes(cfg)
        assert pb > 0, "unsupported shape"
        self.page_bytes = pb
        wb = binding.workspace_bytes(cfg, max_lips, max_tokens, max_entries)
        self.pool = torch.empty(n_layers * n_pages * pb, dtype=torch.uint8, device=self.device)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.device)
        if poison:          # every never-written slot reads as NaN (tests: stale slots must not leak)
            self.pool.fill_(0xFF)
        cfg.pool, cfg.workspace, cfg.workspace_bytes = self.pool.data_ptr(), self.workspace.data_ptr(), wb
        self.ctx = binding.Context(cfg)
        self.h = {}

    @property
    def stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    def setup(self, ops):
        for op in ops:
            if op[0] == "open":
                self.h[op[1]] = self.ctx.kv_open(None)
            elif op[0] == "fork":
                self.h[op[1]] = self.ctx.kv_fork(self.h[op[2]])
            elif op[0] == "append":
                _, fid, K, V = op
                n = K.shape[-3]
                k, v = to_device(K, self.device), to_device(V, self.device)
                if self.n_layers > 1 and K.ndim == 3:          # the same rows for every layer
                    k, v = k.expand(self.n_layers, *k.shape).contiguous(), v.expand(self.n_layers, *v.shape).contiguous()
                self.ctx.kv_append(self.h[fid], n, k, v, self.stream)
                torch.cuda.current_stream(self.device).synchronize()   # k, v are freed on return
            elif op[0] == "remove":
                self.ctx.kv_remove(self.h.pop(op[1]))
            elif op[0] == "extract":                      # ("extract", new fid, source fid, token indices)
                self.h[op[1]] = self.ctx.kv_extract(self.h[op[2]], op[3], self.stream)
            elif op[0] == "merge":                        # ("merge", new fid, [source fids])
                self.h[op[1]] = self.ctx.kv_merge([self.h[f] for f in op[2]], self.stream)
            elif op[0] == "offload":                      # ("offload", [fids]) / ("restore", [fids])
                self.ctx.kv_offload([self.h[f] for f in op[1]], self.stream)
            elif op[0] == "restore":
                self.ctx.kv_restore([self.h[f] for f in op[1]], self.stream)
            else:
                raise ValueError(op[0])

    def upload_batch(self, batch):
        T = int(sum(batch["n_tokens"]))
        s = self.shape
        return dict(kv=[self.h[f] for f in batch["files"]], n_tokens=list(batch["n_tokens"]),
                    q=to_device(batch["q"], self.device), k_new=to_device(batch["k_new"], self.device),
                    v_new=to_device(batch["v_new"], self.device),
                    out=torch.empty((T, s.n_q_heads, s.head_dim), dtype=torch.float32, device=self.device))

    def pred(self, dev_batch):
        self.ctx.pred_batch(dev_batch["kv"], dev_batch["n_tokens"], dev_batch["q"], dev_batch["k_new"], dev_batch["v_new"],
                            dev_batch["out"], self.stream)
        return dev_batch["out"]

    def pages(self, fid):
        return self.ctx.kv_pages(self.h[fid])

    def close(self):
        torch.cuda.synchronize(self.device)
        self.ctx.close()


def run_workload(wl, device="cuda:0", **kw):
    """Builds the files, runs the batch once; returns (outputs as float32 numpy, session)."""
    entries = sum(wl.pages_after_batch().values()) + 64
    sess = HipSession(wl.shape, wl.n_pages, wl.free_order, device, max_lips=max(len(wl.batch_files), 1),
                      max_tokens=max(int(sum(wl.batch_n)), max(wl.lengths.values(), default=1), 1) + 64,
                      max_entries=entries, **kw)
    sess.setup(wl.setup_ops())
    db = sess.upload_batch(wl.batch())
    out = sess.pred(db)
    torch.cuda.synchronize(sess.device)
    return out.cpu().numpy(), sess

"""ctypes binding of libsymphony_kv.so: same names as the C ABI (include/symphony_kv.h),
argument marshalling only.  torch supplies device memory and streams; nothing is computed
here.  Loading fails loudly if the library has not been built: there is no fallback.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# SYMPHONY_KV_LIB: another build of the same library (the host-only sanitizer builds of the CPU tests)
LIB_PATH = os.environ.get("SYMPHONY_KV_LIB") or os.path.join(_HERE, "libsymphony_kv.so")

SYM_OK, SYM_EINVAL, SYM_EBADF, SYM_ENOSPC, SYM_ENOENT, SYM_EEXIST, SYM_EBUSY, SYM_EHIP = 0, -1, -2, -3, -4, -5, -6, -7
SYM_F32, SYM_BF16 = 0, 1
K_PROLOGUE, K_ATTN, K_MERGE, K_MOVE, K_SWAP = 0, 1, 2, 3, 4


TUNING_FIELDS = ("decode_mfma", "min_units", "prefill_min", "share_min_lips", "share_min_pages", "tile_rows",
                 "row_tokens", "range_cost", "bin_tolerance", "bin_waves", "fuse_append", "mix_lead", "mix_spread", "share_tiles")


class SymTuning(C.Structure):
    _fields_ = [(n, C.c_int32) for n in TUNING_FIELDS]


class SymConfig(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_tokens", C.c_int32), ("dtype", C.c_int32), ("device", C.c_int32),
                ("n_pages", C.c_int64), ("pool", C.c_void_p), ("workspace", C.c_void_p),
                ("workspace_bytes", C.c_int64), ("free_order", C.POINTER(C.c_int32)),
                ("softmax_scale", C.c_float), ("decode_waves", C.c_int32), ("n_layers", C.c_int32),
                ("tuning", C.POINTER(SymTuning))]


class SymStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("pages_total", "pages_free", "pages_shared", "cow_copies", "pages_allocated",
                                         "tokens_appended", "pred_batches", "kernel_launches", "files", "handles",
                                         "host_ns_plan", "host_ns_pred", "tokens_moved", "pages_referenced",
                                         "pages_offloaded", "pages_restored", "host_slots", "last_batch_tiles",
                                         "last_batch_shared_rows")]


class SymError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"symphony_kv error {code}: {msg}")
        self.code = code


_lib = None
_I32P, _I64P = C.POINTER(C.c_int32), C.POINTER(C.c_int64)

_SIGNATURES = {
    "sym_page_bytes": (C.c_int64, [C.POINTER(SymConfig)]),
    "sym_tuning_defaults": (C.c_int, [C.POINTER(SymConfig), C.POINTER(SymTuning)]),
    "sym_workspace_bytes": (C.c_int64, [C.POINTER(SymConfig), C.c_int64, C.c_int64, C.c_int64]),
    "sym_init": (C.c_int, [C.POINTER(SymConfig), C.POINTER(C.c_void_p)]),
    "sym_destroy": (None, [C.c_void_p]),
    "sym_strerror": (C.c_char_p, [C.c_void_p]),
    "sym_kv_open": (C.c_int32, [C.c_void_p, C.c_char_p]),
    "sym_kv_fork": (C.c_int32, [C.c_void_p, C.c_int32]),
    "sym_kv_remove": (C.c_int, [C.c_void_p, C.c_int32]),
    "sym_kv_close": (C.c_int, [C.c_void_p, C.c_int32]),
    "sym_kv_len": (C.c_int64, [C.c_void_p, C.c_int32]),
    "sym_kv_truncate": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I64P]),
    "sym_kv_append": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_kv_extract": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I64P, _I64P, _I32P, C.c_void_p]),
    "sym_kv_merge": (C.c_int32, [C.c_void_p, C.c_int32, _I32P, C.c_void_p]),
    "sym_last_moves": (C.c_int64, [C.c_void_p, _I32P, C.c_int64]),
    "sym_kv_offload": (C.c_int, [C.c_void_p, C.c_int32, _I32P, C.c_void_p]),
    "sym_kv_restore": (C.c_int, [C.c_void_p, C.c_int32, _I32P, C.c_void_p]),
    "sym_kv_waiting": (C.c_int, [C.c_void_p, C.c_int32]),
    "sym_last_swaps": (C.c_int64, [C.c_void_p, _I32P, C.c_int64]),
    "sym_pred_batch": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_pred_batch_static": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_static_scratch_bytes": (C.c_int64, []),
    "sym_test_fail_staging": (C.c_int, [C.c_void_p, C.c_int32]),
    "sym_pred_begin": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, C.c_void_p]),
    "sym_pred_layer": (C.c_int, [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_pred_end": (C.c_int, [C.c_void_p]),
    "sym_kv_read_layer": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_pred_batch_raw": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, _I64P, _I64P, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_kv_pages": (C.c_int64, [C.c_void_p, C.c_int32, _I32P, C.c_int64]),
    "sym_page_refcount": (C.c_int32, [C.c_void_p, C.c_int32]),
    "sym_free_pages": (C.c_int64, [C.c_void_p]),
    "sym_get_stats": (C.c_int, [C.c_void_p, C.POINTER(SymStats)]),
    "sym_plan_append": (C.c_int, [C.c_void_p, C.c_int32, _I32P, _I32P, _I32P, C.c_int64, _I32P, _I32P]),
    "sym_plan_copies_first": (C.c_int, [C.c_void_p]),
    "sym_build_desc": (C.c_int64, [C.c_void_p, C.c_int32, _I32P, _I32P, _I64P, _I64P, _I32P, C.c_int64]),
    "sym_kv_read": (C.c_int, [C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]),
    "sym_sched_create": (C.c_void_p, [C.c_int32, C.c_double, C.c_double, C.c_double, C.c_double]),
    "sym_sched_destroy": (None, [C.c_void_p]),
    "sym_sched_arrive": (None, [C.c_void_p, C.c_double]),
    "sym_sched_decide": (C.c_int32, [C.c_void_p, C.c_double, C.c_int]),
    "sym_sched_fired": (None, [C.c_void_p, C.c_int32]),
    "sym_sched_done": (None, [C.c_void_p, C.c_int32, C.c_double]),
    "sym_sched_next_deadline": (C.c_double, [C.c_void_p]),
    "sym_sched_state": (C.c_int, [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double),
                                  C.POINTER(C.c_double), _I64P]),
    "sym_profile_enable": (C.c_int, [C.c_void_p, C.c_int]),
    "sym_profile_read": (C.c_int, [C.c_void_p, C.c_int, C.POINTER(C.c_double), _I64P]),
    "sym_calib_read": (C.c_int, [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]),
    "sym_calib_copy": (C.c_int, [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]),
    "sym_calib_mfma": (C.c_int, [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]),
}


def load():
    """Loads the C-ABI library (once).  Raises if it is missing or lacks a declared symbol."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python __graft_entry__.py` (hipcc, gfx950) first")
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)          # AttributeError if the symbol is missing
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, np.int32)
    return a, a.ctypes.data_as(_I32P)


def as_i32p(a):
    """Pointer to the data of a contiguous int32 numpy array (the caller keeps the array alive)."""
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return C.cast(a.ctypes.data, _I32P)


def _i64(a):
    a = np.ascontiguousarray(a, np.int64)
    return a, a.ctypes.data_as(_I64P)


def _ptr(t):
    """Device (or host) address of a torch tensor / int / None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_contiguous()
    return t.data_ptr()


def make_config(n_q_heads, n_kv_heads, head_dim, page_tokens, dtype, n_pages, device=-1, pool=None, workspace=None,
                workspace_bytes=0, free_order=None, softmax_scale=0.0, decode_waves=0, n_layers=1, tuning=None):
    """`tuning`: dict of sym_tuning fields to change from the library's defaults for this shape."""
    cfg = SymConfig()
    cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.page_tokens = n_q_heads, n_kv_heads, head_dim, page_tokens
    cfg.dtype = {"f32": SYM_F32, "bf16": SYM_BF16}.get(dtype, dtype)
    cfg.device, cfg.n_pages = device, n_pages
    cfg.pool, cfg.workspace, cfg.workspace_bytes = _ptr(pool), _ptr(workspace), workspace_bytes
    keep = None
    if free_order is not None:
        keep, p = _i32(free_order)
        cfg.free_order = p
    cfg.softmax_scale, cfg.decode_waves, cfg.n_layers = softmax_scale, decode_waves, n_layers
    cfg._keep = keep
    if tuning:
        t = SymTuning()
        if load().sym_tuning_defaults(C.byref(cfg), C.byref(t)) != SYM_OK:
            raise SymError(SYM_EINVAL, "sym_tuning_defaults: unsupported shape")
        for name, value in tuning.items():
            if name not in TUNING_FIELDS:
                raise KeyError(f"no planner setting called {name!r}")
            setattr(t, name, int(value))
        cfg._tuning = t
        cfg.tuning = C.pointer(t)
    return cfg


def page_bytes(cfg):
    return load().sym_page_bytes(C.byref(cfg))


def workspace_bytes(cfg, max_lips, max_tokens, max_table_entries):
    return load().sym_workspace_bytes(C.byref(cfg), max_lips, max_tokens, max_table_entries)


class BatchTimer:
    """The batch-firing controller of the inference scheduler (paper section 4.4): marshalling only."""

    def __init__(self, max_batch, max_wait_us, weight=0.125, a_us=50.0, c_us=1.0):
        self.lib = load()
        self.s = self.lib.sym_sched_create(max_batch, max_wait_us, weight, a_us, c_us)
        if not self.s:
            raise SymError(SYM_EINVAL, "sym_sched_create: bad argument")

    def arrive(self, now_us):
        self.lib.sym_sched_arrive(self.s, now_us)

    def decide(self, now_us, gpu_idle=True):
        return self.lib.sym_sched_decide(self.s, now_us, 1 if gpu_idle else 0)

    def fired(self, n):
        self.lib.sym_sched_fired(self.s, n)

    def done(self, n, service_us):
        self.lib.sym_sched_done(self.s, n, service_us)

    def next_deadline(self):
        return self.lib.sym_sched_next_deadline(self.s)

    def state(self):
        r, t, a, c = C.c_double(), C.c_double(), C.c_double(), C.c_double()
        p = C.c_int64()
        self.lib.sym_sched_state(self.s, C.byref(r), C.byref(t), C.byref(a), C.byref(c), C.byref(p))
        return dict(rate=r.value, target=t.value, a=a.value, c=c.value, pending=p.value)

    def close(self):
        if self.s:
            self.lib.sym_sched_destroy(self.s)
            self.s = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Context:
    """One sym_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, cfg):
        self.lib = load()
        self.cfg = cfg
        h = C.c_void_p()
        rc = self.lib.sym_init(C.byref(cfg), C.byref(h))
        if rc != SYM_OK:
            raise SymError(rc, "sym_init failed")
        self.h = h

    def close(self):
        if self.h:
            self.lib.sym_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, rc):
        if rc < 0:
            raise SymError(rc, self.lib.sym_strerror(self.h).decode())
        return rc

    # ---- KVFS ----
    def kv_open(self, name=None):
        return self._chk(self.lib.sym_kv_open(self.h, None if name is None else name.encode()))

    def kv_fork(self, parent):
        return self._chk(self.lib.sym_kv_fork(self.h, parent))

    def kv_remove(self, kv):
        self._chk(self.lib.sym_kv_remove(self.h, kv))

    def kv_close(self, kv):
        self._chk(self.lib.sym_kv_close(self.h, kv))

    def kv_len(self, kv):
        return self._chk(self.lib.sym_kv_len(self.h, kv))

    def kv_truncate(self, kv, new_len):
        kv_a, kv_p = _i32(kv)
        ln_a, ln_p = _i64(new_len)
        self._chk(self.lib.sym_kv_truncate(self.h, len(kv_a), kv_p, ln_p))

    def kv_append(self, kv, n, k, v, stream=None):
        self._chk(self.lib.sym_kv_append(self.h, kv, n, _ptr(k), _ptr(v), stream))

    def kv_extract(self, src, idx, stream=None):
        """One file: handle of the new file holding tokens idx of file src."""
        return self.kv_extract_batch([src], [idx], stream)[0]

    def kv_extract_batch(self, srcs, idx_lists, stream=None, flat=None, off=None):
        """Several files in one call (one copy launch): list of new handles.  idx_lists: one index
        list per file, or None with the flattened indices `flat` and their offsets `off` given."""
        s_a, s_p = _i32(srcs)
        if idx_lists is not None:
            off = np.zeros(len(s_a) + 1, np.int64)
            off[1:] = np.cumsum([len(i) for i in idx_lists])
            flat = np.concatenate([np.asarray(i, np.int64).ravel() for i in idx_lists]) if len(idx_lists) else np.zeros(0, np.int64)
        ix_a, ix_p = _i64(flat)
        of_a, of_p = _i64(off)
        out = np.empty(len(s_a), np.int32)
        self._chk(self.lib.sym_kv_extract(self.h, len(s_a), s_p, of_p, ix_p, out.ctypes.data_as(_I32P), stream))
        return [int(h) for h in out]

    def kv_merge(self, files, stream=None):
        f_a, f_p = _i32(files)
        return self._chk(self.lib.sym_kv_merge(self.h, len(f_a), f_p, stream))

    def kv_offload(self, kv, stream=None):
        kv_a, kv_p = _i32(kv)
        self._chk(self.lib.sym_kv_offload(self.h, len(kv_a), kv_p, stream))

    def kv_restore(self, kv, stream=None):
        kv_a, kv_p = _i32(kv)
        self._chk(self.lib.sym_kv_restore(self.h, len(kv_a), kv_p, stream))

    def kv_waiting(self, kv):
        return bool(self._chk(self.lib.sym_kv_waiting(self.h, kv)))

    def last_swaps(self):
        n = self._chk(self.lib.sym_last_swaps(self.h, None, 0))
        out = np.empty((n, 2), np.int32)
        self._chk(self.lib.sym_last_swaps(self.h, out.ctypes.data_as(_I32P), n))
        return out

    def last_moves(self):
        n = self._chk(self.lib.sym_last_moves(self.h, None, 0))
        out = np.empty((n, 2), np.int32)
        self._chk(self.lib.sym_last_moves(self.h, out.ctypes.data_as(_I32P), n))
        return out

    # ---- pred ----
    def pred_batch(self, kv, n_tokens, q, k_new, v_new, out, stream=None):
        kv_a, kv_p = _i32(kv)
        nt_a, nt_p = _i32(n_tokens)
        self._chk(self.lib.sym_pred_batch(self.h, len(kv_a), kv_p, nt_p, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), stream))

    def pred_begin(self, kv, n_tokens, stream=None):
        kv_a, kv_p = _i32(kv)
        nt_a, nt_p = _i32(n_tokens)
        self._chk(self.lib.sym_pred_begin(self.h, len(kv_a), kv_p, nt_p, stream))

    def pred_layer(self, layer, q, k_new, v_new, out, stream=None):
        rc = self.lib.sym_pred_layer(self.h, layer, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), stream)
        if rc < 0:
            self._chk(rc)

    def pred_end(self):
        self._chk(self.lib.sym_pred_end(self.h))

    def pred_batch_static(self, kv, n_tokens, q, k_new, v_new, out, stream=None):
        kv_a, kv_p = _i32(kv)
        nt_a, nt_p = _i32(n_tokens)
        self._chk(self.lib.sym_pred_batch_static(self.h, len(kv_a), kv_p, nt_p, _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out), stream))

    def test_fail_staging(self, count):
        self._chk(self.lib.sym_test_fail_staging(self.h, count))

    def prepare_batch(self, kv, n_tokens, q, k_new, v_new, out):
        """Marshals the arguments of pred_batch once, for callers that issue the same batch many
        times (a decode loop): returns an object for pred_prepared.  The arrays and tensors are
        kept alive by the object."""
        kv_a, nt_a = np.ascontiguousarray(kv, np.int32), np.ascontiguousarray(n_tokens, np.int32)
        keep = (kv_a, nt_a, q, k_new, v_new, out)
        args = (len(kv_a), C.cast(kv_a.ctypes.data, _I32P), C.cast(nt_a.ctypes.data, _I32P), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(out))
        return keep, args

    def pred_prepared(self, prepared, stream=None):
        rc = self.lib.sym_pred_batch(self.h, *prepared[1], stream)
        if rc < 0:
            self._chk(rc)

    def pred_batch_raw(self, n_tokens, page_table_flat, pt_offsets, lengths, q, out, stream=None):
        nt_a, nt_p = _i32(n_tokens)
        pt_a, pt_p = _i32(page_table_flat)
        po_a, po_p = _i64(pt_offsets)
        ln_a, ln_p = _i64(lengths)
        self._chk(self.lib.sym_pred_batch_raw(self.h, len(nt_a), nt_p, pt_p, po_p, ln_p, _ptr(q), _ptr(out), stream))

    # ---- introspection ----
    def kv_pages(self, kv):
        n = self._chk(self.lib.sym_kv_pages(self.h, kv, None, 0))
        out = np.zeros(max(n, 1), np.int32)
        self._chk(self.lib.sym_kv_pages(self.h, kv, out.ctypes.data_as(_I32P), n))
        return out[:n].tolist()

    def page_refcount(self, page):
        return self._chk(self.lib.sym_page_refcount(self.h, page))

    def free_pages(self):
        return self._chk(self.lib.sym_free_pages(self.h))

    def get_stats(self):
        s = SymStats()
        self._chk(self.lib.sym_get_stats(self.h, C.byref(s)))
        return {n: getattr(s, n) for n, _ in SymStats._fields_}

    def plan_append(self, kv, n_tokens):
        kv_a, kv_p = _i32(kv)
        nt_a, nt_p = _i32(n_tokens)
        cow = np.zeros(3 * max(len(kv_a), 1), np.int32)
        slots = np.zeros(max(int(nt_a.sum()) if len(nt_a) else 0, 1), np.int32)
        n_cow = C.c_int32(0)
        self._chk(self.lib.sym_plan_append(self.h, len(kv_a), kv_p, nt_p, cow.ctypes.data_as(_I32P), len(kv_a),
                                           C.byref(n_cow), slots.ctypes.data_as(_I32P)))
        T = int(nt_a.sum())
        return [tuple(int(x) for x in cow[3 * i:3 * i + 3]) for i in range(n_cow.value)], slots[:T].copy()

    def plan_copies_first(self):
        return bool(self._chk(self.lib.sym_plan_copies_first(self.h)))

    def build_desc(self, n_tokens, page_table_flat, pt_offsets, lengths):
        nt_a, nt_p = _i32(n_tokens)
        pt_a, pt_p = _i32(page_table_flat)
        po_a, po_p = _i64(pt_offsets)
        ln_a, ln_p = _i64(lengths)
        n = self._chk(self.lib.sym_build_desc(self.h, len(nt_a), nt_p, pt_p, po_p, ln_p, None, 0))
        out = np.zeros(n, np.int32)
        self._chk(self.lib.sym_build_desc(self.h, len(nt_a), nt_p, pt_p, po_p, ln_p, out.ctypes.data_as(_I32P), n))
        return out

    def kv_read(self, kv, start, n, k_out, v_out, stream=None, layer=0):
        self._chk(self.lib.sym_kv_read_layer(self.h, kv, layer, start, n, _ptr(k_out), _ptr(v_out), stream))

    # ---- measurement ----
    def profile_enable(self, mask, stride=1):
        """mask: bit k = time kernel id k; stride s: only every s-th launch of each id."""
        return self._profile_enable(int(mask) | (int(stride) << 8))

    def _profile_enable(self, mask):
        """mask: bit k = time kernel id k (K_ATTN ...); 0 = off."""
        self._chk(self.lib.sym_profile_enable(self.h, int(mask)))

    def profile_read(self, kernel_id):
        ms, n = C.c_double(0), C.c_int64(0)
        self._chk(self.lib.sym_profile_read(self.h, kernel_id, C.byref(ms), C.byref(n)))
        return ms.value, n.value


def calib_read(src, nbytes, out8, stream=None):
    rc = load().sym_calib_read(_ptr(src), nbytes, _ptr(out8), stream)
    if rc:
        raise SymError(rc, "calib_read")


def calib_mfma(out, blocks, iters, stream=None):
    """flops of the launch: blocks * 8 * iters * 16 * 32768."""
    rc = load().sym_calib_mfma(_ptr(out), blocks, iters, stream)
    if rc:
        raise SymError(rc, "calib_mfma")
    return blocks * 8 * iters * 16 * 32768


def calib_copy(dst, src, nbytes, stream=None):
    rc = load().sym_calib_copy(_ptr(dst), _ptr(src), nbytes, stream)
    if rc:
        raise SymError(rc, "calib_copy")

#!/usr/bin/env python3
"""Benchmark of the pred hot path on one MI355X.

A step = one pred over one batch of a synthetic LIP workload = the whole hot path: collect the calls,
plan the append, build and upload the batch descriptor (once per step), then for every attention
layer of the step the launches of that layer (copy-on-write copies and the rows of multi-token
LIPs if any; the attention kernel: decode bins with the single-token appends, MFMA tiles for prefill
chunks and shared prefixes; the merge of divided ranges).  Every layer has K/V pages of its own
(as a real pred walks the model's layers), so the KV bytes of a launch come from HBM and not from
the 256 MB last-level cache.

Default: the workload the headline metric is quoted on, the "decode batch" (64 LIPs, 32 Q / 8 KV
heads, head dim 128, bf16, contexts uniform 512..4096, one new token each, 32 layers per step),
and under "workloads" the same measurements, briefly, for the fork tree, the mixed batch, the
prefill chunks alone, the long contexts, draft verification and short contexts.
`--workload decode|fork|mixed|prefill|long|draft|short` times one of them alone;
`--workload prune` times kv_extract (context pruning, paper section 4.2) on the decode batch's files;
`--workload offload` times kv_offload + kv_restore (paper section 4.3) of those files over the host link;
`--workload rag` drives the library with the paper's section 5 workload (100 documents x 3000 tokens,
prompt caching of the 20 most requested topics, Poisson requests, batches fired by the library's
controller) for several Pareto indices, end to end in virtual time.

Prints ONE JSON line: whole-path throughput in algorithmic KV TB/s, plus `roofline` for the
dominant kernel (the attention launch, timed with HIP events on its stream inside the timed region) and `cpu_baseline`
(the CPU oracle timed on the same workload for a bounded time).
"""
import argparse
import contextlib
import gc
import json
import os
import sys
import time


@contextlib.contextmanager
def timed_region():
    """No cyclic garbage collection inside a timed region: one full collection of the interpreter's heap
    (tens of milliseconds with the workload's setup data alive) in the middle of a 40 ms loop would be
    charged to the GPU path (seen on the mixed workload: 3.3 ms per step instead of 1.9 ms)."""
    gc.collect()
    gc.disable()
    try:
        yield
    finally:
        gc.enable()

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_TBPS = 8.0        # MI355X published HBM3E peak
MFMA_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16/fp16 matrix peak


def kv_token_bytes(shape):
    return 2 * shape.n_kv_heads * shape.head_dim * (4 if shape.dtype == "f32" else 2)


def algorithmic_bytes(shape, kv_tokens, n_tokens, table_entries):
    """Bytes one launch must move: `kv_tokens` valid KV tokens read once, the appended rows
    written, Q read, O written (fp32), page-table entries read."""
    es = 4 if shape.dtype == "f32" else 2
    T = sum(n_tokens)
    return (kv_tokens * kv_token_bytes(shape) + T * kv_token_bytes(shape) + T * shape.n_q_heads * shape.head_dim * es +
            T * shape.n_q_heads * shape.head_dim * 4 + table_entries * 4)


def read_traffic_note(name):
    """HBM traffic per launch of the dominant kernel from the committed counter summary."""
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def stats_shared_pairs(sess, wl, after, P):
    """(query row, key) pairs that the shared-prefix tiles compute: for every group of single-token
    LIPs the library forms, members x tokens of their common full pages.  Recomputed here from the
    page tables with the library's rule of thumb (same first page, at least 4 files, 8 pages)."""
    groups = {}
    for f, n, L in zip(wl.batch_files, wl.batch_n, after):
        if n == 1:
            pages = sess.pages(f)
            groups.setdefault(pages[0] if pages else -1, []).append((pages, (L - 1) // P))
    pairs = 0
    for members in groups.values():
        if len(members) < 4:
            continue
        c = min(m[1] for m in members)
        first = members[0][0]
        for pages, _ in members[1:]:
            k = 0
            while k < c and pages[k] == first[k]:
                k += 1
            c = k
        c &= ~1
        if c >= 8:
            pairs += len(members) * c * P
    return pairs


def cpu_baseline(wl, budget_s, np, reset_lengths):
    """The oracle as it stands on the same workload: all LIPs, one pred step after another,
    until about `budget_s` seconds have passed (at least one step)."""
    from oracle.driver import OracleSession
    from threadpoolctl import threadpool_info
    osess = OracleSession(wl.shape, wl.n_pages, wl.free_order)
    osess.setup(wl.setup_ops())
    b = wl.batch()
    n_lips = len(b["files"])
    P = wl.shape.page_tokens
    steps, nbytes = 0, 0
    t0 = time.perf_counter()
    while True:
        before = [osess.model.kv_len(osess.h[f]) for f in b["files"]]
        after = [L + n for L, n in zip(before, b["n_tokens"])]
        osess.pred(b, dtype=np.float32)
        nbytes += algorithmic_bytes(wl.shape, sum(after), b["n_tokens"], sum(-(-L // P) for L in after))
        if reset_lengths:
            for f, L in zip(b["files"], before):
                osess.model.kv_truncate(osess.h[f], L)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s:
            break
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": nbytes / dt / 1e12, "unit": "TB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{steps} pred step(s) of the same {n_lips}-LIP batch (append + page gather + fp32 softmax attention per "
                      f"LIP; logical bytes, every reader counted), {dt:.1f} s wall", "lip_steps_per_s": steps * n_lips / dt}


def bench_prune(args, np, torch, binding, synth, HipSession, dev):
    """kv_extract over the 64 files of the decode batch in one call: every file keeps its first page
    and each later token with probability 1/2, in order (a pruned context).  A step = the whole call
    (planning on the host, move list through pinned staging, the copy kernel) + removing the new
    files again.  Roofline: the copy kernel against HBM, bytes = kept tokens x K/V bytes, read + written."""
    wl = synth.config2(slack_pages=8192)
    shape, P = wl.shape, wl.shape.page_tokens
    layers = args.layers or 4
    steps = args.steps if args.steps is not None else 200
    warmup = args.warmup if args.warmup is not None else 20
    n_files = len(wl.batch_files)
    sessions = []
    for li in range(layers):
        s = HipSession(shape, wl.n_pages, wl.free_order, dev, max_lips=n_files, max_tokens=max(wl.lengths.values()) + 64,
                       max_entries=sum(wl.pages_after_batch().values()) + 64 * n_files)
        s.setup(wl.setup_ops())
        sessions.append(s)
        print(f"[bench] layer pool {li + 1}/{layers} built", file=sys.stderr, flush=True)
    rng = np.random.default_rng(1002)
    lengths = [wl.lengths[f] for f in wl.batch_files]
    idx_lists = [np.r_[np.arange(P), P + np.flatnonzero(rng.random(L - P) < 0.5)].astype(np.int64) for L in lengths]
    off = np.zeros(n_files + 1, np.int64)
    off[1:] = np.cumsum([len(i) for i in idx_lists])
    flat = np.concatenate(idx_lists)
    srcs = [[s.h[f] for f in wl.batch_files] for s in sessions]
    stream = torch.cuda.current_stream(dev).cuda_stream
    torch.cuda.synchronize()

    def step(i):
        s = sessions[i % layers]
        for h in s.ctx.kv_extract_batch(srcs[i % layers], None, stream, flat=flat, off=off):
            s.ctx.kv_remove(h)

    with timed_region():
        for i in range(warmup):
            step(i)
        torch.cuda.synchronize()
        st0 = sessions[0].ctx.get_stats()
        for s in sessions:
            s.ctx.profile_enable(1 << binding.K_MOVE)
        t0 = time.perf_counter()
        for i in range(warmup, warmup + steps):
            step(i)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    ms, n = 0.0, 0
    for s in sessions:
        a, b = s.ctx.profile_read(binding.K_MOVE)
        ms, n = ms + a, n + b
        s.ctx.profile_enable(0)
    st1 = sessions[0].ctx.get_stats()
    if not args.no_calib:
        # one plain copy of known size (1 GiB read + 1 GiB written): the reference dispatch that
        # scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command
        buf = torch.empty(2 << 30, dtype=torch.uint8, device=dev)
        buf.random_(0, 255)
        binding.calib_copy(buf[1 << 30:], buf, 1 << 30, stream)
        torch.cuda.synchronize()
        del buf
    moved = (st1["tokens_moved"] - st0["tokens_moved"]) / max(1, len([i for i in range(warmup, warmup + steps) if i % layers == 0]))
    step_bytes = moved * (2 * kv_token_bytes(shape) + 16)          # rows read + written, move list read by staging and kernel
    move_ms = ms / max(n, 1)
    ach = step_bytes / (move_ms * 1e-3) / 1e9
    for s in sessions:
        s.close()
    del sessions
    torch.cuda.empty_cache()
    cpu = None
    cpu_s = args.cpu_seconds if args.cpu_seconds is not None else 8.0
    if cpu_s > 0:
        from oracle.driver import OracleSession
        from threadpoolctl import threadpool_info
        small = synth.config2(n_lips=4, slack_pages=512)
        osess = OracleSession(small.shape, small.n_pages)
        osess.setup(small.setup_ops())
        t1 = time.perf_counter()
        done, toks = 0, 0
        while time.perf_counter() - t1 < cpu_s:
            f = done % 4
            h, moves = osess.model.kv_extract(osess.h[f], [int(i) for i in idx_lists[f]])
            osess.pool.move_tokens(moves)
            osess.model.kv_remove(h)
            toks += len(moves)
            done += 1
        dt = time.perf_counter() - t1
        cpu = {"value": toks * 2 * kv_token_bytes(shape) / dt / 1e12, "unit": "TB/s", "cores": int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1])),
               "kind": "oracle", "sample": f"{done} kv_extract calls on the first 4 files of the same workload (page decisions + row copies), {dt:.1f} s wall"}
    line = {"metric": "kv_extract moved KV TB/s (read + written)", "value": round(step_bytes / (wall / steps) / 1e12, 4), "unit": "TB/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(wall / steps * 1e3, 5), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "prune: kv_extract of the 64 decode-batch files (contexts U{512..4096}, 32Q/8KV, bf16) in one call, first page "
                                   "kept (shared), later tokens kept with probability 1/2; new files removed after every step",
                       "layer_pools_rotated": layers, "tokens_copied_per_step": int(moved), "algorithmic_bytes_per_step": int(step_bytes)},
            "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_TBPS * 1e3, "unit": "GB/s", "frac": round(ach / (HBM_PEAK_TBPS * 1e3), 4),
                         "traffic": read_traffic_note("move_prune_pmc.txt"), "kernel": "move_kernel", "avg_launch_us": round(move_ms * 1e3, 2), "launches": n},
            "cpu_baseline": cpu}
    print(json.dumps(line))


PCIE_PEAK_GBPS = 64.0      # PCIe 5.0 x16, one direction, before protocol overhead


def bench_offload(args, np, torch, binding, synth, HipSession, dev):
    """kv_offload then kv_restore of the 64 files of the decode batch (every page leaves for pinned
    host memory and comes back).  A step = both calls.  The copy kernel is bound by the host link,
    not by HBM: its rate is reported against the link's one-direction peak."""
    wl = synth.config2()
    shape = wl.shape
    steps = args.steps if args.steps is not None else 10
    warmup = args.warmup if args.warmup is not None else 2
    s = HipSession(shape, wl.n_pages, wl.free_order, dev, max_lips=64, max_tokens=max(wl.lengths.values()) + 64,
                   max_entries=sum(wl.pages_after_batch().values()) + 64 * 64)
    s.setup(wl.setup_ops())
    hs = [s.h[f] for f in wl.batch_files]
    stream = torch.cuda.current_stream(dev).cuda_stream
    n_pages = sum(len(s.pages(f)) for f in wl.batch_files)
    nbytes = n_pages * s.page_bytes
    torch.cuda.synchronize()
    out_ms, in_ms = [], []
    t_wall = 0.0
    with timed_region():
        for i in range(warmup + steps):
            s.ctx.profile_enable(1 << binding.K_SWAP)
            t0 = time.perf_counter()
            s.ctx.kv_offload(hs, stream)
            torch.cuda.synchronize()
            a, _ = s.ctx.profile_read(binding.K_SWAP)
            s.ctx.kv_restore(hs, stream)
            torch.cuda.synchronize()
            b, _ = s.ctx.profile_read(binding.K_SWAP)
            dt = time.perf_counter() - t0
            if i >= warmup:
                out_ms.append(a)
                in_ms.append(b)
                t_wall += dt
    st = s.ctx.get_stats()
    s.close()
    o, r = float(np.mean(out_ms)), float(np.mean(in_ms))
    slow = max(o, r)
    line = {"metric": "kv_offload + kv_restore GB/s over the host link", "value": round(2 * nbytes / (t_wall / steps) / 1e9, 2), "unit": "GB/s",
            "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(t_wall / steps * 1e3, 3), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "offload: all 64 files of the decode batch (contexts U{512..4096}, 32Q/8KV, bf16) leave for pinned host "
                                   "memory in one call and come back in one call", "pages": n_pages, "bytes_each_way": int(nbytes)},
            "offload_GBps": round(nbytes / (o * 1e-3) / 1e9, 2), "restore_GBps": round(nbytes / (r * 1e-3) / 1e9, 2),
            "offload_ms": round(o, 3), "restore_ms": round(r, 3),
            "roofline": {"bound": "pcie", "achieved": round(nbytes / (slow * 1e-3) / 1e9, 2), "peak": PCIE_PEAK_GBPS, "unit": "GB/s",
                         "frac": round(nbytes / (slow * 1e-3) / 1e9 / PCIE_PEAK_GBPS, 4), "traffic": None, "kernel": "swap_kernel (slower direction)",
                         "avg_launch_us": round(slow * 1e3, 1), "launches": 2 * steps},
            "cpu_baseline": None, "pool_stats": {"host_slots": st["host_slots"], "pages_offloaded": st["pages_offloaded"]}}
    print(json.dumps(line))


def bench_rag(args, np, torch, binding, synth, HipSession, dev):
    """Section 5's RAG scenario on the attention path alone: throughput and latency against the
    Pareto index of the topic popularity, with and without the LIP's prompt cache."""
    from paper_2510_25412_amd import rag
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    n_req = args.steps if args.steps is not None else 1500
    rows = []
    for pareto, retain in ((0.5, 20), (1.0, 20), (2.0, 20), (1.0, 0)):
        cfg = rag.RagConfig(pareto_index=pareto, retain=retain, n_requests=n_req, rate_per_s=args.rag_rate)
        # room for every request's file at once (no admission control here) + the retained documents
        n_pages = (n_req + retain + 8) * ((cfg.doc_tokens + cfg.answer_tokens) // 16 + 2)
        s = HipSession(shape, n_pages, None, dev, max_lips=cfg.max_batch, max_tokens=cfg.max_batch * cfg.prefill_chunk + 64,
                       max_entries=cfg.max_batch * ((cfg.doc_tokens + cfg.answer_tokens) // 16 + 2) + 64)
        d = rag.RagDriver(s, cfg)
        with timed_region():
            r = d.run()
        r.update(pareto_index=pareto, retain=retain)
        rows.append(r)
        print(f"[bench] rag pareto {pareto} retain {retain}: {r['requests_per_s']:.0f} req/s, hit {r['hit_rate']:.2f}", file=sys.stderr, flush=True)
        d.close()
        s.close()
        torch.cuda.empty_cache()
    head = rows[1]
    line = {"metric": "RAG LIP-steps/s (pred calls per second, attention path only)", "value": round(head["lip_steps_per_s"], 1), "unit": "LIP-steps/s",
            "n_gpus": 1, "steps": n_req, "warmup": 0, "ms_per_step": round(1e3 / head["lip_steps_per_s"], 5), "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"rag: 100 documents x 3000 tokens, 32 answer tokens, top-20 topics retained (prompt caching by fork), Poisson "
                                   f"requests at {args.rag_rate:.0f}/s, Pareto topic popularity, 32Q/8KV bf16, batches fired by sym_sched; virtual time "
                                   "advanced by measured batch wall time; value quoted at Pareto index 1.0"},
            "by_pareto_index": [{k: (round(v, 4) if isinstance(v, float) else v) for k, v in r.items() if k != "scheduler"} for r in rows],
            "roofline": None, "cpu_baseline": None}
    print(json.dumps(line))


WORKLOADS = ("decode", "fork", "mixed", "prefill", "long", "draft", "short", "decode64q")


def workload_table(args, synth):
    """name -> (generator, layers of the model step, steps, warmup, reset lengths after each step, cpu seconds, label).
    `layers`: attention layers per pred (each with its own K/V pages: a real pred walks the model's layers, and the
    KV bytes of a launch then come from HBM and not from the 256 MB last-level cache).  Workloads whose single layer is
    far larger than that cache, or whose files are reset after every step, run one layer per step."""
    return {
        "decode": (synth.config2, 32, 20, 5, False, 12.0, "decode batch: 64 LIPs, 32Q/8KV heads, head_dim 128, bf16, page 16, "
                   "contexts U{512..4096}, 1 new token each"),
        "fork": (lambda: synth.config3(slack_pages=2048), 8, 40, 5, False, 0.0, "fork tree: 16 roots x 2048-token prefix, each forked 16x (256 LIPs), "
                 "private suffix U{1..256}, 32Q/8KV, bf16, 1 new token each"),
        "mixed": (synth.config4, 1, 20, 3, True, 0.0, "mixed: 32 LIPs x 512-token prefill chunk on U{0..8192} + 224 decode LIPs "
                  "U{1024..4096}, 32Q/8KV, bf16 (files truncated back after every step)"),
        "prefill": (lambda: synth.config4(n_decode=0), 1, 20, 3, True, 0.0, "prefill only: the 32 prefill LIPs of the mixed batch (512-token chunk on "
                    "U{0..8192}), 32Q/8KV, bf16 (files truncated back after every step)"),
        "draft": (lambda: synth.config2(n_new=4, slack_pages=1024), 8, 25, 3, False, 0.0, "draft verify: the decode batch (64 LIPs, 32Q/8KV, "
                  "bf16, contexts U{512..4096}) with 4 new tokens per LIP and call"),
        "long": (lambda: synth.config5(n_pages=args.pool_pages), 1, 40, 5, False, 0.0, "long context: 16 LIPs U{32768..131072}, "
                 "64Q/8KV, bf16, pages scattered over a %d-page pool, 1 new token each" % args.pool_pages),
        "decode64q": (lambda: synth.config2(n_q_heads=64), 16, 20, 5, False, 0.0, "decode batch with 8 query heads per kv head: 64 LIPs, 64Q/8KV heads, "
                      "head_dim 128, bf16, contexts U{512..4096}, 1 new token each"),
        "short": (lambda: synth.config2(n_lips=256, lo=100, hi=260, slack_pages=256), 16, 40, 5, False, 0.0, "short contexts: 256 LIPs, 32Q/8KV, bf16, "
                  "contexts U{100..260}, 1 new token each (the answer phase of the RAG scenario, freshly forked threads)"),
    }


def run_attention_workload(args, name, np, torch, binding, synth, HipSession, dev, steps=None, warmup=None, layers=None, cpu_s=None,
                           calib=True):
    """Times one workload.  A step = one pred over the batch = the whole hot path, once per model step: collect the
    calls, plan the append, build and upload the descriptor (sym_pred_begin), then per attention layer the launches of
    sym_pred_layer (page copies / multi-token appends if any, attention with the single-token appends, merge).  Returns
    the metrics as a dict."""
    gen, d_layers, d_steps, d_warmup, reset, d_cpu, label = workload_table(args, synth)[name]
    layers = layers or d_layers
    steps = steps if steps is not None else d_steps
    warmup = warmup if warmup is not None else d_warmup
    cpu_s = cpu_s if cpu_s is not None else d_cpu
    wl = gen()
    shape = wl.shape
    P = shape.page_tokens
    n_lips = len(wl.batch_files)
    T = int(sum(wl.batch_n))
    grow_pages = 0 if reset else -(-(steps + warmup + 64) * max(wl.batch_n) // P) * n_lips      # room for the tokens the steps append
    n_pages = wl.n_pages + grow_pages if wl.free_order is None else wl.n_pages

    # ---- build the files, every layer (inputs resident in HBM before the timed region)
    entries = sum(wl.pages_after_batch().values()) + 64 * n_lips + grow_pages
    sess = HipSession(shape, n_pages, wl.free_order, dev, max_lips=n_lips, max_tokens=max(T, max(wl.lengths.values())) + 64,
                      max_entries=entries, n_layers=layers, tuning=args.tuning_dict, decode_waves=args.decode_waves)
    sess.setup(wl.setup_ops())
    print(f"[bench] {name}: {layers} layer(s) of {n_pages} pages built", file=sys.stderr, flush=True)
    batch = wl.batch()
    db = sess.upload_batch(batch)
    kv_arr, nt_arr = np.asarray(db["kv"], np.int32), np.asarray(db["n_tokens"], np.int32)
    kv_p, nt_p = binding.as_i32p(kv_arr), binding.as_i32p(nt_arr)
    q_p, k_p, v_p, o_p = (db[x].data_ptr() for x in ("q", "k_new", "v_new", "out"))
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream(dev).cuda_stream
    ctx = sess.ctx
    len_before = [ctx.kv_len(h) for h in db["kv"]]
    len_before64 = np.asarray(len_before, np.int64)
    lib, h = ctx.lib, ctx.h
    layered = layers > 1

    def step():
        if layered:
            rc = lib.sym_pred_begin(h, n_lips, kv_p, nt_p, stream)
            for l in range(layers):
                rc = rc or lib.sym_pred_layer(h, l, q_p, k_p, v_p, o_p, stream)
        else:
            rc = lib.sym_pred_batch(h, n_lips, kv_p, nt_p, q_p, k_p, v_p, o_p, stream)
        if rc:
            ctx._chk(rc)
        if reset:
            ctx.kv_truncate(kv_arr, len_before64)

    with timed_region():          # entered before the warm-up: the collection it starts with must not leave the GPU idle just before the timed steps
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        len0 = [ctx.kv_len(hh) for hh in db["kv"]]       # lengths before the timed steps
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    stats = ctx.get_stats()

    # ---- bytes and flops of one layer of a step, at the mean lengths of the timed steps
    grow = 0 if reset else (steps - 1) / 2 * np.asarray(wl.batch_n)
    after = [int(round(L + n + g)) for L, n, g in zip(len0, wl.batch_n, np.broadcast_to(grow, (n_lips,)))]
    logical_tokens = sum(after)
    # unique pages: a page shared by forks is counted once, with the most tokens any reader sees in it
    seen = {}
    for f, L in zip(wl.batch_files, after):
        for idx, pg in enumerate(sess.pages(f)):
            seen[pg] = max(seen.get(pg, 0), min(P, L - idx * P))
    unique_tokens = sum(v for v in seen.values() if v > 0)
    table_entries = sum(-(-L // P) for L in after)
    layer_bytes = algorithmic_bytes(shape, unique_tokens, wl.batch_n, table_entries)
    logical_bytes = algorithmic_bytes(shape, logical_tokens, wl.batch_n, table_entries)
    # matrix-core work of the launch: (query row, key) pairs of prefill chunks (tile kernel), x 4*D flops per head
    min_pre = 16        # LIPs with at least this many new tokens run as prefill tiles
    pre_pairs = sum(n * (L - n) + n * (n + 1) // 2 for L, n in zip(after, wl.batch_n) if n >= min_pre)
    shared_pairs = stats_shared_pairs(sess, wl, after, P)
    mfma_flops = 4 * shape.head_dim * shape.n_q_heads * (pre_pairs + shared_pairs)
    ms_per_step = wall / steps * 1e3
    ms_per_layer = ms_per_step / layers
    tbps = layer_bytes / (ms_per_layer * 1e-3) / 1e12
    G = shape.n_q_heads // shape.n_kv_heads
    model_layers = 80 if shape.n_q_heads == 64 else 32      # layers of the Llama model with this attention shape (70B / 8B)

    # ---- untimed extra passes.  (1) kernel times by HIP events that the library attaches to the dispatches (start of the first
    # kernel of the attention launch, end of its last); events on the timed launches would stretch them.
    # Every extra pass starts from the lengths the timed steps started from (the files are truncated back: host only) and
    # takes as many steps, so that it sees the same contexts as the timed region.
    len0_64 = np.asarray(len0, np.int64)
    n_extra = max(1, min(steps, 64))
    ctx.kv_truncate(kv_arr, len0_64)
    ctx.profile_enable(0x7)
    for _ in range(n_extra):
        step()
    torch.cuda.synchronize()
    breakdown = {}
    for kname, kid in (("prologue", binding.K_PROLOGUE), ("attention", binding.K_ATTN), ("merge", binding.K_MERGE)):
        ms, n = ctx.profile_read(kid)
        breakdown[kname + "_us"] = round(ms / n * 1e3, 2) if n else None
        breakdown[kname + "_launches_per_layer"] = round(n / (n_extra * layers), 3)
    ctx.kv_truncate(kv_arr, len0_64)
    ctx.profile_enable(1 << binding.K_ATTN)
    for _ in range(n_extra):
        step()
    torch.cuda.synchronize()
    attn_ms, attn_n = ctx.profile_read(binding.K_ATTN)
    attn_ms /= max(attn_n, 1)
    ctx.profile_enable(0)
    # (2) the step on the stream: an event between every two steps
    n_dist = n_extra
    ctx.kv_truncate(kv_arr, len0_64)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_dist + 1)]
    evs[0].record()
    for i in range(n_dist):
        step()
        evs[i + 1].record()
    torch.cuda.synchronize()
    per_layer = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 / layers for i in range(n_dist))
    spread = {"steps": n_dist, "p10": round(per_layer[n_dist // 10], 2), "median": round(per_layer[n_dist // 2], 2),
              "p90": round(per_layer[min(n_dist - 1, (9 * n_dist) // 10)], 2), "unit": "us per layer of a step, on the stream"}

    # the attention kernel against both roofs; the one it sits closer to is reported as its bound
    hbm_ach = layer_bytes / (attn_ms * 1e-3) / 1e9
    mfma_ach = mfma_flops / (attn_ms * 1e-3) / 1e12
    note = {"decode": "attn_decode_batch_pmc.txt"}.get(name, f"attn_{name}_pmc.txt")
    # decode ranges run on the matrix cores for 8 query heads per kv head and for multi-token rows
    kname = f"decode_mfma_kernel<G={G}>" if name in ("long", "draft") else (f"decode_only_kernel<bf16, G={G}>" if name in ("decode", "short") else f"attn_kernel<bf16, G={G}>")
    roof_hbm = {"bound": "hbm", "achieved": round(hbm_ach, 1), "peak": HBM_PEAK_TBPS * 1e3, "unit": "GB/s",
                "frac": round(hbm_ach / (HBM_PEAK_TBPS * 1e3), 4), "traffic": read_traffic_note(note),
                "kernel": kname, "avg_launch_us": round(attn_ms * 1e3, 2), "launches": attn_n}
    roof_mfma = {"bound": "mfma", "achieved": round(mfma_ach, 1), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                 "frac": round(mfma_ach / MFMA_PEAK_TFLOPS, 4), "traffic": read_traffic_note(note),
                 "kernel": kname, "avg_launch_us": round(attn_ms * 1e3, 2), "launches": attn_n,
                 "flops_per_launch": int(mfma_flops)}
    dominant, other = (roof_mfma, roof_hbm) if roof_mfma["frac"] > roof_hbm["frac"] else (roof_hbm, roof_mfma)

    stream_read = mfma_sustained = None
    if calib and not args.no_calib:
        nbytes = 4 << 30
        buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        buf.random_(0, 255)     # real bytes in every page
        out8 = torch.zeros(1, dtype=torch.int64, device=dev)
        for _ in range(3):
            binding.calib_read(buf, nbytes, out8, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            binding.calib_read(buf, nbytes, out8, stream)
        e1.record()
        torch.cuda.synchronize()
        stream_read = nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e12
        # one plain copy of known size (1 GiB read + 1 GiB written): the reference dispatch that
        # scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run of this command
        binding.calib_copy(buf[1 << 30:], buf, 1 << 30, stream)
        torch.cuda.synchronize()
        del buf
        if mfma_flops:
            # what the matrix cores sustain on this part with nothing but MFMAs in the loop (two wavefronts
            # per SIMD, operands in registers): the rate under the power limit, below the nominal peak
            blocks = torch.cuda.get_device_properties(dev).multi_processor_count
            sink = torch.empty(blocks * 512, dtype=torch.float32, device=dev)
            binding.calib_mfma(sink, blocks, 2000, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fl = binding.calib_mfma(sink, blocks, 20000, stream)
            e1.record()
            torch.cuda.synchronize()
            mfma_sustained = fl / (e0.elapsed_time(e1) * 1e-3) / 1e12
            del sink

    sess.close()
    del sess, db
    torch.cuda.empty_cache()
    cpu = cpu_baseline(wl, cpu_s, np, reset) if cpu_s > 0 else None
    n_pred = max(stats["pred_batches"], 1)
    return {
        "metric": "pred-batch attention KV TB/s", "value": round(tbps, 4), "unit": "TB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": label + f"; a step = one pred over the batch through {layers} attention layer(s) "
                               "(host: plan + descriptor once per step; device: one attention launch per layer, every layer with K/V pages of its own)",
                   "layers_per_step": layers, "kv_tokens_per_layer": int(unique_tokens), "algorithmic_bytes_per_layer": int(layer_bytes),
                   "algorithmic_bytes_per_step": int(layer_bytes) * layers,
                   "logical_kv_tokens_per_layer": int(logical_tokens), "logical_bytes_per_layer": int(logical_bytes),
                   "tuning": args.tuning_dict or "library defaults"},
        "us_per_layer": round(ms_per_layer * 1e3, 3),
        "pct_hbm_peak": round(100 * tbps / HBM_PEAK_TBPS, 2),
        "effective_TBps_logical": round(logical_bytes / (ms_per_layer * 1e-3) / 1e12, 4),
        # one LIP-step = one LIP through one attention layer (what the metric counted so far); all layers: the model step
        "lip_steps_per_s": round(n_lips / (ms_per_layer * 1e-3), 1),
        "lip_steps_per_s_all_layers": {"layers": model_layers, "value": round(n_lips / (ms_per_layer * 1e-3) / model_layers, 1)},
        "step_us_spread": spread,
        "roofline": dominant,
        "roofline_other": other if mfma_flops else None,
        "kernel_breakdown": breakdown,
        "stream_read_TBps": round(stream_read, 3) if stream_read else None,
        "frac_of_stream_read": round(hbm_ach / 1e3 / stream_read, 4) if stream_read else None,
        "mfma_sustained_TFLOPs": round(mfma_sustained, 1) if mfma_sustained else None,
        "frac_of_mfma_sustained": round(mfma_ach / mfma_sustained, 4) if mfma_sustained else None,
        "cpu_baseline": cpu,
        "host_us_per_step": {"plan_and_descriptor": round(stats["host_ns_plan"] / n_pred / 1e3, 2),
                             "whole_step": round(stats["host_ns_pred"] / n_pred / 1e3, 2)},
        "pool_stats": {"pages_total": stats["pages_total"], "pages_free": stats["pages_free"], "pages_shared": stats["pages_shared"]},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", choices=list(WORKLOADS) + ["prune", "offload", "rag"], default=None,
                    help="time this workload only (default: the decode batch as the headline, and the other configurations briefly under \"workloads\")")
    ap.add_argument("--layers", type=int, default=None, help="attention layers per step (each with its own pool of K/V pages)")
    ap.add_argument("--cpu-seconds", type=float, default=None, help="wall-time budget of the CPU-oracle leg (0 = skip)")
    ap.add_argument("--pool-pages", type=int, default=3_000_000, help="pages of the long-context pool")
    ap.add_argument("--no-calib", action="store_true")
    ap.add_argument("--tuning", default="", help="planner settings to change from the library's defaults, as name=value,name=value "
                                                 "(the fields of sym_tuning); the attention workloads only")
    ap.add_argument("--decode-waves", type=int, default=0, help="sym_config.decode_waves (0 = the library's choice)")
    ap.add_argument("--no-extra", action="store_true", help="headline workload only")
    ap.add_argument("--rag-rate", type=float, default=6000.0, help="request arrivals per second of the rag workload")
    args = ap.parse_args()
    args.tuning_dict = {k.strip(): int(v) for k, v in (kv.split("=") for kv in args.tuning.split(",") if kv.strip())} or None
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path is single-GPU: it would shard by LIP or by kv head, with no exchange inside attention); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_25412_amd import binding, synth
    from paper_2510_25412_amd.driver import HipSession

    binding.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    if args.workload == "prune":
        return bench_prune(args, np, torch, binding, synth, HipSession, dev)
    if args.workload == "offload":
        return bench_offload(args, np, torch, binding, synth, HipSession, dev)
    if args.workload == "rag":
        return bench_rag(args, np, torch, binding, synth, HipSession, dev)
    head = args.workload or "decode"
    line = run_attention_workload(args, head, np, torch, binding, synth, HipSession, dev, steps=args.steps, warmup=args.warmup,
                                  layers=args.layers, cpu_s=args.cpu_seconds)
    if args.workload is None and not args.no_extra:
        # the other configurations, briefly (their own default steps; no calibration, no CPU leg): the same measurements per workload
        extra = {}
        for name in ("fork", "mixed", "prefill", "long", "draft", "short"):
            try:
                r = run_attention_workload(args, name, np, torch, binding, synth, HipSession, dev, cpu_s=0.0, calib=False)
            except Exception as e:                                      # a workload that does not fit this box must not take the headline with it
                extra[name] = {"error": f"{type(e).__name__}: {e}"}
                torch.cuda.empty_cache()
                continue
            extra[name] = {k: r[k] for k in ("value", "unit", "ms_per_step", "steps", "us_per_layer", "pct_hbm_peak", "effective_TBps_logical", "lip_steps_per_s",
                                             "step_us_spread", "roofline", "roofline_other", "kernel_breakdown", "host_us_per_step")}
            extra[name]["workload"] = r["config"]["workload"]
            extra[name]["layers_per_step"] = r["config"]["layers_per_step"]
        line["workloads"] = extra
    print(json.dumps(line))


if __name__ == "__main__":
    main()

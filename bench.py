#!/usr/bin/env python3
"""Benchmark of the pred hot path on one MI355X.

A step = one sym_pred_batch call = the whole hot path (descriptor build, the prologue kernel:
descriptor copy + copy-on-write copies + KV append; the decode attention kernel; the merge of
split ranges) over one batch
of the "decode batch" workload: 64 LIPs, 32 Q / 8 KV heads, head dim 128, bf16, contexts
uniform 512..4096, one new token each.  Successive steps rotate over several independent
layer pools (as a real pred walks the model's layers, each with its own KV pages) so that the
KV bytes of a step come from HBM and not from the 256 MB last-level cache.

Prints ONE JSON line: whole-path throughput in algorithmic KV TB/s, plus `roofline` for the
dominant kernel (decode attention, timed with HIP events on its stream inside the timed
region) and `cpu_baseline` (the CPU oracle timed on a bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_TBPS = 8.0       # MI355X published HBM3E peak


def algorithmic_bytes(shape, lengths_after, n_tokens):
    """Bytes one launch must move: every valid KV token of every file once, the appended rows
    written, Q read, O written (fp32), page-table entries read."""
    es = 4 if shape.dtype == "f32" else 2
    kv_tok = 2 * shape.n_kv_heads * shape.head_dim * es
    T = sum(n_tokens)
    kv_read = sum(lengths_after) * kv_tok
    kv_write = T * kv_tok
    q_read = T * shape.n_q_heads * shape.head_dim * es
    o_write = T * shape.n_q_heads * shape.head_dim * 4
    table = sum(-(-L // shape.page_tokens) for L in lengths_after) * 4
    return kv_read + kv_write + q_read + o_write + table


def read_traffic_note(name):
    """HBM traffic per decode launch from the committed counter summary, if there is one."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(wl, budget_s, np):
    """The oracle as it stands on the same workload: all 64 LIPs, one pred step after another
    (each appends one token per LIP and attends), until about `budget_s` seconds have passed."""
    from oracle.driver import OracleSession
    from threadpoolctl import threadpool_info
    osess = OracleSession(wl.shape, wl.n_pages, wl.free_order)
    osess.setup(wl.setup_ops())
    b = wl.batch()
    n_lips = len(b["files"])
    steps, nbytes = 0, 0
    t0 = time.perf_counter()
    while True:
        lengths_after = [osess.model.kv_len(osess.h[f]) + 1 for f in b["files"]]
        osess.pred(b, dtype=np.float32)
        nbytes += algorithmic_bytes(wl.shape, lengths_after, b["n_tokens"])
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s:
            break
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": nbytes / dt / 1e12, "unit": "TB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{steps} pred steps of the same 64-LIP decode batch (append + page gather + fp32 softmax attention "
                      f"per LIP), {dt:.1f} s wall", "lip_steps_per_s": steps * n_lips / dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--layers", type=int, default=4, help="independent layer pools rotated over (cache honesty)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="wall-time budget of the CPU-oracle leg (0 = skip)")
    ap.add_argument("--no-calib", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path is single-GPU; see DESIGN.md for how it would shard); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_25412_amd import binding, synth
    from paper_2510_25412_amd.driver import HipSession

    binding.load()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    wl = synth.config2()
    shape = wl.shape
    n_lips = len(wl.batch_files)

    # ---- build the layer pools (inputs resident in HBM before the timed region)
    ops = list(wl.setup_ops())
    sessions = []
    for _ in range(args.layers):
        s = HipSession(shape, wl.n_pages, wl.free_order, dev, max_lips=n_lips, max_tokens=8192, max_entries=1 << 16)
        s.setup(ops)
        sessions.append(s)
    del ops
    batch = wl.batch()
    dbs = [s.upload_batch(batch) for s in sessions]
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream(dev).cuda_stream

    def step(i):
        s, db = sessions[i % args.layers], dbs[i % args.layers]
        s.ctx.pred_batch(db["kv"], db["n_tokens"], db["q"], db["k_new"], db["v_new"], db["out"], stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    len0 = [sessions[0].ctx.kv_len(h) for h in dbs[0]["kv"]]       # lengths before the timed steps (layer 0)
    for s in sessions:
        s.ctx.profile_enable(1 << binding.K_DECODE)
    t0 = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        step(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dec_ms, dec_n = 0.0, 0
    for s in sessions:
        ms, n = s.ctx.profile_read(binding.K_DECODE)
        dec_ms, dec_n = dec_ms + ms, dec_n + n
        s.ctx.profile_enable(0)

    # mean lengths over the timed steps: each step on a layer adds one token per LIP
    per_layer = args.steps / args.layers
    lengths_after = [L + 1 + (per_layer - 1) / 2 for L in len0]
    step_bytes = algorithmic_bytes(shape, [int(round(x)) for x in lengths_after], [1] * n_lips)
    ms_per_step = wall / args.steps * 1e3
    tbps = step_bytes / (wall / args.steps) / 1e12
    dec_avg_ms = dec_ms / max(dec_n, 1)
    achieved = step_bytes / (dec_avg_ms * 1e-3) / 1e9 if dec_n else None

    # ---- per-kernel breakdown (untimed extra pass) and streaming-read ceiling
    for s in sessions:
        s.ctx.profile_enable(0xf)
    for i in range(args.layers * 10):
        step(i)
    torch.cuda.synchronize()
    breakdown = {}
    for name, kid in (("prologue", binding.K_PROLOGUE), ("decode", binding.K_DECODE), ("merge", binding.K_MERGE)):
        tot, cnt = 0.0, 0
        for s in sessions:
            ms, n = s.ctx.profile_read(kid)
            tot, cnt = tot + ms, cnt + n
        breakdown[name + "_us"] = round(tot / cnt * 1e3, 2) if cnt else None
    for s in sessions:
        s.ctx.profile_enable(0)
    stream_read = None
    if not args.no_calib:
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

    stats = sessions[0].ctx.get_stats()
    for s in sessions:
        s.close()

    cpu = cpu_baseline(wl, args.cpu_seconds, np) if args.cpu_seconds > 0 else None

    line = {
        "metric": "pred-batch attention KV TB/s", "value": round(tbps, 4), "unit": "TB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "decode batch: 64 LIPs, 32Q/8KV heads, head_dim 128, bf16, page 16, contexts U{512..4096}, "
                               "1 new token each; one attention layer per step", "layer_pools_rotated": args.layers,
                   "kv_tokens_per_step": int(sum(lengths_after)), "algorithmic_bytes_per_step": int(step_bytes)},
        "pct_hbm_peak": round(100 * tbps / HBM_PEAK_TBPS, 2),
        "lip_steps_per_s": round(n_lips / (wall / args.steps), 1),
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1) if achieved else None, "peak": HBM_PEAK_TBPS * 1e3,
                     "unit": "GB/s", "frac": round(achieved / (HBM_PEAK_TBPS * 1e3), 4) if achieved else None,
                     "traffic": read_traffic_note("decode_attn_decode_batch_pmc.txt"),
                     "kernel": "decode_attn_kernel<bf16, G=4>", "avg_launch_us": round(dec_avg_ms * 1e3, 2), "launches": dec_n},
        "kernel_breakdown": breakdown,
        "stream_read_TBps": round(stream_read, 3) if stream_read else None,
        "frac_of_stream_read": round(achieved / 1e3 / stream_read, 4) if (achieved and stream_read) else None,
        "cpu_baseline": cpu,
        "host_us_per_step": {"plan_and_descriptor": round(stats["host_ns_plan"] / max(stats["pred_batches"], 1) / 1e3, 2),
                             "whole_call": round(stats["host_ns_pred"] / max(stats["pred_batches"], 1) / 1e3, 2)},
        "pool_stats": {"pages_total": stats["pages_total"], "pages_free": stats["pages_free"]},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

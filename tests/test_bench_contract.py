"""CPU checks of bench.py's bookkeeping: no GPU, no timing."""
import os
import subprocess
import sys

import numpy as np

from paper_2510_25412_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""


def test_algorithmic_bytes_of_a_layer_written_out_by_hand():
    """Per context token and layer: K and V rows of every kv head (2 * Hkv * D * element size = 4096 bytes in every
    configuration of the decode shape); per new token the same again for the rows written, Q read (Hq * D * 2 bytes)
    and the output written (Hq * D * 4 bytes); 4 bytes per page-table entry."""
    shape = synth.Shape(32, 8, 128, 16, synth.BF16)
    assert bench.kv_token_bytes(shape) == 2 * 8 * 128 * 2 == 4096
    kv_tokens, n_tokens, entries = 1000, [1, 1, 3], 70
    T = 5
    want = kv_tokens * 4096 + T * 4096 + T * 32 * 128 * 2 + T * 32 * 128 * 4 + entries * 4
    assert bench.algorithmic_bytes(shape, kv_tokens, n_tokens, entries) == want
    shape32 = synth.Shape(8, 8, 64, 16, synth.F32)
    assert bench.kv_token_bytes(shape32) == 2 * 8 * 64 * 4 == 4096


def test_every_named_workload_has_an_entry_and_the_headline_is_the_decode_batch():
    class Args:
        pool_pages = 1000
    table = bench.workload_table(Args, synth)
    assert set(table) == set(bench.WORKLOADS) and bench.WORKLOADS[0] == "decode"
    gen, layers, steps, warmup, reset, cpu_s, label = table["decode"]
    assert (layers, steps, warmup, reset) == (32, 20, 5, False) and cpu_s > 0
    wl = gen()
    assert len(wl.batch_files) == 64 and set(wl.batch_n) == {1}
    lengths = np.array([wl.lengths[f] for f in wl.batch_files])
    assert lengths.min() >= 512 and lengths.max() <= 4096
    assert (wl.shape.n_q_heads, wl.shape.n_kv_heads, wl.shape.head_dim, wl.shape.page_tokens) == (32, 8, 128, 16)


def test_traffic_note_reads_the_committed_counter_summary():
    got = bench.read_traffic_note("attn_decode_batch_pmc.txt")
    assert got is not None and 5.0e8 < got < 6.5e8          # one launch of the decode batch moves about 560 MB
    assert bench.read_traffic_note("no_such_file.txt") is None

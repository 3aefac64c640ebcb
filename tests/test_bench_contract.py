"""bench.py pieces that need no GPU: the one-GPU rule and the byte accounting of a step."""
import os
import subprocess
import sys

import numpy as np

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_step_bytes_of_a_small_step_by_hand():
    sys.path.insert(0, ROOT)
    import bench
    wl = workloads.make_custom([40, 16, 0, 513], 8, 2, 64, seed=1, append=True)   # 3 staged rows (L > 0)
    sb = bench.step_bytes(wl, include_append=True)
    kv = (40 + 16 + 513) * 2 * 64 * 2 * 2                   # tokens x kv heads x d x bf16 x (K and V)
    pages = 3 + 1 + 0 + 33
    q, out = 4 * 8 * 64 * 2, 4 * 8 * 64 * 4
    assert sb["kv"] == kv
    assert sb["attention"] == kv + q + pages * 4 + 4 * 4 + out      # no split-K scratch in the useful bytes
    assert sb["append"] == 2 * (3 * 2 * 64) * (2 + 2) + 3 * 12
    assert sb["step"] == sb["attention"] + sb["append"]
    # fp8 pools: one byte per element and two scales per (page, head)
    w8 = workloads.make_custom([40, 16], 8, 2, 128, "fp8", seed=2)
    a8 = bench.step_bytes(w8, include_append=False)
    assert a8["kv"] == 56 * 2 * 128 * 1 * 2
    assert a8["attention"] - a8["kv"] == 2 * 8 * 128 * 2 + 4 * 4 + 2 * 4 + 4 * 2 * 8 + 2 * 8 * 128 * 4


def test_partials_of_the_range_pass_by_hand():
    """Two KV heads -> 1024 ranges per head; 5 + 1 + 17 = 23 tiles, one per range: sequences of 5 and 17 tiles are
    cut into as many parts, the one-tile sequence is not cut."""
    sys.path.insert(0, ROOT)
    import bench
    wl = workloads.make_custom([160, 20, 0, 513], 8, 2, 64, seed=1)
    parts, nbytes = bench.range_partials(wl)
    assert parts == (5 + 17) * 2 and nbytes == (5 + 17) * 8 * (64 + 2) * 4

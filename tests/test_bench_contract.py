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


def test_algorithmic_bytes_of_a_small_step_by_hand():
    sys.path.insert(0, ROOT)
    import bench
    wl = workloads.make_custom([40, 16, 0, 513], 8, 2, 64, seed=1, append=True)   # 3 staged rows (L > 0)
    ab = bench.algorithmic_bytes(wl, chunk=256, include_append=True)
    kv = (40 + 16 + 513) * 2 * 64 * 2 * 2                   # tokens x kv heads x d x bf16 x (K and V)
    pages = 3 + 1 + 0 + 33
    chunks = 1 + 1 + 0 + 3
    partials = chunks * 8 * (64 + 2) * 4
    q, out = 4 * 8 * 64 * 2, 4 * 8 * 64 * 4
    assert ab["kv"] == kv
    assert ab["split"] == kv + q + pages * 4 + 4 * 4 + partials
    assert ab["merge"] == partials + out + 4 * 4
    assert ab["append"] == 2 * (3 * 2 * 64) * (2 + 2) + 3 * 12
    assert ab["step"] == ab["split"] + ab["merge"] + ab["append"]
    # one chunk per sequence: the split pass writes the output itself, nothing else moves
    one = bench.algorithmic_bytes(wl, chunk=640, include_append=False, direct=True)
    assert one["merge"] == 0 and one["split"] == kv + q + pages * 4 + 4 * 4 + out
    # fp8 pools: one byte per element and two scales per (page, head)
    w8 = workloads.make_custom([40, 16], 8, 2, 128, "fp8", seed=2)
    a8 = bench.algorithmic_bytes(w8, chunk=256, include_append=False)
    assert a8["kv"] == 56 * 2 * 128 * 1 * 2
    assert a8["split"] - a8["kv"] == 2 * 8 * 128 * 2 + 4 * 4 + 2 * 4 + 4 * 2 * 8 + 2 * 8 * (128 + 2) * 4

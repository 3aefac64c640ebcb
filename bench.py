#!/usr/bin/env python3
"""Decode-attention benchmark for libseamdecode on one MI355X.

One step = one pass of the whole hot path over one batch: kv_append of one
new token per sequence (kv_append_fp8 for fp8 pools), then
paged_decode_attention (split-K pass + merge pass; the shared-prefix aware
entry point for the branching workload).  Inputs are synthetic, seeded and resident in HBM before
the timed region.  Workloads whose K/V pool is small enough to sit in the
256 MB memory-side cache are rotated over several independent pools.

Prints ONE JSON line: whole-step throughput as algorithmic HBM GB/s, the
split-K kernel's roofline figures (HIP-event durations recorded by the library
around its own launches), the read-probe ceiling, and the CPU oracle timed on
the host cores over a bounded sample of the same workload.
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published peak, 8 TB/s
SMALL_POOL_BYTES = 2 << 30  # rotate pools below this footprint


def algorithmic_bytes(wl, chunk, include_append, unique=False, direct=False):
    """Bytes one step must move if every operand travels exactly once.

    With unique=True pages shared by several sequences count once (what a
    prefix-aware pass has to read); otherwise once per sequence that attends
    them (the logical figure).

    Split pass (per launch): every attended K and V element once per
    (sequence, kv head) = sum(L) * token_bytes; q; one table entry per logical
    page; lengths; fp8 scales; the partials it writes.  Merge pass: partials
    read back, out written.  Append: rows read and written once.  With
    direct=True (every sequence is a single chunk and nothing is shared) the
    split pass writes `out` itself: no partials, no merge pass.
    """
    import numpy as np

    lens = wl.context_lens.astype(np.int64)
    kv = (wl.unique_tokens if unique else int(lens.sum())) * wl.token_bytes
    nb = int(((lens + 15) // 16).sum())
    chunks = int(((lens + chunk - 1) // chunk).sum())
    q = wl.batch * wl.num_q_heads * wl.head_dim * 2
    table = nb * 4 + wl.batch * 4
    scales = nb * wl.num_kv_heads * 8 if wl.kv_dtype == "fp8" else 0
    partials = chunks * wl.num_q_heads * (wl.head_dim + 2) * 4
    out = wl.batch * wl.num_q_heads * wl.head_dim * 4
    split = kv + q + table + scales + (out if direct else partials)
    merge = 0 if direct else partials + out + wl.batch * 4
    append = 0
    if include_append and wl.k_new is not None:
        # rows read (bf16) and written (bf16 or fp8 codes), K and V, plus the index arrays
        append = 2 * wl.k_new.size * (2 + wl.kv_elem_bytes) + wl.k_new.shape[0] * 12
    return {"split": split, "merge": merge, "append": append, "step": split + merge + append, "kv": kv}


def stored_traffic(kernel_sources, workload_key):
    """HBM bytes per split launch from the committed counter summary, or None
    when the kernel source has changed since the counters were taken."""
    import glob

    text = ""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        try:
            text += open(path).read() + "\n"
        except OSError:
            pass
    h = hashlib.sha256()
    for s in kernel_sources:
        h.update(open(s, "rb").read())
    tag = f"source_sha256={h.hexdigest()[:16]}"
    for line in text.splitlines():
        if line.startswith("traffic_bytes_per_launch") and tag in line and f"workload={workload_key}" in line:
            return float(line.split("value=")[1].split()[0])
    return None


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(cfg, wall_target=10.0):
    """The oracle (fp64 build, OpenMP over rows) on the host cores over the
    first sequences of the same workload: as many as about `wall_target`
    seconds allow, the whole workload (repeated) if it is shorter than that."""
    import numpy as np

    import oracle
    import workloads

    oracle.build()
    nthreads = oracle.num_threads()

    def run(wl):
        rows = np.int32([(b, h) for b in range(wl.batch) for h in range(wl.num_q_heads)])
        t0 = time.perf_counter()
        oracle.attend_rows(wl.q, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale, rows,
                           wl.k_scales, wl.v_scales, wl.kv_dtype)
        return time.perf_counter() - t0

    lens = workloads.config_lengths(cfg)[0]
    first = workloads.make_config(cfg, batch=1, append=False, threads=nthreads)
    run(first)  # page the library in
    rate = first.attended_tokens / max(run(first), 1e-6)  # tokens/s; one sequence may not fill all threads
    nb, acc = 0, 0
    while nb < len(lens) and acc < rate * wall_target:
        acc += int(lens[nb])
        nb += 1
    wl = workloads.make_config(cfg, batch=nb, append=False, threads=nthreads)
    times = [run(wl)]
    while sum(times) < wall_target and len(times) < 32:
        times.append(run(wl))
    dt = float(np.mean(times))
    return {
        "value": wl.attended_tokens * wl.token_bytes / dt / 1e9, "unit": "GB/s", "cores": nthreads, "kind": "oracle",
        "cpu_model": cpu_model(),
        "sample": f"first {nb} of {len(lens)} sequences of the workload ({wl.attended_tokens} attended tokens, all "
                  f"query heads), fp64 oracle, mean of {len(times)} passes of {dt:.2f} s",
        "attended_kv_tokens_per_s": wl.attended_tokens / dt,
    }


MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 peak


def prefill_main(args):
    """--prefill: the causal multi-query pass (paged_prefill_attention) at a resume shape: every
    sequence re-computes attention for the last `nq` of its L stored tokens.  One step = one call.
    Reported in TFLOP/s of the causal work, 4 * d flops per (query row, visible token) pair."""
    import numpy as np
    import torch

    import paper_2508_11553_amd as sd
    import workloads
    from paper_2508_11553_amd.device import DeviceWorkload, _to_dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sd.load()
    torch.cuda.set_device(0)
    B, L, nq, Hq, Hkv, d = 16, 8192, 2048, 32, 8, 128
    wl = workloads.make_custom([L] * B, Hq, Hkv, d, args.prefill_kv, seed=0)
    dw = DeviceWorkload(wl)
    rng = np.random.default_rng(1)
    q = workloads.f32_to_bf16_bits(rng.standard_normal((B * nq, Hq, d)).astype(np.float32))
    q_start = (np.arange(B + 1) * nq).astype(np.int32)
    q_dev, qs_dev = _to_dev(q, dw.device), _to_dev(q_start, dw.device)
    out = torch.zeros((B * nq, Hq, d), dtype=torch.float32, device=dw.device)
    stream = torch.cuda.current_stream()

    def call(timer=None):
        sd.paged_prefill_attention(dw.shape, q_dev, qs_dev, B * nq, nq, dw.k_pages, dw.v_pages, dw.k_scales,
                                   dw.v_scales, dw.block_table, dw.context_lens, dw.scale, out, stream, timer)

    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        call()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) / args.steps * 1e3
    timer = sd.KernelTimer(args.steps)
    for _ in range(args.steps):
        call(timer)
    torch.cuda.synchronize()
    kernel_ms = float(np.mean(timer.read()[0]))
    pairs = B * Hq * sum(L - nq + i + 1 for i in range(nq))
    flops = 4.0 * d * pairs
    rec = {
        "metric": "causal re-prefill attention over the paged cache, TFLOP/s, 1 GPU",
        "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wl.kv_dtype == "bf16" else "fp8(e4m3fn KV)->bf16", "data": "synthetic",
        "config": {"workload": f"resume: {B} sequences of {L} tokens re-compute their last {nq}", "batch": B,
                   "q_heads": Hq, "kv_heads": Hkv, "head_dim": d, "page_size": 16, "kv_dtype": wl.kv_dtype,
                   "query_rows": B * nq, "row_token_pairs": pairs, "entry_point": "paged_prefill_attention", "seed": 0},
        "kernel_ms": {"prefill": kernel_ms},
        "roofline": {"bound": "mfma", "achieved": flops / (kernel_ms * 1e-3) / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": flops / (kernel_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": None, "kernel": "causal pass (sd::prefill_kernel)", "flops_per_launch": flops},
    }
    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        b0 = slice(0, 1)

        def run(n):  # the last n query rows of sequence 0, all heads
            qs = np.int32([0, n])
            t = time.perf_counter()
            oracle.paged_prefill_attention(q[nq - n:nq], qs, wl.k_pages, wl.v_pages, wl.block_table[b0],
                                           wl.context_lens[b0], wl.scale, wl.k_scales, wl.v_scales, wl.kv_dtype)
            return time.perf_counter() - t

        run(1)
        n = max(1, min(nq, int(10.0 / max(run(2) / 2, 1e-6))))
        dt = run(n)
        sample_pairs = Hq * sum(L - n + i + 1 for i in range(n))
        rec["cpu_baseline"] = {"value": 4.0 * d * sample_pairs / dt / 1e12, "unit": "TFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": f"the last {n} query rows of sequence 0, all heads, fp64 oracle, {dt:.2f} s"}
    print(json.dumps(rec), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=1, help="workload index 0-4 (see workloads.CONFIG_NAMES), default 1")
    ap.add_argument("--chunk", type=int, default=0, help="split-K chunk override (tokens); default: sd_chunk_for_batch of the batch's token count")
    ap.add_argument("--pools", type=int, default=0, help="number of rotating K/V pools (0 = automatic)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-append", action="store_true")
    ap.add_argument("--no-prefix", action="store_true",
                    help="branching workloads: use the plain entry point instead of the shared-prefix aware one")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a device copy of known size (counter calibration for profiler runs)")
    ap.add_argument("--graph", action="store_true",
                    help="replay each step from a captured HIP graph instead of launching its kernels one by one")
    ap.add_argument("--prefill", action="store_true",
                    help="time the causal multi-query pass at a resume shape instead of the decode step")
    ap.add_argument("--prefill-kv", choices=["bf16", "fp8"], default="bf16")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if args.prefill:
        return prefill_main(args)

    import numpy as np
    import torch

    import paper_2508_11553_amd as sd
    import workloads
    from paper_2508_11553_amd.device import DeviceWorkload
    from workloads.gen import draw_extra_pool

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sd.load()
    torch.cuda.set_device(0)
    cfg = args.config
    t_gen = time.perf_counter()
    do_append = not args.no_append
    wl = workloads.make_config(cfg, append=do_append)
    pool_bytes = 2 * wl.k_pages.nbytes
    npools = args.pools or (4 if pool_bytes < SMALL_POOL_BYTES else 1)
    dw = DeviceWorkload(wl, chunk_tokens=args.chunk, balance_for_batch=wl.group_start is not None and not args.no_prefix)
    pools = [(dw.k_pages, dw.v_pages, dw.k_scales, dw.v_scales)]
    for i in range(1, npools):
        k, v, ks, vs = draw_extra_pool(wl, seed=1000 + i)
        dw.set_pool(k, v, ks, vs)
        pools.append((dw.k_pages, dw.v_pages, dw.k_scales, dw.v_scales))
    t_gen = time.perf_counter() - t_gen
    chunk = dw.chunk_tokens()
    prefix_aware = wl.group_start is not None and not args.no_prefix
    direct = not prefix_aware and chunk >= wl.max_context_len  # the library's own condition for skipping the merge
    ab = algorithmic_bytes(wl, chunk, do_append, unique=prefix_aware, direct=direct)
    ab_logical = algorithmic_bytes(wl, chunk, do_append, unique=False, direct=direct)
    stream = torch.cuda.current_stream()

    def step(i, timer=None):
        dw.set_pool(*pools[i % npools])
        if do_append:
            dw.append(stream)
        if prefix_aware:
            dw.attend_prefix(stream, timer)
        else:
            dw.attend(stream, timer)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    run_step = step
    if args.graph:
        # One HIP graph per pool holds the whole step (append, split pass, merge pass); the timed
        # loop replays them in rotation.  The library's launches neither allocate nor synchronise.
        side = torch.cuda.Stream()
        graphs = []
        with torch.cuda.stream(side):
            for i in range(npools):
                g = torch.cuda.CUDAGraph()
                stream, keep = side, stream
                step(i)  # warm-up on the capture stream
                side.synchronize()
                with torch.cuda.graph(g, stream=side):
                    step(i)
                stream = keep
                graphs.append(g)
        torch.cuda.synchronize()
        run_step = lambda i: graphs[i % npools].replay()
        for i in range(npools):
            run_step(i)
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        run_step(i)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3

    # the same steps again with the library's HIP events around each kernel
    timer = sd.KernelTimer(args.steps)
    for i in range(args.steps):
        step(i, timer)
    torch.cuda.synchronize()
    split_ms, merge_ms = timer.read()
    timer.close()
    split_avg = float(np.mean(split_ms))
    merge_avg = float(np.mean(merge_ms))

    # read-only probe over the same walk: the ceiling of this access pattern
    from paper_2508_11553_amd.binding import probe_read, probe_sink_words
    sink = torch.zeros(probe_sink_words(dw.shape), dtype=torch.int32, device=dw.device)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    nprobe = max(10, min(args.steps, 50))
    for i in range(5):
        probe_read(dw.shape, *pools[i % npools], dw.block_table, dw.context_lens, sink, stream)
    ev[0].record(stream)
    for i in range(nprobe):
        probe_read(dw.shape, *pools[i % npools], dw.block_table, dw.context_lens, sink, stream)
    ev[1].record(stream)
    torch.cuda.synchronize()
    probe_ms = ev[0].elapsed_time(ev[1]) / nprobe

    if args.copy_calibration:
        # 1 GiB read + 1 GiB written by a plain device-to-device copy: the byte counters of a
        # profiler run are scaled by what they report for this known transfer
        src_t = torch.empty(1 << 28, dtype=torch.int32, device=dw.device).fill_(1)
        dst_t = torch.empty_like(src_t)
        for _ in range(3):
            dst_t.copy_(src_t)
        torch.cuda.synchronize()
        del src_t, dst_t

    value = ab["step"] / (ms_per_step * 1e-3) / 1e9
    # MFMA flops the split pass issues: QK^T and PV on 16-row tiles, 2 * 16 * d * 2 flops per token and KV head;
    # plain items run one tile per (sequence, KV head), shared items one per 16 / G sequences
    issued_tokens = float(wl.attended_tokens) if not prefix_aware else (
        float(wl.attended_tokens - int(wl.shared_len.astype(np.int64).sum())) +
        float(wl.shared_len.astype(np.int64).sum()) * (wl.num_q_heads // wl.num_kv_heads) / 16.0)
    issued_flops = issued_tokens * wl.num_kv_heads * 64.0 * wl.head_dim
    achieved = ab["split"] / (split_avg * 1e-3) / 1e9
    src = [os.path.join(ROOT, "paper_2508_11553_amd", "csrc", f) for f in ("attn_split.hip", "attn_tile.h", "kernels.h")]
    rec = {
        "metric": "decode-attention HBM GB/s (% of MI355X peak) + attended KV tokens/sec, 1 GPU",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.kv_dtype == "bf16" else "fp8(e4m3fn KV)->bf16", "data": "synthetic",
        "config": {
            "workload": f"configs[{cfg}] {wl.name}", "batch": wl.batch, "q_heads": wl.num_q_heads,
            "kv_heads": wl.num_kv_heads, "head_dim": wl.head_dim, "page_size": 16, "kv_dtype": wl.kv_dtype,
            "attended_tokens": wl.attended_tokens, "unique_tokens": wl.unique_tokens, "chunk_tokens": chunk,
            "pools_rotated": npools, "entry_point": "paged_decode_attention_prefix" if prefix_aware else
            "paged_decode_attention", "append_rows_per_step": int(wl.k_new.shape[0]) if do_append else 0, "seed": 0,
            "merge_pass": not direct,
        },
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "attended_kv_tokens_per_s": wl.attended_tokens / (ms_per_step * 1e-3),
        "attended_kv_head_tokens_per_s": wl.attended_tokens * wl.num_kv_heads / (ms_per_step * 1e-3),
        "step_bytes": ab, "logical_GBps": ab_logical["step"] / (ms_per_step * 1e-3) / 1e9,
        "kernel_ms": {"split": split_avg, "merge": merge_avg, "split_p10_p50_p90":
                      [float(np.percentile(split_ms, p)) for p in (10, 50, 90)]},
        "probe": {"ms": probe_ms, "GBps": ab["kv"] / (probe_ms * 1e-3) / 1e9,
                  "what": "read-only walk of the same pages, 16-byte loads"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": stored_traffic(src, f"configs[{cfg}]"),
                     "kernel": "split pass (sd::split_*_kernel)", "algorithmic_bytes_per_launch": ab["split"]},
        "mfma": {"issued_tflops": issued_flops / (split_avg * 1e-3) / 1e12,
                 "useful_tflops": 4.0 * wl.head_dim * wl.num_q_heads * wl.attended_tokens / (split_avg * 1e-3) / 1e12,
                 "peak_tflops": MFMA_BF16_PEAK_TFLOPS,
                 "issued_frac_of_peak": issued_flops / (split_avg * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                 "what": "split pass; issued = 64*d flops per (token, KV head): both products on 16-row tiles "
                         "(rows beyond G are padding); shared-prefix tokens counted once per 16 rows"},
        "input_generation_s": t_gen,
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(cfg)
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()

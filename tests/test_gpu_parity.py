"""Parity of the HIP path against the CPU oracle, through the C ABI (GPU only).

Tolerances for bf16 inputs with fp32 accumulation: max abs error <= 1e-2 and
mean abs error <= 1e-3 against the fp64 oracle.  Outputs are O(0.05) at these
lengths, so anything above the alarm level below is treated as a bug even
though it would pass.  Integer/byte work (kv_append) is compared bit for bit.
"""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3
# Softmax weights are rounded to bf16 (relative error 2^-9 each) before the
# weighted sum, so a row's error scales with the size of its output: O(1) for
# a handful of tokens, O(0.05) for thousands.  The alarm follows that.
ALARM_ABS, ALARM_REL = 3e-4, 2.0 ** -8


@pytest.fixture(scope="module")
def sd():
    import torch
    assert torch.cuda.is_available()
    import paper_2508_11553_amd as m
    m.load()
    return m


def device_workload(wl, **kw):
    from device_workload import DeviceWorkload
    return DeviceWorkload(wl, **kw)


def gpu_attend(wl, **kw):
    import torch
    dw = device_workload(wl, **kw)
    out = dw.attend()
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_full(wl, k_pages=None, v_pages=None):
    return oracle.paged_decode_attention(wl.q, wl.k_pages if k_pages is None else k_pages,
                                         wl.v_pages if v_pages is None else v_pages, wl.block_table,
                                         wl.context_lens, wl.scale, wl.k_scales, wl.v_scales, wl.kv_dtype)


def check(got, ref, max_abs=MAX_ABS, mean_abs=MEAN_ABS, alarm_scale=1.0):
    assert not np.isnan(got).any(), "NaN in the GPU output"
    err = np.abs(got.astype(np.float64) - ref)
    assert err.max() <= max_abs and err.mean() <= mean_abs, (err.max(), err.mean())
    alarm = alarm_scale * (ALARM_ABS + ALARM_REL * np.abs(ref).max(axis=-1, keepdims=True))
    worst = (err / alarm).max()
    assert worst <= 1.0, f"passes the stated tolerance but is suspiciously large: {worst:.2f} x the alarm level"


def test_config0_tiny_paged_decode(sd):
    wl = workloads.make_config(0)
    check(gpu_attend(wl), oracle_full(wl))


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 1), (8, 2), (28, 4), (16, 2), (32, 2), (17, 1), (32, 1), (40, 2), (64, 1)])
def test_group_sizes_and_head_dims(sd, Hq, Hkv, d):
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 300, 511, 512, 513, 1025]
    wl = workloads.make_custom(lens, Hq, Hkv, d, seed=100 + Hq + d)
    check(gpu_attend(wl), oracle_full(wl))


@pytest.mark.parametrize("chunk", [128, 256, 512, 1024])
def test_chunk_sizes_and_ragged_tails(sd, chunk):
    lens = [chunk - 1, chunk, chunk + 1, 3 * chunk + 7, 2 * chunk, 5, 2 * chunk + 16, 2 * chunk + 17]
    wl = workloads.make_custom(lens, 8, 2, 128, seed=200 + chunk)
    check(gpu_attend(wl, chunk_tokens=chunk), oracle_full(wl))


def test_results_do_not_depend_on_chunk_beyond_rounding(sd):
    wl = workloads.make_custom([700, 1500, 64, 4000], 28, 4, 128, seed=7)
    a, b = gpu_attend(wl, chunk_tokens=128), gpu_attend(wl, chunk_tokens=1024)
    # different chunkings round the bf16 weights against different running maxima
    assert np.abs(a - b).max() <= ALARM_ABS + ALARM_REL * np.abs(a).max()


def test_two_runs_are_bitwise_equal(sd):
    wl = workloads.make_custom([700, 1500, 64, 4000], 28, 4, 128, seed=8)
    assert np.array_equal(gpu_attend(wl), gpu_attend(wl))


def test_zero_length_sequences_give_zero_rows(sd):
    wl = workloads.make_custom([0, 40, 0, 513], 8, 2, 64, seed=9)
    got = gpu_attend(wl)
    assert np.array_equal(got[0], np.zeros_like(got[0])) and np.array_equal(got[2], np.zeros_like(got[2]))
    check(got, oracle_full(wl))


@pytest.mark.parametrize("kv_dtype,d", [("bf16", 64), ("bf16", 128), ("fp8", 128), ("fp8", 64)])
@pytest.mark.parametrize("min_range", [0, 128, 640, 4096])
def test_whole_and_cut_sequences_in_one_launch(sd, kv_dtype, d, min_range):
    """Ranges of at least `min_range` tokens: from one tile per wave (every sequence cut into many partials
    that the last wave combines) to one wave holding the whole batch (every sequence written by the wave that
    walked it).  Empty sequences must get their zero rows and every element of `out` must be written."""
    import torch
    lens = [0, 40, 1, 513, 0, 640, 639, 16, 17, 0]
    wl = workloads.make_custom(lens, 8, 2, d, kv_dtype, seed=12, max_blocks_per_seq=41)
    dw = device_workload(wl, chunk_tokens=min_range)
    dw.out.fill_(float("nan"))
    got = dw.attend().clone()
    torch.cuda.synchronize()
    g = got.cpu().numpy()
    assert not g[0].any() and not g[4].any() and not g[9].any()
    (check_fp8 if kv_dtype == "fp8" else check)(g, oracle_full(wl))
    # a second call on the same workspace (now holding the first call's partials) gives the same bits
    dw.out.fill_(float("nan"))
    again = dw.attend()
    torch.cuda.synchronize()
    assert torch.equal(again, got)


@pytest.mark.parametrize("Hq,Hkv,d,kv_dtype", [(8, 2, 128, "bf16"), (16, 1, 64, "bf16"), (8, 2, 128, "fp8"), (40, 2, 128, "bf16"), (8, 2, 64, "fp8")])
@pytest.mark.parametrize("min_range", [0, 128, 256, 384, 640])
def test_parts_handed_over_inside_a_workgroup(sd, Hq, Hkv, d, kv_dtype, min_range):
    """The four waves of a workgroup walk neighbouring ranges and hand their parts of one sequence to the first of
    them through LDS.  Sequences of 1 .. 64 tiles against ranges of 1, 4, 8, 12 and 20 tiles put the sequence borders
    at every position of a workgroup's four ranges: runs that hold a whole sequence (written directly), runs that leave one
    part, runs that end because the next range holds a border, sequences spread over several workgroups."""
    import torch
    lens = [32 * k - (k % 3) for k in (1, 2, 3, 4, 5, 7, 8, 9, 12, 13, 16, 17, 23, 29, 31, 40, 47, 64)] + [1, 33, 0, 449, 97, 225, 31, 161]
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=77 + min_range + d)
    dw = device_workload(wl, chunk_tokens=min_range)
    dw.out.fill_(float("nan"))
    got = dw.attend().clone()
    torch.cuda.synchronize()
    (check_fp8 if kv_dtype == "fp8" else check)(got.cpu().numpy(), oracle_full(wl))
    dw.out.fill_(float("nan"))
    assert torch.equal(dw.attend(), got)


def test_more_sequences_than_ranges(sd):
    """1300 short sequences: more than the grid has ranges per head, so the merge pass works from the records the
    range pass leaves per range; ranges of twelve tiles cut many of the sequences, inside workgroups and between them."""
    import torch
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(0, 600, size=1300)]
    wl = workloads.make_custom(lens, 4, 2, 64, seed=78)
    dw = device_workload(wl, chunk_tokens=128)
    dw.out.fill_(float("nan"))
    got = dw.attend().clone()
    torch.cuda.synchronize()
    check(got.cpu().numpy(), oracle_full(wl))
    dw.out.fill_(float("nan"))
    assert torch.equal(dw.attend(), got)


@pytest.mark.parametrize("batch", [4096, 4097])
def test_batches_at_the_limit_of_the_range_pass(sd, batch):
    """4096 sequences is the most the range pass lays out in one workgroup's LDS; one more takes the chunked
    passes.  Both sides of the limit against the oracle, with empty sequences and a few long ones among them."""
    import torch
    rng = np.random.default_rng(9)
    lens = [int(x) for x in rng.integers(0, 90, size=batch)]
    for i in (0, 17, batch - 1):
        lens[i] = 700
    wl = workloads.make_custom(lens, 4, 2, 64, seed=90)
    dw = device_workload(wl, chunk_tokens=128)
    dw.out.fill_(float("nan"))
    got = dw.attend().clone()
    torch.cuda.synchronize()
    check(got.cpu().numpy(), oracle_full(wl))


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("chunk", [128, 512])
def test_lengths_outside_the_bound_are_clamped(sd, chunk, kv_dtype):
    """context_lens above max_context_len count as max_context_len, negative ones as 0 (zero rows), in the
    path that cuts sequences across waves (ranges of 128 tokens) and with ranges that hold whole sequences."""
    import torch
    from device_workload import _to_dev
    true_lens = np.int32([40, 700, 513, 16, 300, 1500, 512])
    wl = workloads.make_custom(true_lens, 8, 2, 128, kv_dtype, seed=21)
    dw = device_workload(wl, chunk_tokens=chunk)
    dw.shape.max_context_len = 512
    dw.ws_bytes = sd.workspace_bytes(dw.shape)
    dw.workspace = torch.empty(dw.ws_bytes, dtype=torch.uint8, device=dw.device)
    passed = np.int32([-3, 700, 513, 16, -2 ** 31, 1500, 512])
    dw.context_lens = _to_dev(passed, dw.device)
    dw.out.fill_(float("nan"))
    got = dw.attend()
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    wl.context_lens = np.clip(passed, 0, 512).astype(np.int32)
    (check_fp8 if kv_dtype == "fp8" else check)(got, oracle_full(wl))
    assert not got[0].any() and not got[4].any()


def test_length_one_returns_v_row_bit_exact(sd):
    wl = workloads.make_custom([1, 1, 1, 1, 1], 8, 2, 128, seed=10)
    got = gpu_attend(wl)
    V = workloads.bf16_bits_to_f32(wl.v_pages)
    for b in range(5):
        for h in range(8):
            assert np.array_equal(got[b, h], V[wl.block_table[b, 0], h // 4, 0])


def test_constant_v_returns_the_constant(sd):
    wl = workloads.make_custom([1, 5, 33, 200, 1300], 8, 2, 64, seed=11)
    c = workloads.f32_to_bf16_bits(np.float32([0.37]))[0]
    keep = wl.v_pages == workloads.BF16_NAN_BITS  # leave the poison where it is
    wl.v_pages[~keep] = c
    got = gpu_attend(wl)
    assert np.abs(got - workloads.bf16_bits_to_f32(np.uint16([c]))[0]).max() <= 1e-6


@pytest.mark.parametrize("min_range", [0, 4096])
def test_fp8_constant_v_returns_the_constant(sd, min_range):
    """fp8 pools: pages with different (power-of-two) V scales whose codes all decode to 0.5.  The weight sum runs
    over the rounded weights the product uses, so the constant comes back to fp32 rounding; both with sequences cut
    across waves and with one workgroup per sequence."""
    wl = workloads.make_custom([1, 5, 33, 200, 1300], 8, 2, 128, "fp8", seed=11, poison=False)
    codes = {0.25: 0x40, 0.5: 0x38, 2.0: 0x28}      # 2.0, 1.0, 0.25 in e4m3fn: code value x scale = 0.5
    for p in range(wl.num_pages):
        s = (0.25, 0.5, 2.0)[p % 3]
        wl.v_scales[p, :] = np.float32(s)
        wl.v_pages[p] = codes[s]
    got = gpu_attend(wl, chunk_tokens=min_range)
    assert np.abs(got - 0.5).max() <= 1e-6


def test_poisoned_slots_and_table_entries_are_never_read(sd):
    a = workloads.make_custom([3, 47, 130, 512, 529], 8, 2, 128, seed=12, poison=True)
    c = workloads.make_custom([3, 47, 130, 512, 529], 8, 2, 128, seed=12, poison=False)
    ga, gc = gpu_attend(a), gpu_attend(c)
    assert not np.isnan(ga).any() and np.array_equal(ga, gc)


def test_permuting_physical_pages_changes_no_bit(sd):
    lens = [100, 31, 257, 1100]
    a = workloads.make_custom(lens, 8, 2, 64, seed=13, permute=True)
    c = workloads.make_custom(lens, 8, 2, 64, seed=13, permute=False)
    # same logical content?  The generator draws pools in physical order, so rebuild c's pool from a's.
    k = np.empty_like(c.k_pages); v = np.empty_like(c.v_pages)
    k[:] = workloads.BF16_NAN_BITS; v[:] = workloads.BF16_NAN_BITS
    for b, L in enumerate(lens):
        for j in range((L + 15) // 16):
            k[c.block_table[b, j]] = a.k_pages[a.block_table[b, j]]
            v[c.block_table[b, j]] = a.v_pages[a.block_table[b, j]]
    c.k_pages, c.v_pages, c.q = k, v, a.q
    assert np.array_equal(gpu_attend(a), gpu_attend(c))


def test_shared_prefix_pages_equal_private_copies(sd):
    lens = np.array([300, 277, 811, 290])
    wl = workloads.make_custom(lens, 8, 2, 128, seed=14, session_of=[0, 0, 0, 1], prefix_len=[200, 200, 200, 96])
    shared = gpu_attend(wl)
    nbs = (lens + 15) // 16
    table = np.full_like(wl.block_table, -1)
    nxt = 0
    for b in range(4):
        table[b, :nbs[b]] = np.arange(nxt, nxt + nbs[b]); nxt += nbs[b]
    k = np.zeros((nxt,) + wl.k_pages.shape[1:], wl.k_pages.dtype); v = k.copy()
    for b in range(4):
        k[table[b, :nbs[b]]] = wl.k_pages[wl.block_table[b, :nbs[b]]]
        v[table[b, :nbs[b]]] = wl.v_pages[wl.block_table[b, :nbs[b]]]
    ref = oracle_full(wl)
    wl.k_pages, wl.v_pages, wl.block_table, wl.num_pages = k, v, table, nxt
    private = gpu_attend(wl)
    assert np.array_equal(shared, private)
    check(shared, ref)


def test_kv_append_is_bit_exact_and_append_then_attend_matches(sd):
    import torch
    wl = workloads.make_custom([20, 33, 512, 513, 1, 16, 17], 8, 2, 128, seed=15, append=True)
    dw = device_workload(wl)
    dw.append()
    out = dw.attend()
    torch.cuda.synchronize()
    k_gpu, v_gpu = dw.pools_to_host()
    k_ref, v_ref = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_append(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, k_ref, v_ref, wl.block_table)
    assert np.array_equal(k_gpu, k_ref) and np.array_equal(v_gpu, v_ref)
    check(out.cpu().numpy(), oracle_full(wl, k_ref, v_ref))


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 128), (28, 4, 128), (8, 1, 64), (32, 1, 128)])
@pytest.mark.parametrize("min_range", [0, 256, 4096])
def test_append_and_attend_in_one_call(sd, Hq, Hkv, d, min_range):
    """paged_decode_attention_append = kv_append of every sequence's newest token + attention over it: pool bytes equal
    the oracle's append bit for bit, the output matches the oracle run over the appended pool.  Lengths put the
    newest token first in its page, last in its page, alone in the sequence, first of a new tile; one sequence is
    empty.  Ranges of 4096 tokens cover every sequence, which takes the path that launches the append separately."""
    import torch
    lens = [1, 2, 16, 17, 32, 33, 34, 0, 64, 65, 513, 700, 1025, 1]
    wl = workloads.make_custom(lens, Hq, Hkv, d, seed=500 + Hq + d, append=True)
    dw = device_workload(wl, chunk_tokens=min_range)
    dw.out.fill_(float("nan"))
    out = dw.append_and_attend()
    torch.cuda.synchronize()
    k_ref, v_ref = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_append(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, k_ref, v_ref, wl.block_table)
    k_gpu, v_gpu = dw.pools_to_host()
    assert np.array_equal(k_gpu, k_ref) and np.array_equal(v_gpu, v_ref)
    got = out.cpu().numpy()
    check(got, oracle_full(wl, k_ref, v_ref))
    assert not got[7].any()
    # a sequence of one token returns that token's V row exactly
    V = workloads.bf16_bits_to_f32(wl.v_new)
    for b in (0, 13):
        j = int(np.nonzero(wl.seq_ids == b)[0][0])
        for h in range(Hq):
            assert np.array_equal(got[b, h], V[j, h // (Hq // Hkv)])
    # and the pool now serves the plain call with the same result up to rounding order
    plain = dw.attend().cpu().numpy()
    assert np.abs(got - plain).max() <= ALARM_ABS + ALARM_REL * np.abs(plain).max()


def test_append_and_attend_rejects_fp8_pools(sd):
    wl = workloads.make_custom([40, 17], 16, 2, 128, "fp8", seed=501)
    dw = device_workload(wl)
    with pytest.raises(sd.SeamDecodeError) as e:
        sd.paged_decode_attention_append(dw.shape, dw.q, dw.q, dw.q, dw.k_pages, dw.v_pages, dw.block_table,
                                         dw.context_lens, dw.scale, dw.out, dw.workspace, dw.ws_bytes)
    assert e.value.code == -2


def test_pool_built_token_by_token_with_kv_append(sd):
    """Resume: rebuild a paused sequence's cache from its stored rows, then attend."""
    import torch
    from paper_2508_11553_amd import binding
    wl = workloads.make_custom([37, 5, 64], 4, 2, 64, seed=16, poison=False)
    dw = device_workload(wl)
    ref = dw.attend().clone()
    # every valid token as one append row, in one bulk call, into an empty pool
    rows_k, rows_v, seqs, poss = [], [], [], []
    for b, L in enumerate(wl.context_lens):
        for t in range(L):
            p, s = wl.block_table[b, t // 16], t % 16
            rows_k.append(wl.k_pages[p, :, s]); rows_v.append(wl.v_pages[p, :, s]); seqs.append(b); poss.append(t)
    from device_workload import _to_dev
    kn, vn = _to_dev(np.stack(rows_k), dw.device), _to_dev(np.stack(rows_v), dw.device)
    si, po = _to_dev(np.int32(seqs), dw.device), _to_dev(np.int32(poss), dw.device)
    dw.k_pages.zero_(); dw.v_pages.zero_()
    binding.kv_append(dw.shape, kn, vn, si, po, len(seqs), dw.k_pages, dw.v_pages, dw.block_table)
    out = dw.attend()
    torch.cuda.synchronize()
    assert torch.equal(out, ref)


def test_workspace_too_small_and_bad_arguments_on_device(sd):
    import ctypes
    wl = workloads.make_custom([40], 8, 2, 64, seed=17)
    dw = device_workload(wl)
    with pytest.raises(sd.SeamDecodeError) as e:
        sd.paged_decode_attention(dw.shape, dw.q, dw.k_pages, dw.v_pages, None, None, dw.block_table,
                                  dw.context_lens, dw.scale, dw.out, dw.workspace, dw.ws_bytes - 1)
    assert e.value.code == -3
    with pytest.raises(sd.SeamDecodeError) as e:
        sd.paged_decode_attention(dw.shape, dw.q, dw.k_pages, None, None, None, dw.block_table,
                                  dw.context_lens, dw.scale, dw.out, dw.workspace, dw.ws_bytes)
    assert e.value.code == -1


def test_runs_on_a_side_stream(sd):
    import torch
    wl = workloads.make_custom([700, 64], 8, 2, 128, seed=18)
    dw = device_workload(wl)
    ref = dw.attend().clone()
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    out2 = torch.zeros_like(ref)
    with torch.cuda.stream(s):
        dw.attend(stream=s, out=out2)
    s.synchronize()
    assert torch.equal(out2, ref)


def test_kernel_timer_reports_the_kernels_of_a_call(sd):
    """Both entry points run two kernels and report both durations."""
    wl = workloads.make_custom([700, 650, 64], 8, 2, 128, seed=19, session_of=[0, 0, 1], prefix_len=[512, 512, 0])
    dw = device_workload(wl)
    t = sd.KernelTimer(8)
    for _ in range(3):
        dw.attend(timer=t)
    first, second = t.read()
    assert len(first) == 3 and all(x > 0 for x in first) and all(x > 0 for x in second)
    t.reset()
    for _ in range(2):
        dw.attend_prefix(timer=t)
    split, merge = t.read()
    assert len(split) == 2 and all(x > 0 for x in split) and all(x > 0 for x in merge)
    t.close()


# ---------------------------------------------------------------- full-size configurations
def oracle_all_rows(wl, k_pages=None, v_pages=None, k_scales=None, v_scales=None):
    """Every (sequence, head) row of a full-size workload through the fp64 oracle; prints what it cost."""
    import time
    t = time.perf_counter()
    ref = oracle.paged_decode_attention(wl.q, wl.k_pages if k_pages is None else k_pages,
                                        wl.v_pages if v_pages is None else v_pages, wl.block_table, wl.context_lens,
                                        wl.scale, wl.k_scales if k_scales is None else k_scales,
                                        wl.v_scales if v_scales is None else v_scales, wl.kv_dtype)
    print(f"[oracle] {wl.name}: {wl.batch * wl.num_q_heads} rows, {wl.attended_tokens} attended tokens, "
          f"{time.perf_counter() - t:.1f} s on {oracle.num_threads()} threads", flush=True)
    return ref


@pytest.mark.parametrize("cfg", [1, 2])
def test_full_size_config_every_row(sd, cfg):
    """The step bench.py times at these workloads: one call that appends every sequence's newest token and attends."""
    import torch
    wl = workloads.make_config(cfg, append=True)
    dw = device_workload(wl)
    out = dw.append_and_attend()
    torch.cuda.synchronize()
    oracle.kv_append(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, wl.k_pages, wl.v_pages, wl.block_table)  # in place on the host copy
    k_gpu, v_gpu = dw.pools_to_host()
    assert np.array_equal(k_gpu, wl.k_pages) and np.array_equal(v_gpu, wl.v_pages)
    ref = oracle_all_rows(wl)
    check(out.cpu().numpy(), ref)
    check(dw.attend().cpu().numpy(), ref)   # the plain call over the same pool


def test_full_size_branching_mix_with_append(sd):
    import torch
    wl = workloads.make_config(3)
    dw = device_workload(wl, balance_for_batch=True)
    dw.append()
    out = dw.attend()
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    k_ref, v_ref = wl.k_pages, wl.v_pages  # append in place on the host copy
    oracle.kv_append(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, k_ref, v_ref, wl.block_table)
    k_gpu, v_gpu = dw.pools_to_host()
    assert np.array_equal(k_gpu, k_ref) and np.array_equal(v_gpu, v_ref)
    ref = oracle_all_rows(wl, k_ref, v_ref)
    check(got, ref)
    # the shared-prefix aware entry point on the same step (the one bench.py times at this workload)
    out2 = dw.attend_prefix()
    torch.cuda.synchronize()
    check(out2.cpu().numpy(), ref)


# ---------------------------------------------------------------- fp8 e4m3fn KV
# Tolerance for fp8 KV: max abs error <= 5e-2 against the oracle that applies
# the same dequantisation (code * scale).  The device decodes the codes
# exactly, so the same alarm as for bf16 applies on top.
FP8_MAX_ABS = 5e-2


def check_fp8(got, ref, alarm_scale=1.0):
    assert not np.isnan(got).any()
    err = np.abs(got.astype(np.float64) - ref)
    assert err.max() <= FP8_MAX_ABS, err.max()
    alarm = alarm_scale * (ALARM_ABS + 2 * ALARM_REL * np.abs(ref).max(axis=-1, keepdims=True))
    assert (err / alarm).max() <= 1.0, f"suspiciously large: {(err / alarm).max():.2f} x the alarm level"


@pytest.mark.parametrize("Hq,Hkv", [(8, 1), (8, 2), (64, 8), (28, 4), (16, 1)])
def test_fp8_small_shapes(sd, Hq, Hkv):
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 64, 65, 127, 129, 300, 511, 512, 513, 1025, 2049]
    wl = workloads.make_custom(lens, Hq, Hkv, 128, "fp8", seed=300 + Hq)
    check_fp8(gpu_attend(wl), oracle_full(wl))


@pytest.mark.parametrize("chunk", [128, 512, 2048])
def test_fp8_chunk_sizes(sd, chunk):
    lens = [chunk - 1, chunk, chunk + 1, 3 * chunk + 7, 5, 2 * chunk + 17]
    wl = workloads.make_custom(lens, 16, 2, 128, "fp8", seed=320 + chunk)
    check_fp8(gpu_attend(wl, chunk_tokens=chunk), oracle_full(wl))


def test_fp8_every_code_decodes_exactly_on_the_device(sd):
    """Length-1 sequences return their V row: with power-of-two scales the
    output must equal code * scale bit for bit, for all 254 finite codes.
    This pins the fp8 flavour (OCP e4m3fn, not fnuz) on the device."""
    wl = workloads.make_custom([1, 1, 1, 1], 2, 2, 128, "fp8", seed=330, poison=False)
    codes = np.arange(256, dtype=np.uint8)
    codes[0x7F] = 0; codes[0xFF] = 0x80  # the two NaN codes
    for b in range(4):
        p = wl.block_table[b, 0]
        wl.v_pages[p, 0, 0, :] = codes[:128] if b % 2 == 0 else codes[128:]
        wl.v_pages[p, 1, 0, :] = codes[128:] if b % 2 == 0 else codes[:128]
    wl.v_scales[:] = np.float32(2.0 ** -5); wl.k_scales[:] = np.float32(0.25)
    got = gpu_attend(wl)
    table = np.array([oracle.e4m3fn_to_float(int(c)) for c in codes], dtype=np.float32) * np.float32(2.0 ** -5)
    for b in range(4):
        lo, hi = (table[:128], table[128:]) if b % 2 == 0 else (table[128:], table[:128])
        assert np.array_equal(got[b, 0], lo) and np.array_equal(got[b, 1], hi)


def test_fp8_k_codes_decode_like_the_oracle(sd):
    """Two tokens with one-hot queries: the weights are a logistic of the
    difference of two decoded K codes, for every pair of adjacent codes."""
    B = 126
    wl = workloads.make_custom([2] * B, 1, 1, 128, "fp8", seed=331, poison=False)
    q = np.zeros((B, 1, 128), np.float32); q[:, 0, 5] = 1.0
    wl.q = workloads.f32_to_bf16_bits(q)
    wl.scale = 1.0
    for b in range(B):
        p = wl.block_table[b, 0]
        wl.k_pages[p, 0, 0, 5] = b; wl.k_pages[p, 0, 1, 5] = b + 1  # codes 0..126, positive range
        wl.k_scales[p, 0] = np.float32(2.0 ** -4)
    check_fp8(gpu_attend(wl), oracle_full(wl))


def test_fp8_poison_is_never_read(sd):
    a = workloads.make_custom([3, 47, 130, 512, 529], 16, 2, 128, "fp8", seed=332, poison=True)
    c = workloads.make_custom([3, 47, 130, 512, 529], 16, 2, 128, "fp8", seed=332, poison=False)
    ga, gc = gpu_attend(a), gpu_attend(c)
    assert not np.isnan(ga).any() and np.array_equal(ga, gc)


@pytest.mark.parametrize("Hq,Hkv", [(8, 1), (8, 2), (64, 8), (28, 4), (16, 1), (40, 2), (1, 1)])
@pytest.mark.parametrize("min_range", [0, 128, 4096])
def test_fp8_head_dim_64(sd, Hq, Hkv, min_range):
    """fp8 pools with 64-wide heads: the range pass (ranges of one tile and of 128 tokens) and the
    workgroup-per-sequence kernel (ranges that cover every sequence), on lengths around page and tile edges."""
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 64, 65, 127, 129, 300, 511, 512, 513, 1025, 2049, 0]
    wl = workloads.make_custom(lens, Hq, Hkv, 64, "fp8", seed=340 + Hq)
    check_fp8(gpu_attend(wl, chunk_tokens=min_range), oracle_full(wl))


def test_fp8_head_dim_64_every_code_decodes_exactly_on_the_device(sd):
    """As for 128-wide heads: length-1 sequences with power-of-two scales return code * scale bit for bit,
    all 254 finite codes, spread over four rows of 64."""
    wl = workloads.make_custom([1, 1, 1, 1], 1, 1, 64, "fp8", seed=341, poison=False)
    codes = np.arange(256, dtype=np.uint8)
    codes[0x7F] = 0; codes[0xFF] = 0x80  # the two NaN codes
    for b in range(4):
        wl.v_pages[wl.block_table[b, 0], 0, 0, :] = codes[64 * b:64 * b + 64]
    wl.v_scales[:] = np.float32(2.0 ** -5); wl.k_scales[:] = np.float32(0.25)
    got = gpu_attend(wl)
    table = np.array([oracle.e4m3fn_to_float(int(c)) for c in codes], dtype=np.float32) * np.float32(2.0 ** -5)
    for b in range(4):
        assert np.array_equal(got[b, 0], table[64 * b:64 * b + 64])


def test_fp8_head_dim_64_k_codes_decode_like_the_oracle(sd):
    """One-hot queries at every d in turn: the two-token weights are a logistic of the difference of two
    decoded K codes, so a K element that lands at the wrong d, or a wrong code, shows."""
    B = 128
    wl = workloads.make_custom([2] * B, 1, 1, 64, "fp8", seed=342, poison=False)
    q = np.zeros((B, 1, 64), np.float32)
    for b in range(B):
        q[b, 0, b % 64] = 1.0
    wl.q = workloads.f32_to_bf16_bits(q)
    wl.scale = 1.0
    for b in range(B):
        p = wl.block_table[b, 0]
        wl.k_pages[p, 0, 0, b % 64] = (3 * b) % 127; wl.k_pages[p, 0, 1, b % 64] = (3 * b + 5) % 127
        wl.k_scales[p, 0] = np.float32(2.0 ** -4)
    check_fp8(gpu_attend(wl), oracle_full(wl))


def test_fp8_head_dim_64_poison_is_never_read(sd):
    a = workloads.make_custom([3, 47, 130, 512, 529], 16, 2, 64, "fp8", seed=343, poison=True)
    c = workloads.make_custom([3, 47, 130, 512, 529], 16, 2, 64, "fp8", seed=343, poison=False)
    ga, gc = gpu_attend(a), gpu_attend(c)
    assert not np.isnan(ga).any() and np.array_equal(ga, gc)


def test_full_size_fp8_large_batch(sd):
    """The step bench.py times at this workload: quantising append of one token per sequence, then attention
    in one launch."""
    import torch
    wl = workloads.make_config(4, append=True)
    dw = device_workload(wl, balance_for_batch=True)
    dw.append()
    got = dw.attend()
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    assert not np.isnan(got).any()
    k, v, ks, vs = wl.k_pages, wl.v_pages, wl.k_scales, wl.v_scales
    oracle.kv_append_fp8(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, np.arange(len(wl.seq_ids) + 1, dtype=np.int32),
                         k, v, ks, vs, wl.block_table)
    assert np.array_equal(dw.k_pages.cpu().numpy(), k) and np.array_equal(dw.v_pages.cpu().numpy(), v)
    check_fp8(got, oracle_all_rows(wl, k, v, ks, vs))


# ---------------------------------------------------------------- shared-prefix aware entry point
def gpu_attend_prefix(wl, **kw):
    import torch
    dw = device_workload(wl, **kw)
    out = dw.attend_prefix()
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 2, 128), (28, 4, 128), (8, 1, 64), (16, 1, 128), (3, 1, 128), (40, 2, 128)])
@pytest.mark.parametrize("chunk", [128, 512])
def test_prefix_entry_point_matches_oracle(sd, Hq, Hkv, d, chunk):
    """Groups of 1, 2, 5, 16 and 19 sequences; shared prefixes that are shorter than a chunk, end inside
    a chunk, end on a chunk boundary, and cover a whole sequence."""
    sizes = [1, 2, 5, 16, 19, 3]
    prefix = [300, 3 * chunk, chunk + 77, 2 * chunk + 16, 40, 4 * chunk]
    session_of = np.repeat(np.arange(len(sizes)), sizes)
    prefix_len = np.repeat(prefix, sizes)
    rng = np.random.default_rng(chunk + Hq)
    lens = prefix_len + rng.integers(0, 2 * chunk, size=len(session_of), endpoint=True)
    lens[7] = prefix_len[7]  # one sequence is nothing but its shared prefix
    wl = workloads.make_custom(lens, Hq, Hkv, d, seed=400 + Hq + chunk, session_of=session_of, prefix_len=prefix_len)
    got = gpu_attend_prefix(wl, chunk_tokens=chunk)
    check(got, oracle_full(wl))
    plain = gpu_attend(wl, chunk_tokens=chunk)
    assert np.abs(got - plain).max() <= ALARM_ABS + ALARM_REL * np.abs(plain).max()


@pytest.mark.parametrize("d", [128, 64])
def test_prefix_entry_point_fp8(sd, d):
    sizes = [4, 16, 1]
    session_of = np.repeat(np.arange(3), sizes)
    prefix_len = np.repeat([1024 + 5, 2048 + 512, 512 - 9], sizes)  # two prefixes end inside a page
    lens = prefix_len + np.random.default_rng(5).integers(1, 700, size=len(session_of))
    wl = workloads.make_custom(lens, 16, 2, d, "fp8", seed=410, session_of=session_of, prefix_len=prefix_len)
    check_fp8(gpu_attend_prefix(wl, chunk_tokens=512), oracle_full(wl))


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("scale", [-0.09, 0.0])
def test_prefix_entry_point_with_negative_and_zero_scale(sd, scale, kv_dtype):
    """The shared-prefix items work with |scale| and sign-flipped (or zeroed) queries; the plain items
    with the scale itself.  Both must give the oracle's result for the scale that was passed."""
    sizes = [5, 2]
    session_of = np.repeat(np.arange(2), sizes)
    prefix_len = np.repeat([512, 256], sizes)
    lens = prefix_len + np.random.default_rng(9).integers(1, 300, size=len(session_of))
    wl = workloads.make_custom(lens, 8, 2, 128, kv_dtype, seed=420, session_of=session_of, prefix_len=prefix_len,
                               scale=scale)
    got, want = gpu_attend_prefix(wl, chunk_tokens=256), oracle_full(wl)
    (check_fp8 if kv_dtype == "fp8" else check)(got, want)


def test_prefix_entry_point_without_groups_is_the_plain_call(sd):
    import torch
    wl = workloads.make_custom([700, 1500, 64], 8, 2, 128, seed=420)
    dw = device_workload(wl)
    a = dw.attend().clone()
    b = torch.zeros_like(a)
    sd.paged_decode_attention_prefix(dw.shape, dw.q, dw.k_pages, dw.v_pages, None, None, dw.block_table,
                                     dw.context_lens, None, None, 0, 0, 0, dw.scale, b, dw.workspace, dw.ws_bytes)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ---------------------------------------------------------------- fp8 quantising append
def _fp8_append_case(sd, ranges, Hkv=2, num_pages=12, seed=0, scales=(1.0,), prefill=None, d=128):
    """Run the same range append on the device and in the oracle; both start from the same pool."""
    import torch
    from paper_2508_11553_amd import binding
    from device_workload import _to_dev
    rng = np.random.default_rng(seed)
    nseq = max(r[0] for r in ranges) + 1
    maxnb = 6
    bt = rng.permutation(num_pages)[:nseq * maxnb].reshape(nseq, maxnb).astype(np.int32)
    T = sum(r[2] for r in ranges)
    mag = rng.choice(scales, size=(T, 1, 1))
    kn = workloads.f32_to_bf16_bits((rng.standard_normal((T, Hkv, d)) * mag).astype(np.float32))
    vn = workloads.f32_to_bf16_bits((rng.standard_normal((T, Hkv, d)) * mag[::-1]).astype(np.float32))
    k = np.full((num_pages, Hkv, 16, d), 0x7F, np.uint8); v = k.copy()
    ks = np.full((num_pages, Hkv), np.nan, np.float32); vs = ks.copy()
    if prefill is not None:  # earlier tokens, written by the oracle on both sides
        pk = workloads.f32_to_bf16_bits(rng.standard_normal((sum(p[2] for p in prefill), Hkv, d)).astype(np.float32))
        oracle.kv_append_fp8(pk, pk, np.int32([p[0] for p in prefill]), np.int32([p[1] for p in prefill]),
                             np.int32(np.concatenate([[0], np.cumsum([p[2] for p in prefill])])), k, v, ks, vs, bt)
    rs, st = np.int32([r[0] for r in ranges]), np.int32([r[1] for r in ranges])
    r0 = np.int32(np.concatenate([[0], np.cumsum([r[2] for r in ranges])]))
    shape = sd.Shape(batch=nseq, num_q_heads=Hkv, num_kv_heads=Hkv, head_dim=d, page_size=16, num_pages=num_pages,
                     max_blocks_per_seq=maxnb, kv_dtype=sd.SD_FP8_E4M3, max_context_len=16 * maxnb, chunk_tokens=0)
    dev = "cuda:0"
    dk, dv, dks, dvs = _to_dev(k, dev), _to_dev(v, dev), _to_dev(ks, dev), _to_dev(vs, dev)
    binding.kv_append_fp8(shape, _to_dev(kn, dev), _to_dev(vn, dev), _to_dev(rs, dev), _to_dev(st, dev), _to_dev(r0, dev),
                          len(ranges), max(r[2] for r in ranges), dk, dv, dks, dvs, _to_dev(bt, dev))
    torch.cuda.synchronize()
    oracle.kv_append_fp8(kn, vn, rs, st, r0, k, v, ks, vs, bt)
    assert np.array_equal(dk.cpu().numpy(), k) and np.array_equal(dv.cpu().numpy(), v)
    assert np.array_equal(dks.cpu().numpy().view(np.uint32), ks.view(np.uint32))
    assert np.array_equal(dvs.cpu().numpy().view(np.uint32), vs.view(np.uint32))


@pytest.mark.parametrize("d", [128, 64])
def test_fp8_append_fresh_ranges_bit_exact(sd, d):
    _fp8_append_case(sd, [(0, 0, 96), (1, 0, 1), (2, 0, 17)], num_pages=20, seed=1, scales=(1.0, 0.01, 30.0), d=d)


@pytest.mark.parametrize("d", [128, 64])
def test_fp8_append_into_partly_filled_pages_bit_exact(sd, d):
    # sequence 0 holds 5 tokens, 1 holds 21, 2 holds 16 (next append opens a page)
    pre = [(0, 0, 5), (1, 0, 21), (2, 0, 16)]
    _fp8_append_case(sd, [(0, 5, 3), (1, 21, 40), (2, 16, 1)], num_pages=20, seed=2, scales=(0.05, 1.0, 8.0), prefill=pre, d=d)
    _fp8_append_case(sd, [(0, 5, 1), (1, 21, 1), (2, 16, 1)], num_pages=20, seed=3, scales=(0.05,), prefill=pre, d=d)   # no growth
    _fp8_append_case(sd, [(0, 5, 1), (1, 21, 1), (2, 16, 1)], num_pages=20, seed=4, scales=(40.0,), prefill=pre, d=d)   # growth


@pytest.mark.parametrize("d", [128, 64])
def test_fp8_append_quotients_over_many_scales_bit_exact(sd, d):
    """The kernels divide by a tile's scale through a reciprocal refined once per tile; the codes must be those of
    the plain division the oracle uses.  Magnitudes from 2^-70 to 2^70 (beyond the range in which the kernels use the shortcut), mixed within
    a tile and one per tile, rows of random values."""
    rng = np.random.default_rng(77)
    mags = tuple(float(2.0 ** k * (1 + rng.random())) for k in range(-70, 71, 2))
    _fp8_append_case(sd, [(b, 0, 16) for b in range(40)], num_pages=260, seed=100, scales=mags, d=d)   # mixed within a tile
    for i, m in enumerate(mags[::3]):   # and one magnitude per call: every element of a tile within its range
        _fp8_append_case(sd, [(b, 0, 16) for b in range(8)], num_pages=60, seed=200 + i, scales=(m,), d=d)


@pytest.mark.parametrize("d", [128, 64])
def test_fp8_append_encoder_matches_the_oracle_on_every_bf16_magnitude(sd, d):
    """One page whose first row pins the scale to 1 (a 448 in it); the other rows sweep bf16 values
    across every binade the format covers, including exact ties between neighbouring codes."""
    import torch
    from paper_2508_11553_amd import binding
    from device_workload import _to_dev
    Hkv = 1
    vals = []
    for e in range(-12, 9):
        for m in range(0, 128, 128 // d):   # every bf16 mantissa at d = 128, every other one at d = 64: both hold all ties
            vals.append((1 + m / 128.0) * 2.0 ** e)
    vals = np.float32(vals)[:15 * d]
    x = np.zeros((16, Hkv, d), np.float32)
    x[0, 0, 0] = 448.0
    x[1:, 0, :].flat[:len(vals)] = vals
    x[1::2] *= -1
    kn = workloads.f32_to_bf16_bits(x)
    bt = np.int32([[0]])
    k = np.zeros((1, Hkv, 16, d), np.uint8); v = k.copy(); ks = np.zeros((1, Hkv), np.float32); vs = ks.copy()
    shape = sd.Shape(batch=1, num_q_heads=1, num_kv_heads=1, head_dim=d, page_size=16, num_pages=1,
                     max_blocks_per_seq=1, kv_dtype=sd.SD_FP8_E4M3, max_context_len=16, chunk_tokens=0)
    dev = "cuda:0"
    dk, dv, dks, dvs = _to_dev(k, dev), _to_dev(v, dev), _to_dev(ks, dev), _to_dev(vs, dev)
    binding.kv_append_fp8(shape, _to_dev(kn, dev), _to_dev(kn, dev), _to_dev(np.int32([0]), dev), _to_dev(np.int32([0]), dev),
                          _to_dev(np.int32([0, 16]), dev), 1, 16, dk, dv, dks, dvs, _to_dev(bt, dev))
    torch.cuda.synchronize()
    oracle.kv_append_fp8(kn, kn, np.int32([0]), np.int32([0]), np.int32([0, 16]), k, v, ks, vs, bt)
    assert ks[0, 0] == 1.0
    assert np.array_equal(dk.cpu().numpy(), k) and np.array_equal(dv.cpu().numpy(), v)


@pytest.mark.parametrize("d", [128, 64])
def test_fp8_resume_then_attend(sd, d):
    """Rebuild an fp8 cache from bf16 rows in one bulk call per sequence, then attend: the result must match
    the oracle run over the oracle-built pool."""
    import torch
    from paper_2508_11553_amd import binding
    from device_workload import _to_dev
    src = workloads.make_custom([700, 33, 1500], 16, 2, d, "bf16", seed=30, poison=False)
    rows_k, rows_v = [], []
    for b, L in enumerate(src.context_lens):
        t = np.arange(L)
        rows_k.append(src.k_pages[src.block_table[b, t // 16], :, t % 16]); rows_v.append(src.v_pages[src.block_table[b, t // 16], :, t % 16])
    kn, vn = np.concatenate(rows_k), np.concatenate(rows_v)
    r0 = np.int32(np.concatenate([[0], np.cumsum(src.context_lens)]))
    wl = workloads.make_custom(src.context_lens, 16, 2, d, "fp8", seed=31)  # same table shape; pools get overwritten
    wl.q, wl.block_table = src.q, src.block_table
    wl.k_pages[:] = 0x7F; wl.v_pages[:] = 0x7F; wl.k_scales[:] = np.nan; wl.v_scales[:] = np.nan
    dw = device_workload(wl)
    binding.kv_append_fp8(dw.shape, _to_dev(kn, dw.device), _to_dev(vn, dw.device), _to_dev(np.int32([0, 1, 2]), dw.device),
                          _to_dev(np.int32([0, 0, 0]), dw.device), _to_dev(r0, dw.device), 3, int(src.context_lens.max()),
                          dw.k_pages, dw.v_pages, dw.k_scales, dw.v_scales, dw.block_table)
    out = dw.attend()
    torch.cuda.synchronize()
    oracle.kv_append_fp8(kn, vn, np.int32([0, 1, 2]), np.int32([0, 0, 0]), r0, wl.k_pages, wl.v_pages, wl.k_scales, wl.v_scales, wl.block_table)
    assert np.array_equal(dw.k_pages.cpu().numpy(), wl.k_pages) and np.array_equal(dw.v_pages.cpu().numpy(), wl.v_pages)
    check_fp8(out.cpu().numpy(), oracle_full(wl))


@pytest.mark.parametrize("d", [128, 64])
def test_fp8_decode_step_append_then_attend(sd, d):
    """One decode step on an fp8 cache: quantising append of one token per sequence, then attention."""
    import torch
    wl = workloads.make_custom([17, 33, 5, 16, 700, 1025], 16, 2, d, "fp8", seed=33, append=True)
    dw = device_workload(wl)
    dw.append()
    out = dw.attend()
    torch.cuda.synchronize()
    k, v, ks, vs = wl.k_pages, wl.v_pages, wl.k_scales, wl.v_scales
    oracle.kv_append_fp8(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, np.arange(len(wl.seq_ids) + 1, dtype=np.int32),
                         k, v, ks, vs, wl.block_table)
    assert np.array_equal(dw.k_pages.cpu().numpy(), k) and np.array_equal(dw.v_pages.cpu().numpy(), v)
    assert np.array_equal(dw.k_scales.cpu().numpy().view(np.uint32), ks.view(np.uint32))
    check_fp8(out.cpu().numpy(), oracle_full(wl))


# ---------------------------------------------------------------- table check
def test_validate_tables_counts_what_a_launch_would_dereference(sd):
    import torch
    from device_workload import _to_dev
    wl = workloads.make_custom([40, 0, 513, 16, 700], 8, 2, 64, seed=70)
    dw = device_workload(wl)
    report = torch.full((4,), 77, dtype=torch.int32, device=dw.device)
    sd.validate_tables(dw.shape, dw.block_table, dw.context_lens, report)
    torch.cuda.synchronize()
    assert report.cpu().tolist()[:2] == [0, 0]
    # corrupt entries inside and outside the used part of the rows, and two lengths
    bt, lens = wl.block_table.copy(), wl.context_lens.copy()
    bt[0, 1] = -1                      # used (40 tokens = 3 pages)
    bt[0, 5] = wl.num_pages + 9        # not used
    bt[2, 32] = wl.num_pages           # used (513 tokens = 33 pages)
    bt[4, 0] = 1 << 30                 # used
    bt[1, 0] = -5                      # not used: the sequence is empty
    lens[3] = -2
    lens[4] = wl.max_context_len + 1   # clamped: its first 44 pages count, among them bt[4, 0]
    sd.validate_tables(dw.shape, _to_dev(bt, dw.device), _to_dev(lens, dw.device), report)
    torch.cuda.synchronize()
    used = (np.clip(lens, 0, wl.max_context_len) + 15) // 16
    want_bad = sum(int(((bt[b, :used[b]] < 0) | (bt[b, :used[b]] >= wl.num_pages)).sum()) for b in range(wl.batch))
    assert want_bad == 3
    assert report.cpu().tolist()[:2] == [want_bad, 2]


def test_validate_groups_reports_inconsistent_group_arrays(sd):
    """Deliberately inconsistent group arrays go to the check only, never to the attention kernel."""
    import torch
    from device_workload import _to_dev
    sizes = [3, 5, 2]
    session_of = np.repeat(np.arange(3), sizes)
    prefix_len = np.repeat([64, 160, 32], sizes)
    lens = prefix_len + np.arange(1, 11) * 7
    wl = workloads.make_custom(np.concatenate([lens, [50]]), 8, 2, 64, seed=71,
                               session_of=np.concatenate([session_of, [3]]), prefix_len=np.concatenate([prefix_len, [0]]))
    dw = device_workload(wl)
    report = torch.full((4,), 77, dtype=torch.int32, device=dw.device)

    def run(gs, sh, table=None, max_group=5, max_shared=160, ngroups=None):
        gs = np.int32(gs)
        sd.validate_groups(dw.shape, dw.block_table if table is None else _to_dev(table, dw.device), dw.context_lens,
                           _to_dev(gs, dw.device), _to_dev(np.int32(sh), dw.device), len(gs) - 1 if ngroups is None else ngroups,
                           max_group, max_shared, report)
        torch.cuda.synchronize()
        return report.cpu().tolist()

    gs, sh = wl.group_start[:4], wl.shared_len           # the last sequence is in no group
    assert run(gs, sh) == [0, 0, 0, 0]
    assert run(gs, sh, max_group=4) == [1, 0, 0, 0]      # the group of five is too large
    bad = sh.copy(); bad[4] = 144; bad[10] = 16          # a member disagrees; the ungrouped sequence claims a prefix
    assert run(gs, bad) == [0, 2, 0, 0]
    bad = sh.copy(); bad[8:10] = 112                     # a whole group claims more than its members hold (95, 102)
    assert run(gs, bad)[1] == 2
    tbl = wl.block_table.copy(); tbl[6, 3] = tbl[6, 4]   # a member's shared page is not the first member's
    tbl[1, 7] = 0                                         # beyond the shared pages: not looked at
    assert run(gs, sh, table=tbl) == [0, 0, 1, 0]
    assert run([0, 3, 3, 20], sh)[0] == 2                # an empty group and one that leaves the batch


# ---------------------------------------------------------------- HIP graph capture
def test_decode_step_replays_from_a_hip_graph(sd):
    """The library neither allocates nor synchronises, so a whole decode step (append + attention) can be
    captured once and replayed.  Every replay, with new queries and new appended rows written into the same
    buffers and with eager work in between, must equal the eager result bit for bit."""
    import torch
    wl = workloads.make_custom([700, 33, 1500, 64], 8, 2, 128, seed=40, append=True)
    dw = device_workload(wl)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        dw.append(stream); dw.attend(stream)  # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            dw.append(); dw.attend()
    rng = np.random.default_rng(0)
    from device_workload import _to_dev
    for it in range(4):
        q = workloads.f32_to_bf16_bits(rng.standard_normal(wl.q.shape).astype(np.float32))
        kn = workloads.f32_to_bf16_bits(rng.standard_normal(wl.k_new.shape).astype(np.float32))
        dw.q.copy_(_to_dev(q, dw.device)); dw.k_new.copy_(_to_dev(kn, dw.device))
        graph.replay()
        torch.cuda.synchronize()
        got = dw.out.clone()
        dw.out.zero_()                      # eager work between replays
        dw.append(); eager = dw.attend().clone()
        torch.cuda.synchronize()
        assert torch.equal(got, eager), f"replay {it} differs from the eager step"
    k, v = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_append(kn, wl.v_new, wl.seq_ids, wl.positions, k, v, wl.block_table)
    wl.q = q
    check(got.cpu().numpy(), oracle_full(wl, k, v))


def test_one_call_decode_step_replays_from_a_hip_graph(sd):
    """The same for the decode step as ONE call (range pass that appends, then the merge pass): captured once,
    replayed with new queries and new rows, compared with the eager call bit for bit and with the oracle."""
    import torch
    from device_workload import _to_dev
    lens = [700, 33, 1500, 64, 1, 257]
    wl = workloads.make_custom(lens, 8, 2, 128, seed=41, append=True)
    dw = device_workload(wl, chunk_tokens=128)
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        dw.append_and_attend(stream)  # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            dw.append_and_attend()
    rng = np.random.default_rng(1)
    for it in range(3):
        q = workloads.f32_to_bf16_bits(rng.standard_normal(wl.q.shape).astype(np.float32))
        kn = workloads.f32_to_bf16_bits(rng.standard_normal(wl.k_new.shape).astype(np.float32))
        rows = np.zeros((wl.batch,) + kn.shape[1:], np.uint16)
        rows[wl.seq_ids] = kn
        dw.q.copy_(_to_dev(q, dw.device)); dw.k_new_rows.copy_(_to_dev(rows, dw.device))
        graph.replay()
        torch.cuda.synchronize()
        got = dw.out.clone()
        dw.out.zero_()                      # eager work between replays
        eager = dw.append_and_attend().clone()
        torch.cuda.synchronize()
        assert torch.equal(got, eager), f"replay {it} differs from the eager step"
    k, v = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_append(kn, wl.v_new, wl.seq_ids, wl.positions, k, v, wl.block_table)
    wl.q = q
    check(got.cpu().numpy(), oracle_full(wl, k, v))

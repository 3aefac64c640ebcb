"""Parity of the causal multi-query kernel against the CPU oracle, through the C ABI (GPU only).

Same arithmetic as the decode step (bf16 operands, fp32 accumulation, bf16 weights), so the same
tolerances and the same alarm level apply; see test_gpu_parity.py."""
import numpy as np
import pytest

import oracle
import workloads
from workloads import bf16_bits_to_f32, f32_to_bf16_bits
from tests.test_gpu_parity import check as check_decode, check_fp8, device_workload, sd  # noqa: F401  (sd is a fixture)

pytestmark = pytest.mark.gpu


def check(got, ref, kv_dtype="bf16"):
    # The alarm level is set relative to a row's largest output.  With a handful of tokens the bf16
    # rounding of the weights is bounded by 2^-8 * sum_t p_t |V_t| instead, which exceeds that when the
    # terms cancel; a causal batch holds hundreds of such rows (every sequence's first positions) where a
    # decode batch holds a few, so the tail is seen.  The stated tolerance itself is unchanged.
    if kv_dtype == "fp8":
        check_fp8(got, ref, alarm_scale=2.0)
    else:
        check_decode(got, ref, alarm_scale=2.0)


def make(lens, nq, Hq, Hkv, d, kv_dtype="bf16", seed=0):
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=seed)
    rng = np.random.default_rng(seed + 1)
    q_start = np.concatenate([[0], np.cumsum(nq)]).astype(np.int32)
    q = f32_to_bf16_bits(rng.standard_normal((int(q_start[-1]), Hq, d)).astype(np.float32))
    return wl, q, q_start


def ref(wl, q, q_start):
    return oracle.paged_prefill_attention(q, q_start, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens,
                                          wl.scale, wl.k_scales, wl.v_scales, wl.kv_dtype)


def gpu(wl, q, q_start):
    import torch
    out = device_workload(wl).attend_prefill(q, q_start)
    torch.cuda.synchronize()
    return out.cpu().numpy()


@pytest.mark.parametrize("kv_dtype,d", [("bf16", 64), ("bf16", 128), ("fp8", 128), ("fp8", 64)])
@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 2), (8, 1), (28, 4), (6, 2), (16, 1), (32, 4), (17, 1), (40, 2), (64, 1)])
def test_ragged_query_counts_over_several_tiles(sd, Hq, Hkv, d, kv_dtype):
    # query counts below, at and above a workgroup's block, context lengths across page, tile and round edges
    lens = [1, 7, 16, 33, 64, 129, 130, 257, 300, 511, 640, 1000]
    nq = [1, 7, 3, 33, 17, 128, 1, 65, 300, 100, 129, 77]
    wl, q, q_start = make(lens, nq, Hq, Hkv, d, kv_dtype, seed=700 + Hq + d)
    check(gpu(wl, q, q_start), ref(wl, q, q_start), kv_dtype)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("scale", [-0.11, 0.0])
def test_negative_and_zero_scale(sd, scale, kv_dtype):
    # the kernel works with |scale| and sign-flipped (or zeroed) queries; the result must be the oracle's for the scale given
    lens, nq = [100, 33, 257], [40, 33, 9]
    wl = workloads.make_custom(lens, 8, 2, 128, kv_dtype, seed=61, scale=scale)
    rng = np.random.default_rng(62)
    q_start = np.concatenate([[0], np.cumsum(nq)]).astype(np.int32)
    q = f32_to_bf16_bits(rng.standard_normal((int(q_start[-1]), 8, 128)).astype(np.float32))
    check(gpu(wl, q, q_start), ref(wl, q, q_start), kv_dtype)


def test_one_query_per_sequence_equals_the_decode_step(sd):
    import torch
    lens = [1, 15, 16, 17, 200, 513, 1500]
    wl = workloads.make_custom(lens, 8, 2, 128, seed=31)
    dw = device_workload(wl)
    dec = dw.attend().clone()
    pre = dw.attend_prefill(wl.q, np.arange(len(lens) + 1, dtype=np.int32))
    torch.cuda.synchronize()
    # different split of the token range, same arithmetic: equal up to the rounding of the partial sums
    ref_ = oracle.paged_decode_attention(wl.q, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale)
    check(pre.cpu().numpy(), ref_)
    # the two kernels round their weights at slightly different points (one fuses the scale into the exponent):
    # a weight that lands on the other side of a bf16 rounding boundary moves a short row by up to 2^-8 of its V
    diff = np.abs(pre.cpu().numpy() - dec.cpu().numpy())
    assert (diff <= 2 * (3e-4 + 2.0 ** -8 * np.abs(ref_).max(axis=-1, keepdims=True))).all()


@pytest.mark.parametrize("kv_dtype,d", [("bf16", 64), ("bf16", 128), ("fp8", 128), ("fp8", 64)])
def test_constant_v_returns_the_constant(sd, kv_dtype, d):
    """Every row is a convex combination of V rows, normalised by the sum of the very weights the product uses,
    so with all V rows equal the result is that row up to fp32 rounding, however the weights round."""
    lens, nq = [70, 300, 33], [70, 40, 33]
    wl, q, q_start = make(lens, nq, 8, 2, d, kv_dtype, seed=51)
    if kv_dtype == "bf16":
        cst = f32_to_bf16_bits(np.float32([0.37]))[0]
        wl.v_pages[...] = cst
        want = float(workloads.bf16_bits_to_f32(np.uint16([cst]))[0])
    else:
        wl.v_pages[...] = 0x38            # e4m3fn 1.0
        wl.v_scales[...] = np.float32(0.25)
        want = 0.25
    got = gpu(wl, q, q_start)
    assert np.abs(got - want).max() <= 2e-6 * abs(want) + 1e-7


def test_sequences_without_queries_with_too_many_and_empty(sd):
    lens = [40, 0, 5, 100, 16]
    nq = [0, 3, 9, 100, 16]          # none; queries but no tokens; more queries than tokens; full; full
    wl, q, q_start = make(lens, nq, 4, 2, 64, seed=41)
    got, want = gpu(wl, q, q_start), ref(wl, q, q_start)
    check(got, want)
    assert not got[q_start[1]:q_start[2]].any()                      # no tokens: zero rows
    assert not got[q_start[2]:q_start[2] + 4].any()                  # positions before the first token: zero rows
    assert got[q_start[2] + 4].any()


def test_rows_nobody_owns_are_left_untouched_and_bad_ranges_are_skipped(sd):
    import torch
    import paper_2508_11553_amd as m
    wl, q, _ = make([50, 60], [8, 8], 4, 2, 64, seed=43)
    dw = device_workload(wl)
    q_dev = torch.from_numpy(q.view(np.int16)).to("cuda:0")
    out = torch.full((16, 4, 64), 7.0, dtype=torch.float32, device="cuda:0")
    # sequence 0 owns rows 0..7; sequence 1 claims rows 8..23 of a 16-row q: skipped
    qs = torch.tensor([0, 8, 24], dtype=torch.int32, device="cuda:0")
    m.paged_prefill_attention(dw.shape, q_dev, qs, 16, 16, dw.k_pages, dw.v_pages, None, None, dw.block_table,
                              dw.context_lens, dw.scale, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert (got[8:] == 7.0).all()
    want = ref(wl, q[:8], np.array([0, 8, 8], dtype=np.int32))
    check(got[:8], want[:8])


def test_long_stretch_at_a_rollout_shape(sd):
    # a resumed 8k trajectory re-computing its last 1024 tokens, Qwen3-8B-like heads, next to short ones
    lens = [8192, 700, 2049]
    nq = [1024, 700, 512]
    wl, q, q_start = make(lens, nq, 32, 8, 128, seed=47)
    got = gpu(wl, q, q_start)
    rows = np.concatenate([np.arange(0, 1024, 97), [1023], q_start[1] + np.arange(0, 700, 61), q_start[2] + np.arange(0, 512, 53)])
    # the oracle one row at a time: a row is the decode problem with context pos + 1
    for r in rows:
        b = int(np.searchsorted(q_start, r, side="right") - 1)
        pos = lens[b] - nq[b] + (r - q_start[b])
        one = oracle.paged_decode_attention(q[r:r + 1], wl.k_pages, wl.v_pages, wl.block_table[b:b + 1],
                                            np.array([pos + 1], dtype=np.int32), wl.scale)
        check(got[r:r + 1], one)


@pytest.mark.parametrize("kv_dtype,d", [("bf16", 128), ("bf16", 64), ("fp8", 128), ("fp8", 64)])
@pytest.mark.parametrize("shape", ["ramp", "jumps", "decay"])
def test_scores_that_outgrow_the_running_reference(sd, shape, d, kv_dtype):
    """Keys whose size depends on the position, so that a row's largest score moves all along the
    range: steadily (ramp: the exponent's reference has to follow many times), in rare leaps far
    beyond anything seen before (jumps: weights of earlier tokens underflow at once), or not at
    all after the first tiles (decay: the reference stays where the first tile put it).  bf16 pools:
    every K row is scaled; fp8 pools: every page's K scale (a page's tokens grow together)."""
    lens, nq = [1500, 777, 96], [400, 777, 96]
    wl, q, q_start = make(lens, nq, 8, 2, d, kv_dtype, seed=900 + d)

    def factor(t):
        if shape == "ramp":
            return 1.0 + 0.03 * t
        if shape == "jumps":
            return np.where(t % 211 >= 208, 40.0 * (1 + t // 211), 1.0)
        return 30.0 / (1.0 + 0.05 * t)

    if kv_dtype == "bf16":
        k = bf16_bits_to_f32(wl.k_pages)                       # [pages][Hkv][16][d]
        for b, L in enumerate(lens):
            t = np.arange(L)
            k[wl.block_table[b, t // 16], :, t % 16, :] *= factor(t)[:, None, None].astype(np.float32)
        wl.k_pages = f32_to_bf16_bits(k)
    else:
        for b, L in enumerate(lens):
            first = np.arange(0, L, 16)
            wl.k_scales[wl.block_table[b, first // 16], :] *= factor(first + 15)[:, None].astype(np.float32)
    check(gpu(wl, q, q_start), ref(wl, q, q_start), kv_dtype)

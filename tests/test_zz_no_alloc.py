"""paged_decode_attention_static: the entry point for callers that cannot allocate.

It keeps the partial results and arrival counters in an array that is part of the library instead of
a caller's workspace.  Checked through the C ABI against paged_decode_attention (same kernels, so the
outputs must agree bit for bit) and against the CPU oracle, on two calls in a row of which the
second is smaller, so that whatever the first call left in the shared array is in the way.
Collected last on purpose: a failure here must not hide the other GPU tests.
"""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS, FP8_MAX_ABS = 1e-2, 1e-3, 5e-2


@pytest.fixture(scope="module")
def sd():
    import torch
    assert torch.cuda.is_available()
    import paper_2508_11553_amd as m
    m.load()
    return m


def both_entry_points(sd, wl, chunk):
    """-> (out of paged_decode_attention, out of paged_decode_attention_static), numpy."""
    import torch
    from device_workload import DeviceWorkload
    dw = DeviceWorkload(wl, chunk_tokens=chunk)
    assert sd.workspace_bytes(dw.shape) <= 48 << 20
    want = dw.attend().clone()
    got = torch.full_like(want, float("nan"))
    sd.paged_decode_attention_static(dw.shape, dw.q, dw.k_pages, dw.v_pages, dw.k_scales, dw.v_scales,
                                     dw.block_table, dw.context_lens, dw.scale, got)
    torch.cuda.synchronize()
    return want.cpu().numpy(), got.cpu().numpy()


def oracle_out(wl):
    return oracle.paged_decode_attention(wl.q, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale,
                                         wl.k_scales, wl.v_scales, wl.kv_dtype)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_static_scratch_entry_point_twice_in_a_row(sd, kv_dtype):
    big = workloads.make_custom([1500, 700, 0, 2049, 64, 3000, 1], 16, 2, 128, kv_dtype, seed=900)
    small = workloads.make_custom([300, 129, 5], 8, 2, 128, kv_dtype, seed=901)
    for wl, chunk in ((big, 256), (small, 128)):   # sequences are cut across waves: the scratch array is in use
        want, got = both_entry_points(sd, wl, chunk)
        assert not np.isnan(got).any()
        assert np.array_equal(got, want)
        err = np.abs(got.astype(np.float64) - oracle_out(wl))
        if kv_dtype == "fp8":
            assert err.max() <= FP8_MAX_ABS
        else:
            assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS


def test_static_scratch_entry_point_single_chunk_and_head_dim_64(sd):
    wl = workloads.make_custom([40, 0, 513, 16], 8, 2, 64, seed=902)
    for chunk in (128, 640):   # ranges of 640 tokens hold whole sequences: their waves write `out` themselves
        want, got = both_entry_points(sd, wl, chunk)
        assert np.array_equal(got, want)
        err = np.abs(got.astype(np.float64) - oracle_out(wl))
        assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS

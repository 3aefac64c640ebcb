"""Pins for the oracle's whole-page copy (CPU only): what a private copy of a page must mean for attention."""
import numpy as np
import pytest

import oracle
import workloads


@pytest.mark.parametrize("kv_dtype,d", [("bf16", 64), ("fp8", 128)])
def test_a_sequence_that_reads_the_copy_attends_exactly_as_before(kv_dtype, d):
    wl = workloads.make_custom([40, 70, 5], 4, 2, d, kv_dtype, seed=11, spare_pages=8)
    ref = oracle.paged_decode_attention(wl.q, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale,
                                        wl.k_scales, wl.v_scales, wl.kv_dtype)
    free = [p for p in range(wl.num_pages) if p not in set(wl.block_table.ravel().tolist())][:3]
    assert len(free) == 3
    # re-point the last page of every sequence at a copy
    src = np.int32([wl.block_table[b, (L - 1) // 16] for b, L in enumerate(wl.context_lens)])
    dst = np.int32(free)
    k0, v0 = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_copy_pages(src, dst, wl.k_pages, wl.v_pages, wl.k_scales, wl.v_scales)
    bt = wl.block_table.copy()
    for b, L in enumerate(wl.context_lens):
        bt[b, (L - 1) // 16] = dst[b]
    got = oracle.paged_decode_attention(wl.q, wl.k_pages, wl.v_pages, bt, wl.context_lens, wl.scale, wl.k_scales,
                                        wl.v_scales, wl.kv_dtype)
    assert np.array_equal(got, ref)
    # nothing but the destination pages changed
    keep = np.ones(wl.num_pages, bool); keep[dst] = False
    assert np.array_equal(wl.k_pages[keep], k0[keep]) and np.array_equal(wl.v_pages[keep], v0[keep])
    assert np.array_equal(wl.k_pages[dst], k0[src]) and np.array_equal(wl.v_pages[dst], v0[src])


def test_invalid_and_identity_pairs_do_nothing():
    wl = workloads.make_custom([20], 2, 2, 64, seed=3, spare_pages=2)
    k0, v0 = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_copy_pages(np.int32([0, -1, 1, wl.num_pages]), np.int32([0, 1, wl.num_pages, 0]), wl.k_pages, wl.v_pages)
    assert np.array_equal(wl.k_pages, k0) and np.array_equal(wl.v_pages, v0)

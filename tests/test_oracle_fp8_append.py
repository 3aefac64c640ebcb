"""Pins for the oracle's fp8 quantising append (CPU only).

The encoder is pinned to torch's float8_e4m3fn conversion and to the input
generator's own numpy encoder (three independent implementations); the append
is pinned to a numpy transcription of its definition on whole-tile cases, and
to properties that must hold whatever the arithmetic: scales never shrink,
untouched slots keep their bits, values survive a scale change within the
new quantisation step.
"""
import numpy as np
import pytest

import oracle
import workloads
from workloads import bf16_bits_to_f32, f32_to_bf16_bits, f32_to_e4m3fn_bits

TABLE = None


def table():
    global TABLE
    if TABLE is None:
        TABLE = np.array([oracle.e4m3fn_to_float(c) for c in range(256)], dtype=np.float32)
    return TABLE


def test_encoder_matches_torch_and_the_generator():
    import torch

    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(5000).astype(np.float32) * s for s in (0.01, 1.0, 50.0, 200.0)])
    x = np.concatenate([x, table()[~np.isnan(table())], np.float32([447.9, 448.0, -448.0, 2.0 ** -10, 3 * 2.0 ** -10,
                                                                     2.0 ** -9, 0.0, -0.0, 464.0, 1e6, -1e6])])
    mine = np.array([oracle.float_to_e4m3fn(v) for v in x], dtype=np.uint8)
    gen = f32_to_e4m3fn_bits(x)
    assert np.array_equal(mine, gen)
    inside = np.abs(x) <= 448
    t = torch.from_numpy(x[inside]).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(mine[inside], t)


def empty_pool(num_pages, Hkv, d):
    k = np.full((num_pages, Hkv, 16, d), 0x7F, np.uint8)
    return k, k.copy(), np.full((num_pages, Hkv), np.nan, np.float32), np.full((num_pages, Hkv), np.nan, np.float32)


def rows(rng, T, Hkv, d, scale=1.0):
    return f32_to_bf16_bits((rng.standard_normal((T, Hkv, d)) * scale).astype(np.float32))


def test_fresh_whole_pages_follow_the_recipe():
    """A range that fills whole fresh pages: scale = absmax/448, codes = nearest(x/scale)."""
    rng = np.random.default_rng(1)
    Hkv, d, T = 2, 64, 48
    kn, vn = rows(rng, T, Hkv, d), rows(rng, T, Hkv, d, 3.0)
    table_ = np.int32([[4, 1, 3, 0]])
    k, v, ks, vs = empty_pool(6, Hkv, d)
    oracle.kv_append_fp8(kn, vn, np.int32([0]), np.int32([0]), np.int32([0, T]), k, v, ks, vs, table_)
    for src, pool, sc in ((kn, k, ks), (vn, v, vs)):
        x = bf16_bits_to_f32(src)
        for pg in range(3):
            for g in range(Hkv):
                tile = x[16 * pg:16 * pg + 16, g]
                s = np.float32(np.abs(tile).max()) / np.float32(448.0)
                assert sc[table_[0, pg], g] == s
                assert np.array_equal(pool[table_[0, pg], g], f32_to_e4m3fn_bits(tile / s))
    # pages 5, 2 and the table's unused entry stay untouched
    assert (k[[5, 2, 0]] == 0x7F).all() and np.isnan(ks[[5, 2, 0]]).all()


def numpy_append(k_new, start, tile, scale):
    """Transcription of the definition for one (page, head) tile; rows land at slots start.."""
    x = bf16_bits_to_f32(k_new)
    tile = tile.copy()
    s0, s1 = start, start + x.shape[0]
    amax_new = np.float32(np.abs(x).max()) if x.size else np.float32(0)
    old_amax = np.float32(scale) * np.float32(448.0) if s0 > 0 else np.float32(0)
    if s0 > 0 and amax_new <= old_amax:
        new_scale = np.float32(scale)
    else:
        new_scale = amax_new / np.float32(448.0) if amax_new > 0 else np.float32(1.0)
        ratio = np.float32(scale) / new_scale
        tile[:s0] = f32_to_e4m3fn_bits((table()[tile[:s0]] * ratio).astype(np.float32))
    tile[s0:s1] = f32_to_e4m3fn_bits((x / new_scale).astype(np.float32))
    return tile, new_scale


@pytest.mark.parametrize("grow", [False, True])
def test_append_into_a_partly_filled_page(grow):
    rng = np.random.default_rng(2 + grow)
    Hkv, d = 2, 64
    first = rows(rng, 5, Hkv, d), rows(rng, 5, Hkv, d)
    second = rows(rng, 3, Hkv, d, 4.0 if grow else 0.1), rows(rng, 3, Hkv, d, 4.0 if grow else 0.1)
    bt = np.int32([[1, 0]])
    k, v, ks, vs = empty_pool(2, Hkv, d)
    oracle.kv_append_fp8(first[0], first[1], np.int32([0]), np.int32([0]), np.int32([0, 5]), k, v, ks, vs, bt)
    k1, v1, ks1, vs1 = k.copy(), v.copy(), ks.copy(), vs.copy()
    oracle.kv_append_fp8(second[0], second[1], np.int32([0]), np.int32([5]), np.int32([0, 3]), k, v, ks, vs, bt)
    for new, before, after, sb, sa in ((second[0], k1, k, ks1, ks), (second[1], v1, v, vs1, vs)):
        for g in range(Hkv):
            want, want_scale = numpy_append(new[:, g], 5, before[1, g], sb[1, g])
            assert sa[1, g] == want_scale
            assert np.array_equal(after[1, g, :8], want[:8])
            assert (after[1, g, 8:] == 0x7F).all()  # slots past the range keep their bits
            if grow:
                assert sa[1, g] > sb[1, g]
                # old tokens survive the re-quantisation within half a step of the new grid
                old_vals = table()[before[1, g, :5]] * sb[1, g]
                new_vals = table()[after[1, g, :5]] * sa[1, g]
                assert np.abs(new_vals - old_vals).max() <= sa[1, g] * 16.0 + 1e-12  # half of the top binade's step (32)
            else:
                assert sa[1, g] == sb[1, g] and np.array_equal(after[1, g, :5], before[1, g, :5])
    assert np.array_equal(k[0], k1[0]) and np.array_equal(v[0], v1[0])  # the other page


def test_ranges_token_by_token_equal_one_range_when_scales_do_not_grow():
    """Decode advance (one row per call) after a resume gives the same pool as one bulk
    range, provided no later row raises a tile's scale (first row of every tile is the largest)."""
    rng = np.random.default_rng(5)
    Hkv, d, T = 2, 64, 40
    x = rng.standard_normal((T, Hkv, d)).astype(np.float32)
    x[::16] *= 50.0  # the row that opens each page dominates it
    kn = vn = f32_to_bf16_bits(x)
    bt = np.int32([[2, 0, 1]])
    a = empty_pool(3, Hkv, d)
    oracle.kv_append_fp8(kn, vn, np.int32([0]), np.int32([0]), np.int32([0, T]), *a, bt)
    b = empty_pool(3, Hkv, d)
    for t in range(T):
        oracle.kv_append_fp8(kn[t:t + 1], vn[t:t + 1], np.int32([0]), np.int32([t]), np.int32([0, 1]), *b, bt)
    valid = np.zeros((3, 16), bool)
    for t in range(T):
        valid[bt[0, t // 16], t % 16] = True
    for pa, pb in zip(a[:2], b[:2]):
        assert np.array_equal(pa.transpose(0, 2, 1, 3)[valid], pb.transpose(0, 2, 1, 3)[valid])
    assert np.array_equal(a[2], b[2]) and np.array_equal(a[3], b[3])


def test_attention_over_an_appended_fp8_pool_tracks_the_bf16_values():
    wl = workloads.make_custom([70, 33], 4, 2, 64, "bf16", seed=6, poison=False)
    ref = oracle.paged_decode_attention(wl.q, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale)
    k, v, ks, vs = empty_pool(wl.num_pages, 2, 64)
    kn = np.concatenate([wl.k_pages[wl.block_table[b, np.arange(L) // 16], :, np.arange(L) % 16] for b, L in enumerate(wl.context_lens)])
    vn = np.concatenate([wl.v_pages[wl.block_table[b, np.arange(L) // 16], :, np.arange(L) % 16] for b, L in enumerate(wl.context_lens)])
    oracle.kv_append_fp8(kn, vn, np.int32([0, 1]), np.int32([0, 0]), np.int32([0, 70, 103]), k, v, ks, vs, wl.block_table)
    got = oracle.paged_decode_attention(wl.q, k, v, wl.block_table, wl.context_lens, wl.scale, ks, vs, "fp8")
    assert np.abs(got - ref).max() <= 5e-2

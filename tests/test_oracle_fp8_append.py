"""Pins for the oracle's fp8 quantising append (CPU only).

The encoder is pinned to torch's float8_e4m3fn conversion and to the input
generator's own numpy encoder (three independent implementations).  The append
is pinned to what does not come from its own formula: fresh tiles to the recipe
(absmax/448, nearest code); the re-encode branch (a tile whose scale must grow)
to a table derived by hand from the format definition for power-of-two growth
(tests/golden/e4m3fn_rescale.txt) and, for arbitrary growth, to the property
that every old value lands on a nearest code of the new grid; plus scales never
shrink and untouched slots keep their bits.  numpy_append below re-types the
definition and only guards the tile bookkeeping (which slots change).
"""
import os

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


def assert_reencoded_to_a_nearest_code(old_codes, old_scale, new_codes, new_scale):
    """The value an old code stood for, dec(c) * old_scale, expressed in units of the new scale, must
    have gone to a code whose value is as near to it as any code's (computed in fp64 from the code
    table: this is half a step of the format AT THAT MAGNITUDE, not of the top binade).  The fp32
    ratio may move an exact tie by one part in 2^23, hence the slack."""
    finite = np.array([c for c in range(256) if (c & 0x7F) != 0x7F])
    vals = table()[finite].astype(np.float64)
    y = table()[old_codes.ravel()].astype(np.float64) * np.float64(old_scale) / np.float64(new_scale)
    got = table()[new_codes.ravel()].astype(np.float64)
    best = np.abs(vals[None, :] - y[:, None]).min(axis=1)
    assert (np.abs(got - y) <= best + 2.0 ** -20 * np.abs(y)).all()
    assert (np.signbit(got) == np.signbit(y)).all()  # the sign survives, also when the value rounds to zero


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "e4m3fn_rescale.txt")


@pytest.mark.parametrize("ratio,new_amax", [(0.5, 3.5), (0.25, 7.0)])
def test_growth_by_a_power_of_two_shifts_exponents_as_derived_by_hand(ratio, new_amax):
    """Pins the re-encode branch to values that do not come from its own formula: every finite code
    (both signs) under a scale that doubles or quadruples, against the table derived by hand from the
    format definition in tests/golden/e4m3fn_rescale.txt."""
    want = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            r, c, n = line.split()
            want[(float(r), int(c))] = int(n)
    d = 128
    pos = table()[:127].astype(np.float32) * np.float32(2.0 ** -8)   # dec(c) / 256 for c = 0 .. 126; 448 / 256 = 1.75
    first = np.zeros((2, 1, d), np.float32)
    first[0, 0, :127], first[1, 0, :127] = pos, -pos
    bt = np.int32([[0]])
    k, v, ks, vs = empty_pool(1, 1, d)
    kn = f32_to_bf16_bits(first)
    assert np.array_equal(bf16_bits_to_f32(kn), first)                # every value is a bf16 number
    oracle.kv_append_fp8(kn, kn, np.int32([0]), np.int32([0]), np.int32([0, 2]), k, v, ks, vs, bt)
    assert ks[0, 0] == np.float32(2.0 ** -8)                          # 1.75 / 448
    assert np.array_equal(k[0, 0, 0, :127], np.arange(127, dtype=np.uint8))          # codes are stored as themselves
    assert np.array_equal(k[0, 0, 1, :127], np.arange(127, dtype=np.uint8) | 0x80)
    grow = np.zeros((1, 1, d), np.float32)
    grow[0, 0, 5] = -new_amax
    gn = f32_to_bf16_bits(grow)
    oracle.kv_append_fp8(gn, gn, np.int32([0]), np.int32([2]), np.int32([0, 1]), k, v, ks, vs, bt)
    assert ks[0, 0] == np.float32(2.0 ** -8 / ratio) and vs[0, 0] == ks[0, 0]
    expect = np.array([want[(ratio, c)] for c in range(127)], dtype=np.uint8)
    for pool in (k, v):
        assert np.array_equal(pool[0, 0, 0, :127], expect)
        assert np.array_equal(pool[0, 0, 1, :127], expect | 0x80)
        assert pool[0, 0, 2, 5] == 0xFE and pool[0, 0, 2, 6] == 0     # the new row: -448 in units of the new scale


def test_growth_by_arbitrary_ratios_lands_on_a_nearest_code():
    """Random tiles, scales growing by 1.01x .. 300x: every old value goes to a nearest code of the new grid."""
    rng = np.random.default_rng(11)
    Hkv, d = 2, 128
    bt = np.int32([[0]])
    for factor in (1.01, 1.3, 2.0, 3.7, 17.0, 300.0):
        k, v, ks, vs = empty_pool(1, Hkv, d)
        first = rows(rng, 9, Hkv, d, 0.7)
        oracle.kv_append_fp8(first, first, np.int32([0]), np.int32([0]), np.int32([0, 9]), k, v, ks, vs, bt)
        k1, ks1 = k.copy(), ks.copy()
        second = np.zeros((1, Hkv, d), np.float32)
        second[0, :, 3] = ks1[0] * 448.0 * factor
        sn = f32_to_bf16_bits(second)
        oracle.kv_append_fp8(sn, sn, np.int32([0]), np.int32([9]), np.int32([0, 1]), k, v, ks, vs, bt)
        for g in range(Hkv):
            assert ks[0, g] > ks1[0, g]
            assert_reencoded_to_a_nearest_code(k1[0, g, :9], ks1[0, g], k[0, g, :9], ks[0, g])


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
                assert_reencoded_to_a_nearest_code(before[1, g, :5], sb[1, g], after[1, g, :5], sa[1, g])
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

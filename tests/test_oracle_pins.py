"""Pins for the CPU oracle: everything here runs without a GPU.

The paper prints no worked numbers for the decode step (it names the
inference engine in its System Overview and never opens it), so the oracle is
pinned to what the mathematics fixes: dense fp64 brute force, a library
routine on the gathered dense problem, closed forms, layout invariances that
the paper's token-exact pause/resume/branch semantics (Data Plane, Trajectory
Manager paragraph) require, and the split/merge identity.
"""
import math
import os

import numpy as np
import pytest

import oracle
import workloads
from workloads import bf16_bits_to_f32, f32_to_bf16_bits, f32_to_e4m3fn_bits
from tests.brute import brute_attention, decode_pool, gather_dense

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(wl, precision="f64", **over):
    a = dict(q=wl.q, k_pages=wl.k_pages, v_pages=wl.v_pages, block_table=wl.block_table,
             context_lens=wl.context_lens, scale=wl.scale, k_scales=wl.k_scales, v_scales=wl.v_scales,
             kv_dtype=wl.kv_dtype, precision=precision)
    a.update(over)
    return oracle.paged_decode_attention(**a)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("precision,tol", [("f64", 1e-12), ("f32", 1e-5)])
def test_config0_matches_dense_bruteforce(precision, tol):
    wl = workloads.make_config(0)
    assert np.abs(run_oracle(wl, precision) - brute_attention(wl)).max() <= tol


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (4, 4), (8, 2), (7, 1), (28, 4), (16, 1)])
@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_random_small_shapes_match_bruteforce(Hq, Hkv, d, kv_dtype):
    rng = np.random.default_rng(Hq * 131 + d + (kv_dtype == "fp8"))
    lens = rng.integers(1, 64, size=5, endpoint=True)
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=int(rng.integers(1 << 30)))
    br = brute_attention(wl)
    assert np.abs(run_oracle(wl, "f64") - br).max() <= 1e-12
    assert np.abs(run_oracle(wl, "f32") - br).max() <= 1e-5


def test_library_sdpa_on_gathered_dense():
    """Third witness: torch's scaled_dot_product_attention (CPU fp32) on the
    dense gathered K/V with the KV heads repeated for GQA."""
    import torch
    import torch.nn.functional as F

    wl = workloads.make_custom([37, 64, 1, 16, 17], 8, 2, 64, seed=11)
    ref = run_oracle(wl, "f64")
    Kp, Vp = decode_pool(wl.k_pages, None, "bf16"), decode_pool(wl.v_pages, None, "bf16")
    qf = bf16_bits_to_f32(wl.q)
    G = wl.num_q_heads // wl.num_kv_heads
    for b, L in enumerate(wl.context_lens):
        K = np.stack([gather_dense(Kp, wl.block_table, b, h // G, L) for h in range(wl.num_q_heads)])
        V = np.stack([gather_dense(Vp, wl.block_table, b, h // G, L) for h in range(wl.num_q_heads)])
        o = F.scaled_dot_product_attention(torch.from_numpy(qf[b])[None, :, None, :],
                                           torch.from_numpy(K.astype(np.float32))[None],
                                           torch.from_numpy(V.astype(np.float32))[None], scale=wl.scale)
        assert np.abs(o[0, :, 0].numpy() - ref[b]).max() <= 1e-5


def test_head_grouping_is_consecutive():
    """Query head h reads KV head h // G: making KV head 1 differ must change
    exactly the query heads G..2G-1."""
    wl = workloads.make_custom([40], 8, 2, 64, seed=3)
    base = run_oracle(wl)
    k2 = wl.k_pages.copy()
    k2[:, 1] = f32_to_bf16_bits(np.random.default_rng(0).standard_normal(k2[:, 1].shape).astype(np.float32))
    alt = run_oracle(wl, k_pages=k2)
    changed = np.abs(alt - base).max(axis=(0, 2)) > 0
    assert changed.tolist() == [False] * 4 + [True] * 4


# ---------------------------------------------------------------- closed forms
def test_constant_v_returns_the_constant():
    wl = workloads.make_custom([1, 5, 33, 200], 8, 2, 64, seed=5)
    c = f32_to_bf16_bits(np.float32([0.37]))[0]
    v = np.full_like(wl.v_pages, c)
    for prec, tol in (("f64", 1e-12), ("f32", 1e-6)):
        out = run_oracle(wl, prec, v_pages=v)
        assert np.abs(out - float(bf16_bits_to_f32(np.uint16([c]))[0])).max() <= tol


def test_length_one_returns_v_row_bit_exact():
    wl = workloads.make_custom([1, 1, 1], 4, 2, 128, seed=6)
    Vp = bf16_bits_to_f32(wl.v_pages)
    for prec in ("f64", "f32"):
        out = run_oracle(wl, prec)
        for b in range(3):
            for h in range(4):
                row = Vp[wl.block_table[b, 0], h // 2, 0]
                assert np.array_equal(out[b, h].astype(np.float32), row)


def test_zero_query_or_zero_scale_gives_mean_of_v():
    wl = workloads.make_custom([7, 50, 129], 4, 1, 64, seed=7)
    Vp = decode_pool(wl.v_pages, None, "bf16")
    means = [gather_dense(Vp, wl.block_table, b, 0, L).mean(axis=0) for b, L in enumerate(wl.context_lens)]
    out_q0 = run_oracle(wl, q=np.zeros_like(wl.q))
    out_s0 = run_oracle(wl, scale=0.0)
    for b in range(3):
        for h in range(4):
            assert np.abs(out_q0[b, h] - means[b]).max() <= 1e-12
            assert np.abs(out_s0[b, h] - means[b]).max() <= 1e-12


def test_equal_keys_give_mean_of_v():
    wl = workloads.make_custom([19, 64], 2, 1, 64, seed=8)
    k = wl.k_pages.copy()
    k[:] = k[wl.block_table[0, 0], 0, 0][None, None, None, :]
    Vp = decode_pool(wl.v_pages, None, "bf16")
    out = run_oracle(wl, k_pages=k)
    for b, L in enumerate(wl.context_lens):
        assert np.abs(out[b, 0] - gather_dense(Vp, wl.block_table, b, 0, L).mean(axis=0)).max() <= 1e-12


def test_dominant_key_selects_its_v_row():
    """One key = lambda * q/|q|, the others 0: out -> that V row with error
    <= (L-1) * exp(-scale*lambda*|q|) * 2*max|V|."""
    wl = workloads.make_custom([45], 1, 1, 64, seed=9)
    qf = bf16_bits_to_f32(wl.q)[0, 0]
    lam, t_star, L = 64.0, 29, 45
    k = np.zeros_like(wl.k_pages)
    krow = f32_to_bf16_bits((lam * qf / np.linalg.norm(qf)).astype(np.float32))
    k[wl.block_table[0, t_star // 16], 0, t_star % 16] = krow
    out = run_oracle(wl, k_pages=k)
    Vp = decode_pool(wl.v_pages, None, "bf16")
    V = gather_dense(Vp, wl.block_table, 0, 0, L)
    s_star = wl.scale * float(bf16_bits_to_f32(krow).astype(np.float64) @ qf.astype(np.float64))
    bound = (L - 1) * math.exp(-s_star) * 2 * np.abs(V).max()
    assert bound < 1e-3
    assert np.abs(out[0, 0] - V[t_star]).max() <= bound


def _golden_logistic():
    rows = []
    with open(os.path.join(GOLDEN, "two_token_weights.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(tuple(float(x) for x in line.split()))
    return rows


@pytest.mark.parametrize("delta,w_hi", _golden_logistic())
def test_two_tokens_weights_are_logistic(delta, w_hi):
    """Two tokens whose scores differ by delta get weights sigma(delta) and
    1 - sigma(delta); the tabulated sigma values are the textbook ones."""
    d = 64
    q = np.zeros((1, 1, d), np.float32); q[0, 0, 0] = 1.0
    k = np.zeros((1, 1, 16, d), np.float32); k[0, 0, 1, 0] = delta  # token 1 scores delta, token 0 scores 0
    v = np.zeros((1, 1, 16, d), np.float32); v[0, 0, 0, :] = -1.0; v[0, 0, 1, :] = 3.0
    out = oracle.paged_decode_attention(f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v),
                                        np.zeros((1, 1), np.int32), np.int32([2]), 1.0)
    assert abs(w_hi - 1.0 / (1.0 + math.exp(-delta))) < 1e-15  # the fixture itself
    assert np.abs(out[0, 0] - (3.0 * w_hi - 1.0 * (1 - w_hi))).max() <= 1e-12


def test_length_zero_gives_zero_row():
    wl = workloads.make_custom([0, 5], 2, 1, 64, seed=10)
    out = run_oracle(wl)
    assert np.array_equal(out[0], np.zeros_like(out[0])) and not np.isnan(out).any()


# ---------------------------------------------------------------- layout invariances (bit-exact)
def _repack(wl, new_table, new_num_pages):
    """Move every referenced page to the physical id new_table dictates."""
    k = np.full((new_num_pages,) + wl.k_pages.shape[1:], workloads.BF16_NAN_BITS, wl.k_pages.dtype)
    v = k.copy()
    for b in range(wl.batch):
        nb = (int(wl.context_lens[b]) + 15) // 16
        for j in range(nb):
            k[new_table[b, j]] = wl.k_pages[wl.block_table[b, j]]
            v[new_table[b, j]] = wl.v_pages[wl.block_table[b, j]]
    return k, v


def test_permuting_physical_pages_changes_nothing():
    wl = workloads.make_custom([100, 31, 257], 8, 2, 64, seed=12)
    perm = np.random.default_rng(1).permutation(wl.num_pages + 5).astype(np.int32)
    table = np.where(wl.block_table >= 0, perm[np.clip(wl.block_table, 0, None)], -1).astype(np.int32)
    k, v = _repack(wl, table, wl.num_pages + 5)
    for prec in ("f64", "f32"):
        assert np.array_equal(run_oracle(wl, prec), run_oracle(wl, prec, k_pages=k, v_pages=v, block_table=table))


def test_shared_prefix_pages_equal_private_copies():
    lens = np.array([300, 277, 411, 290])
    wl = workloads.make_custom(lens, 4, 2, 64, seed=13, session_of=[0, 0, 0, 1], prefix_len=[200, 200, 200, 96])
    # the three branches of session 0 really share pages, and the tail is copied
    assert np.array_equal(wl.block_table[0, :12], wl.block_table[1, :12])
    assert wl.block_table[0, 12] != wl.block_table[1, 12]
    # unshare: give every (sequence, logical page) its own physical page
    nbs = (lens + 15) // 16
    table = np.full_like(wl.block_table, -1)
    nxt = 0
    for b in range(4):
        table[b, :nbs[b]] = np.arange(nxt, nxt + nbs[b]); nxt += nbs[b]
    k, v = _repack(wl, table, nxt)
    a, c = run_oracle(wl), run_oracle(wl, k_pages=k, v_pages=v, block_table=table)
    assert np.array_equal(a, c)
    # and the shared prefix really is common: same K rows at logical position 150 and 199
    Kp = decode_pool(wl.k_pages, None, "bf16")
    for t in (150, 199):
        r0 = Kp[wl.block_table[0, t // 16], 0, t % 16]
        r2 = Kp[wl.block_table[2, t // 16], 0, t % 16]
        assert np.array_equal(r0, r2)


def test_pool_built_by_append_equals_pool_built_directly():
    wl = workloads.make_custom([37, 5, 64], 4, 2, 64, seed=14, poison=False)
    k = np.zeros_like(wl.k_pages); v = np.zeros_like(wl.v_pages)
    for b, L in enumerate(wl.context_lens):
        for t in range(L):  # one token at a time, as a decode loop would
            p, s = wl.block_table[b, t // 16], t % 16
            oracle.kv_append(wl.k_pages[p, :, s][None], wl.v_pages[p, :, s][None], np.int32([b]), np.int32([t]),
                             k, v, wl.block_table)
    valid = np.arange(16)[None, :] < wl.valid_slots[:, None]
    assert np.array_equal(k[valid.nonzero()[0], :, valid.nonzero()[1]], wl.k_pages[valid.nonzero()[0], :, valid.nonzero()[1]])
    assert np.array_equal(v[valid.nonzero()[0], :, valid.nonzero()[1]], wl.v_pages[valid.nonzero()[0], :, valid.nonzero()[1]])
    assert np.array_equal(run_oracle(wl), run_oracle(wl, k_pages=k, v_pages=v))


def test_kv_append_touches_only_its_slots():
    wl = workloads.make_custom([20, 33], 4, 2, 64, seed=15, append=True)
    k, v = wl.k_pages.copy(), wl.v_pages.copy()
    oracle.kv_append(wl.k_new, wl.v_new, wl.seq_ids, wl.positions, k, v, wl.block_table)
    diff = (k != wl.k_pages) | (v != wl.v_pages)
    where = set(zip(*[x.tolist() for x in diff.any(axis=3).nonzero()[:3:2]]))  # (page, slot)
    expect = {(int(wl.block_table[b, p // 16]), int(p % 16)) for b, p in zip(wl.seq_ids, wl.positions)}
    assert where == expect
    for j, (b, p) in enumerate(zip(wl.seq_ids, wl.positions)):
        assert np.array_equal(k[wl.block_table[b, p // 16], :, p % 16], wl.k_new[j])
        assert np.array_equal(v[wl.block_table[b, p // 16], :, p % 16], wl.v_new[j])
    assert not np.isnan(run_oracle(wl, k_pages=k, v_pages=v)).any()


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_poisoned_masked_slots_are_never_read(kv_dtype):
    a = workloads.make_custom([3, 47, 130], 8, 2, 64, kv_dtype, seed=16, poison=True)
    c = workloads.make_custom([3, 47, 130], 8, 2, 64, kv_dtype, seed=16, poison=False)
    assert (a.block_table[0, 1:] == -1).all()
    oa, oc = run_oracle(a), run_oracle(c)
    assert not np.isnan(oa).any() and np.array_equal(oa, oc)


# ---------------------------------------------------------------- split / merge identity
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_partials_merge_to_the_whole(kv_dtype):
    wl = workloads.make_custom([300], 4, 2, 64, kv_dtype, seed=17)
    whole = run_oracle(wl)
    kw = dict(k_scales=wl.k_scales, v_scales=wl.v_scales, kv_dtype=kv_dtype)
    for cuts in ([0, 300], [0, 1, 300], [0, 128, 256, 300], [0, 64, 64, 299, 300]):
        for h in range(4):
            parts = [oracle.partial(wl.q, wl.k_pages, wl.v_pages, wl.block_table, wl.scale, 0, h, a, b, **kw)
                     for a, b in zip(cuts[:-1], cuts[1:])]
            merged = oracle.combine([p[0] for p in parts], [p[1] for p in parts], np.stack([p[2] for p in parts]))
            assert np.abs(merged - whole[0, h]).max() <= 1e-12


def test_merge_of_empty_parts_is_zero():
    out = oracle.combine([-np.inf, -np.inf], [0.0, 0.0], np.zeros((2, 8)))
    assert np.array_equal(out, np.zeros(8))


# ---------------------------------------------------------------- fp8
def test_e4m3fn_decode_table_matches_torch():
    import torch

    codes = np.arange(256, dtype=np.uint8)
    ref = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float32).numpy()
    mine = np.array([oracle.e4m3fn_to_float(c) for c in codes], dtype=np.float32)
    assert np.array_equal(np.isnan(ref), np.isnan(mine)) and np.isnan(mine).sum() == 2
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], mine[ok])
    assert mine[0x7E] == 448.0 and mine[0x01] == 2.0 ** -9 and mine[0x08] == 2.0 ** -6


def test_e4m3fn_encoder_roundtrip_and_nearest():
    table = np.array([oracle.e4m3fn_to_float(c) for c in range(256)], dtype=np.float64)
    finite = ~np.isnan(table)
    codes = np.arange(256, dtype=np.uint8)[finite]
    back = f32_to_e4m3fn_bits(table[finite].astype(np.float32))
    keep = codes != 0x80  # -0 encodes as -0 too, but compare by value there
    assert np.array_equal(back[keep], codes[keep])
    x = np.random.default_rng(2).standard_normal(20000).astype(np.float32) * np.float32(100.0)
    got = table[f32_to_e4m3fn_bits(x)]
    best = np.abs(table[finite][None, :] - np.clip(x, -448, 448).astype(np.float64)[:, None]).min(axis=1)
    assert np.allclose(np.abs(got - np.clip(x, -448, 448)), best, rtol=0, atol=0)
    assert np.array_equal(f32_to_e4m3fn_bits(np.float32([1e9, -1e9])), np.uint8([0x7E, 0xFE]))


def test_fp8_with_power_of_two_scales_equals_bf16_of_dequantised():
    """code * 2^k is exactly representable in bf16 (3 mantissa bits), so the
    fp8 path must agree with the bf16 path on the dequantised values."""
    wl = workloads.make_custom([33, 90], 8, 2, 64, "fp8", seed=18)
    ks = np.exp2(np.round(np.log2(wl.k_scales))).astype(np.float32)
    vs = np.exp2(np.round(np.log2(wl.v_scales))).astype(np.float32)
    ks[np.isnan(ks)] = 1.0; vs[np.isnan(vs)] = 1.0
    kd = decode_pool(wl.k_pages, ks, "fp8").astype(np.float32)
    vd = decode_pool(wl.v_pages, vs, "fp8").astype(np.float32)
    kd[np.isnan(kd)] = 0; vd[np.isnan(vd)] = 0
    kb, vb = f32_to_bf16_bits(kd), f32_to_bf16_bits(vd)
    assert np.array_equal(bf16_bits_to_f32(kb), kd)  # exactness of the premise
    a = run_oracle(wl, k_scales=ks, v_scales=vs)
    b = oracle.paged_decode_attention(wl.q, kb, vb, wl.block_table, wl.context_lens, wl.scale)
    assert np.array_equal(a, b)


def test_fp8_scales_follow_the_recipe():
    wl = workloads.make_custom([20, 16], 2, 2, 64, "fp8", seed=19, poison=False)
    table = np.array([oracle.e4m3fn_to_float(c) for c in range(256)])
    for b, L in enumerate(wl.context_lens):
        for j in range((L + 15) // 16):
            p = wl.block_table[b, j]
            nvalid = min(16, L - 16 * j)
            for g in range(2):
                codes = wl.k_pages[p, g, :nvalid]
                assert np.abs(table[codes]).max() == 448.0  # absmax maps to the top code


# ---------------------------------------------------------------- generator sanity
def test_generator_is_deterministic_and_shaped():
    a, b = workloads.make_config(0), workloads.make_config(0)
    assert np.array_equal(a.k_pages, b.k_pages) and np.array_equal(a.block_table, b.block_table)
    assert a.batch == 4 and a.num_q_heads == 8 and a.num_kv_heads == 2 and a.head_dim == 64
    assert a.scale == 0.125 and (a.context_lens >= 1).all() and (a.context_lens <= 512).all()
    used = a.block_table[a.block_table >= 0]
    assert len(set(used.tolist())) == len(used)  # no page used twice without sharing
    c = workloads.make_config(0, seed=1)
    assert not np.array_equal(a.q, c.q)


def test_f32_oracle_agrees_with_f64_oracle():
    wl = workloads.make_custom([513, 700], 8, 2, 128, seed=20)
    assert np.abs(run_oracle(wl, "f32") - run_oracle(wl, "f64")).max() <= 1e-5

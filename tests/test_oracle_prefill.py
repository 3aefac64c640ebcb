"""Pins for the oracle's causal multi-query attention (CPU only): dense fp64 brute force with a
lower-right aligned causal mask, torch's scaled_dot_product_attention with the same mask, and the
special cases that tie it to single-query attention."""
import numpy as np
import pytest

import oracle
import workloads
from workloads import bf16_bits_to_f32, f32_to_bf16_bits
from tests.brute import decode_pool, gather_dense


def make(lens, nq, Hq, Hkv, d, kv_dtype="bf16", seed=0):
    wl = workloads.make_custom(lens, Hq, Hkv, d, kv_dtype, seed=seed)
    rng = np.random.default_rng(seed + 1)
    q_start = np.concatenate([[0], np.cumsum(nq)]).astype(np.int32)
    q = f32_to_bf16_bits(rng.standard_normal((int(q_start[-1]), Hq, d)).astype(np.float32))
    return wl, q, q_start


def run(wl, q, q_start, precision="f64"):
    return oracle.paged_prefill_attention(q, q_start, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens,
                                          wl.scale, wl.k_scales, wl.v_scales, wl.kv_dtype, precision)


def brute(wl, q, q_start):
    Kp, Vp = decode_pool(wl.k_pages, wl.k_scales, wl.kv_dtype), decode_pool(wl.v_pages, wl.v_scales, wl.kv_dtype)
    qf = bf16_bits_to_f32(q).astype(np.float64)
    G = wl.num_q_heads // wl.num_kv_heads
    out = np.zeros(qf.shape)
    for b, L in enumerate(wl.context_lens):
        n = q_start[b + 1] - q_start[b]
        for h in range(wl.num_q_heads):
            K, V = gather_dense(Kp, wl.block_table, b, h // G, L), gather_dense(Vp, wl.block_table, b, h // G, L)
            S = np.float64(np.float32(wl.scale)) * (qf[q_start[b]:q_start[b + 1], h] @ K.T)       # [n, L]
            pos = L - n + np.arange(n)
            S[np.arange(L)[None, :] > pos[:, None]] = -np.inf
            P = np.exp(S - S.max(axis=1, keepdims=True))
            out[q_start[b]:q_start[b + 1], h] = (P / P.sum(axis=1, keepdims=True)) @ V
    return out


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("Hq,Hkv,d", [(4, 2, 64), (7, 1, 128), (8, 8, 64)])
def test_prefill_matches_dense_causal_bruteforce(Hq, Hkv, d, kv_dtype):
    if kv_dtype == "fp8" and d != 128:
        d = 128
    wl, q, qs = make([40, 17, 64, 1], [40, 5, 16, 1], Hq, Hkv, d, kv_dtype, seed=Hq)
    assert np.abs(run(wl, q, qs) - brute(wl, q, qs)).max() <= 1e-12
    assert np.abs(run(wl, q, qs, "f32") - brute(wl, q, qs)).max() <= 1e-5


def test_prefill_matches_torch_sdpa_with_lower_right_causal_mask():
    import torch
    import torch.nn.functional as F
    wl, q, qs = make([50, 33], [20, 33], 4, 2, 64, seed=3)
    ref = run(wl, q, qs)
    Kp, Vp = decode_pool(wl.k_pages, None, "bf16"), decode_pool(wl.v_pages, None, "bf16")
    qf = bf16_bits_to_f32(q)
    for b, L in enumerate(wl.context_lens):
        n = qs[b + 1] - qs[b]
        K = np.stack([gather_dense(Kp, wl.block_table, b, h // 2, L) for h in range(4)]).astype(np.float32)
        V = np.stack([gather_dense(Vp, wl.block_table, b, h // 2, L) for h in range(4)]).astype(np.float32)
        Q = torch.from_numpy(qf[qs[b]:qs[b + 1]].transpose(1, 0, 2).copy())[None]                 # [1, H, n, d]
        mask = torch.from_numpy(np.arange(L)[None, :] <= (L - n + np.arange(n))[:, None])
        o = F.scaled_dot_product_attention(Q, torch.from_numpy(K)[None], torch.from_numpy(V)[None], attn_mask=mask, scale=wl.scale)
        assert np.abs(o[0].numpy().transpose(1, 0, 2) - ref[qs[b]:qs[b + 1]]).max() <= 1e-5


def test_one_query_per_sequence_is_the_decode_step():
    wl, q, qs = make([37, 64, 5], [1, 1, 1], 8, 2, 64, seed=4)
    dec = oracle.paged_decode_attention(q, wl.k_pages, wl.v_pages, wl.block_table, wl.context_lens, wl.scale)
    assert np.array_equal(run(wl, q, qs), dec)


def test_first_query_of_a_full_prefill_returns_the_first_v_row():
    wl, q, qs = make([20], [20], 2, 1, 64, seed=5)
    out = run(wl, q, qs)
    V = bf16_bits_to_f32(wl.v_pages)
    assert np.array_equal(out[0, 0].astype(np.float32), V[wl.block_table[0, 0], 0, 0])


def test_sequences_without_queries_and_with_too_many():
    wl, q, qs = make([10, 4], [0, 6], 2, 1, 64, seed=6)   # second sequence: 6 queries, 4 tokens
    out = run(wl, q, qs)
    assert out.shape[0] == 6 and not np.isnan(out).any()
    assert np.array_equal(out[:2], np.zeros_like(out[:2]))  # positions -2 and -1 do not exist
    assert np.abs(out[2:]).max() > 0

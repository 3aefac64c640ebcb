"""Dense fp64 brute force used to pin the oracle (never the other way round).

Gathers one sequence's K and V into dense [L, d] arrays through the block
table, then evaluates softmax(scale * K q) @ V with numpy in float64.  fp8
codes are decoded with torch's float8_e4m3fn, which is independent of the
oracle's own decoder.
"""
import numpy as np

from workloads import bf16_bits_to_f32


def decode_pool(pages, scales, kv_dtype):
    """Whole pool -> float64 [num_pages][Hkv][16][d]."""
    if kv_dtype == "bf16":
        return bf16_bits_to_f32(pages).astype(np.float64)
    import torch

    x = torch.from_numpy(pages.copy()).view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    return x * scales.astype(np.float64)[:, :, None, None]


def gather_dense(pool_f64, block_table, b, g, L):
    """[L, d] rows of sequence b, kv head g, in logical order."""
    t = np.arange(L)
    return pool_f64[block_table[b, t // 16], g, t % 16, :]


def brute_attention(wl, k_pages=None, v_pages=None, block_table=None, lens=None, q=None):
    k_pages = wl.k_pages if k_pages is None else k_pages
    v_pages = wl.v_pages if v_pages is None else v_pages
    block_table = wl.block_table if block_table is None else block_table
    lens = wl.context_lens if lens is None else lens
    q = wl.q if q is None else q
    Kp = decode_pool(k_pages, wl.k_scales, wl.kv_dtype)
    Vp = decode_pool(v_pages, wl.v_scales, wl.kv_dtype)
    qf = bf16_bits_to_f32(q).astype(np.float64)
    B, Hq, d = qf.shape
    G = Hq // wl.num_kv_heads
    out = np.zeros((B, Hq, d))
    for b in range(B):
        L = int(lens[b])
        if L == 0:
            continue
        for h in range(Hq):
            K = gather_dense(Kp, block_table, b, h // G, L)
            V = gather_dense(Vp, block_table, b, h // G, L)
            s = np.float64(np.float32(wl.scale)) * (K @ qf[b, h])
            p = np.exp(s - s.max())
            out[b, h] = (p / p.sum()) @ V
    return out

"""The prefix tree driving the kernels: trajectories of branching sessions are stored through
sd_tree, only their unmatched tokens are appended, and attention runs with the tree's block
tables and groups.  Checked against the oracle on the same pool (GPU only)."""
import numpy as np
import pytest

import oracle
import workloads
from tests.test_gpu_parity import check, sd  # noqa: F401  (fixture)
from tests.test_prefix_tree import random_session

pytestmark = pytest.mark.gpu


def test_tree_tables_and_groups_feed_the_prefix_entry_point(sd):
    import torch
    from paper_2508_11553_amd import binding
    from device_workload import _to_dev
    from paper_2508_11553_amd.prefix_tree import PrefixTree

    rng = np.random.default_rng(0)
    Hq, Hkv, d, num_pages = 8, 2, 128, 2048
    tree = PrefixTree(num_pages)
    ids, toks, matched = [], [], []
    for s in range(4):
        stem = rng.integers(0, 1000, size=600 + 300 * s).tolist()  # the session's common history
        for br in range(int(rng.integers(2, 9))):
            cut = len(stem) if br else 560  # one branch leaves the stem early, inside a page
            tr = stem[:cut] + rng.integers(0, 1000, size=int(rng.integers(1, 200))).tolist()
            i, m = tree.insert(tr)
            ids.append(i); toks.append(tr); matched.append(m)
    for tr in random_session(rng, 5, 300, vocab=1000):  # and a session that branches at random points
        i, m = tree.insert(tr)
        ids.append(i); toks.append(tr); matched.append(m)
    B = len(ids)
    lens = np.int32([len(t) for t in toks])
    maxnb = int((lens.max() + 15) // 16)
    bt = np.full((B, maxnb), -1, np.int32)
    for b, i in enumerate(ids):
        row = tree.block_table(i)
        bt[b, :len(row)] = row
    gs, sh = tree.batch_groups(ids)
    assert sh.max() >= 512  # the sessions really share long prefixes

    # append only what the tree says is new, on both sides
    k = np.full((num_pages, Hkv, 16, d), workloads.BF16_NAN_BITS, np.uint16); v = k.copy()
    rows_k, rows_v, seqs, poss = [], [], [], []
    for b in range(B):
        n = int(lens[b] - matched[b])
        rows_k.append(workloads.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d)).astype(np.float32)))
        rows_v.append(workloads.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d)).astype(np.float32)))
        seqs.append(np.full(n, b, np.int32)); poss.append(np.arange(matched[b], lens[b], dtype=np.int32))
    kn, vn, seqs, poss = np.concatenate(rows_k), np.concatenate(rows_v), np.concatenate(seqs), np.concatenate(poss)
    oracle.kv_append(kn, vn, seqs, poss, k, v, bt)
    q = workloads.f32_to_bf16_bits(rng.standard_normal((B, Hq, d)).astype(np.float32))
    scale = float(np.float32(1 / np.sqrt(d)))
    ref = oracle.paged_decode_attention(q, k, v, bt, lens, scale)
    assert not np.isnan(ref).any()  # every attended slot was written: the tree's bookkeeping is complete

    dev = "cuda:0"
    shape = sd.Shape(batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=16, num_pages=num_pages,
                     max_blocks_per_seq=maxnb, kv_dtype=sd.SD_BF16, max_context_len=int(lens.max()), chunk_tokens=256)
    dk = _to_dev(np.full_like(k, workloads.BF16_NAN_BITS), dev); dv = _to_dev(np.full_like(k, workloads.BF16_NAN_BITS), dev)
    dbt = _to_dev(bt, dev)
    binding.kv_append(shape, _to_dev(kn, dev), _to_dev(vn, dev), _to_dev(seqs, dev), _to_dev(poss, dev), len(seqs), dk, dv, dbt)
    out = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
    ws = torch.empty(sd.workspace_bytes(shape), dtype=torch.uint8, device=dev)
    binding.paged_decode_attention_prefix(shape, _to_dev(q, dev), dk, dv, None, None, dbt, _to_dev(lens, dev),
                                          _to_dev(gs, dev), _to_dev(sh, dev), len(gs) - 1, int(np.diff(gs).max()),
                                          int(sh.max()), scale, out, ws, ws.numel())
    torch.cuda.synchronize()
    assert np.array_equal(dk.cpu().numpy().view(np.uint16), k)
    check(out.cpu().numpy(), ref)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_copy_pages_matches_the_oracle_bit_for_bit(sd, kv_dtype):
    import torch
    from paper_2508_11553_amd import binding
    from device_workload import DeviceWorkload, _to_dev

    wl = workloads.make_custom([40, 70, 5, 130], 8, 4, 128, kv_dtype, seed=21, spare_pages=12)
    dw = DeviceWorkload(wl)
    free = [p for p in range(wl.num_pages) if p not in set(wl.block_table.ravel().tolist())]
    src = [int(wl.block_table[b, (L - 1) // 16]) for b, L in enumerate(wl.context_lens)]
    # valid pairs, then pairs that must be skipped: identity, out of range on either side
    srcs = np.int32(src + [src[0], -1, src[1], wl.num_pages])
    dsts = np.int32(free[:4] + [src[0], free[5], wl.num_pages, free[6]])
    binding.kv_copy_pages(dw.shape, _to_dev(srcs, dw.device), _to_dev(dsts, dw.device), len(srcs), dw.k_pages,
                          dw.v_pages, dw.k_scales, dw.v_scales)
    torch.cuda.synchronize()
    oracle.kv_copy_pages(srcs, dsts, wl.k_pages, wl.v_pages, wl.k_scales, wl.v_scales)
    k, v = dw.pools_to_host()
    assert np.array_equal(k, wl.k_pages) and np.array_equal(v, wl.v_pages)
    if kv_dtype == "fp8":
        # bit patterns: the scales of unused pages are NaN poison on both sides
        assert np.array_equal(dw.k_scales.cpu().numpy().view(np.uint32), wl.k_scales.view(np.uint32))
        assert np.array_equal(dw.v_scales.cpu().numpy().view(np.uint32), wl.v_scales.view(np.uint32))


def test_a_session_branches_inside_a_page_and_decodes_on(sd):
    """insert -> fork (copy the partly filled page) -> decode steps with sd_tree_append, kv_append and the
    prefix-aware attention; every step is checked against the oracle run on the host copy of the pool."""
    import torch
    from paper_2508_11553_amd import binding
    from device_workload import _to_dev
    from paper_2508_11553_amd.prefix_tree import PrefixTree

    rng = np.random.default_rng(7)
    Hq, Hkv, d, num_pages, maxnb = 8, 2, 128, 64, 8
    dev = "cuda:0"
    scale = float(np.float32(1 / np.sqrt(d)))
    tree = PrefixTree(num_pages)
    k = np.full((num_pages, Hkv, 16, d), workloads.BF16_NAN_BITS, np.uint16); v = k.copy()
    dk, dv = _to_dev(k, dev), _to_dev(v, dev)

    def rows(n):
        return (workloads.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d)).astype(np.float32)),
                workloads.f32_to_bf16_bits(rng.standard_normal((n, Hkv, d)).astype(np.float32)))

    def table(ids):
        bt = np.full((len(ids), maxnb), -1, np.int32)
        for b, i in enumerate(ids):
            r = tree.block_table(i)
            bt[b, :len(r)] = r
        return bt

    def shape_for(B, maxlen):
        return sd.Shape(batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=16, num_pages=num_pages,
                        max_blocks_per_seq=maxnb, kv_dtype=sd.SD_BF16, max_context_len=maxlen, chunk_tokens=128)

    def append_both(kn, vn, seqs, poss, bt, B, maxlen):
        oracle.kv_append(kn, vn, seqs, poss, k, v, bt)
        binding.kv_append(shape_for(B, maxlen), _to_dev(kn, dev), _to_dev(vn, dev), _to_dev(seqs, dev),
                          _to_dev(poss, dev), len(seqs), dk, dv, _to_dev(bt, dev))

    # the session's history: 41 tokens = two full pages and nine tokens of a third
    prompt = rng.integers(0, 1000, size=41).tolist()
    root, _ = tree.insert(prompt)
    kn, vn = rows(41)
    append_both(kn, vn, np.zeros(41, np.int32), np.arange(41, dtype=np.int32), table([root]), 1, 41)
    # three more branches: each gets a private copy of the third page
    ids, src, dst = [root], [], []
    for _ in range(3):
        i, s, t_ = tree.fork(root)
        ids.append(i); src.append(s); dst.append(t_)
    src, dst = np.int32(src), np.int32(dst)
    oracle.kv_copy_pages(src, dst, k, v)
    binding.kv_copy_pages(shape_for(4, 41), _to_dev(src, dev), _to_dev(dst, dev), 3, dk, dv)
    B = len(ids)
    for step in range(20):  # crosses the page boundary at 48 and fills a second private page
        poss = np.int32([tree.length(i) for i in ids])
        for i in ids:
            tree.append(i, int(rng.integers(0, 1000)))
        bt = table(ids)
        lens = poss + 1
        kn, vn = rows(B)
        append_both(kn, vn, np.arange(B, dtype=np.int32), poss, bt, B, int(lens.max()))
        q = workloads.f32_to_bf16_bits(rng.standard_normal((B, Hq, d)).astype(np.float32))
        gs, sh = tree.batch_groups(ids)
        assert gs.tolist() == [0, B] and sh.tolist() == [32] * B   # the two full pages of the history stay shared
        ref = oracle.paged_decode_attention(q, k, v, bt, lens, scale)
        assert not np.isnan(ref).any()
        shp = shape_for(B, int(lens.max()))
        out = torch.empty((B, Hq, d), dtype=torch.float32, device=dev)
        ws = torch.empty(sd.workspace_bytes(shp), dtype=torch.uint8, device=dev)
        binding.paged_decode_attention_prefix(shp, _to_dev(q, dev), dk, dv, None, None, _to_dev(bt, dev),
                                              _to_dev(lens, dev), _to_dev(gs, dev), _to_dev(sh, dev), 1, B, 32, scale,
                                              out, ws, ws.numel())
        torch.cuda.synchronize()
        check(out.cpu().numpy(), ref)
    assert np.array_equal(dk.cpu().numpy().view(np.uint16), k) and np.array_equal(dv.cpu().numpy().view(np.uint16), v)

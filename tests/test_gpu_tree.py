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
    from paper_2508_11553_amd.device import _to_dev
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

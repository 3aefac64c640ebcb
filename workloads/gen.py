"""Seeded generators for the paged-KV decode workloads.

Layout produced (and nothing else is assumed anywhere downstream):

  q            uint16  [B][Hq][d]                 bf16 bit patterns
  k_pages      uint16  [num_pages][Hkv][16][d]    bf16 bits   (kv_dtype 'bf16')
               uint8   [num_pages][Hkv][16][d]    e4m3fn codes (kv_dtype 'fp8')
  v_pages      same shape/dtype as k_pages, separate pool
  k_scales     float32 [num_pages][Hkv]           fp8 only, absmax(valid)/448
  v_scales     float32 [num_pages][Hkv]           fp8 only
  block_table  int32   [B][max_blocks_per_seq]    physical page of logical page j
  context_lens int32   [B]

Token t of sequence b lives in page block_table[b][t // 16], slot t % 16.

Random streams: numpy PCG64 generators keyed by SeedSequence([seed, tag, i])
with one tag per quantity (lengths, q, permutation, pools, appended rows) and
i the chunk index for pools, so pools can be drawn in parallel chunks and in
physical order while staying reproducible.  Values are N(0,1) in float32 and
then rounded to the storage format; every consumer starts from the rounded
bytes.

Everything that must never be read is poisoned: slots past a sequence's
length in its last page, pages nobody references, block-table entries past
the last logical page (-1), the scales of unreferenced pages, and (when an
append is requested) the slot the append will fill.
"""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

from .formats import (
    BF16_NAN_BITS,
    E4M3FN_MAX,
    E4M3FN_NAN_BITS,
    f32_to_bf16_bits,
    f32_to_e4m3fn_bits,
)

PAGE = 16
_TAG_LENS, _TAG_Q, _TAG_PERM, _TAG_K, _TAG_V, _TAG_APPEND, _TAG_MISC = range(7)
_CHUNK_PAGES = 256  # pages drawn per random stream chunk (small enough to stay in cache)


def _rng(seed, tag, idx=0):
    return np.random.default_rng(np.random.SeedSequence([int(seed), int(tag), int(idx)]))


@dataclass
class Workload:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    kv_dtype: str  # 'bf16' | 'fp8'
    scale: float
    num_pages: int
    max_blocks_per_seq: int
    max_context_len: int
    q: np.ndarray
    k_pages: np.ndarray
    v_pages: np.ndarray
    block_table: np.ndarray
    context_lens: np.ndarray
    k_scales: Optional[np.ndarray] = None
    v_scales: Optional[np.ndarray] = None
    # rows the caller appends before attending (None when no append is staged)
    k_new: Optional[np.ndarray] = None  # uint16 [T][Hkv][d]
    v_new: Optional[np.ndarray] = None
    seq_ids: Optional[np.ndarray] = None  # int32 [T]
    positions: Optional[np.ndarray] = None  # int32 [T]
    # sessions whose branches share prefix pages: group j = sequences group_start[j] .. group_start[j+1]-1,
    # shared_len[b] = leading tokens of b whose pages all members of its group share (a multiple of 16)
    group_start: Optional[np.ndarray] = None  # int32 [num_groups + 1]
    shared_len: Optional[np.ndarray] = None  # int32 [B]
    # bookkeeping for reports
    unique_tokens: int = 0
    seed: int = 0
    page_size: int = PAGE
    valid_slots: Optional[np.ndarray] = field(default=None, repr=False)  # int32 [num_pages]

    @property
    def attended_tokens(self) -> int:
        return int(self.context_lens.astype(np.int64).sum())

    @property
    def kv_elem_bytes(self) -> int:
        return 1 if self.kv_dtype == "fp8" else 2

    @property
    def token_bytes(self) -> int:
        """K+V bytes of one token over all KV heads."""
        return self.num_kv_heads * self.head_dim * 2 * self.kv_elem_bytes


def _draw_pool(seed, tag, num_pages, Hkv, d, kv_dtype, valid, threads):
    """Draw one pool in physical order, chunk by chunk."""
    if kv_dtype == "bf16":
        pool = np.empty((num_pages, Hkv, PAGE, d), dtype=np.uint16)
        scales = None
    else:
        pool = np.empty((num_pages, Hkv, PAGE, d), dtype=np.uint8)
        scales = np.empty((num_pages, Hkv), dtype=np.float32)
    slot = np.arange(PAGE, dtype=np.int32)

    def work(ci):
        p0 = ci * _CHUNK_PAGES
        p1 = min(num_pages, p0 + _CHUNK_PAGES)
        x = _rng(seed, tag, ci).standard_normal((p1 - p0, Hkv, PAGE, d), dtype=np.float32)
        if kv_dtype == "bf16":
            pool[p0:p1] = f32_to_bf16_bits(x)
        else:
            ok = slot[None, :] < valid[p0:p1, None]  # [pages][16]
            ax = np.abs(x) * ok[:, None, :, None]
            amax = ax.max(axis=(2, 3))
            sc = np.where(amax > 0, amax / np.float32(E4M3FN_MAX), np.float32(1.0)).astype(np.float32)
            scales[p0:p1] = sc
            pool[p0:p1] = f32_to_e4m3fn_bits(x / sc[:, :, None, None])

    nchunks = (num_pages + _CHUNK_PAGES - 1) // _CHUNK_PAGES
    if threads > 1 and nchunks > 1:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(nchunks)))
    else:
        for ci in range(nchunks):
            work(ci)
    return pool, scales


def build_paged(
    name,
    lens,
    Hq,
    Hkv,
    d,
    kv_dtype="bf16",
    seed=0,
    scale=None,
    session_of=None,
    prefix_len=None,
    append=False,
    poison=True,
    spare_pages=2,
    permute=True,
    max_blocks_per_seq=None,
    threads=None,
):
    """Build a paged workload for given context lengths.

    lens[b] is the length attention runs with.  With append=True the token at
    position lens[b]-1 is NOT in the pool: its K/V rows are returned as
    k_new/v_new for the caller to append first.

    session_of[b], prefix_len[b]: sequences of one session share the physical
    pages that lie fully inside their common prefix (prefix_len must be equal
    within a session); a prefix tail that does not fill a page is copied into
    each branch's own page.
    """
    lens = np.asarray(lens, dtype=np.int64)
    B = int(lens.shape[0])
    assert Hq % Hkv == 0
    assert kv_dtype in ("bf16", "fp8")
    if threads is None:
        threads = min(16, os.cpu_count() or 1)
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    nb = (lens + PAGE - 1) // PAGE
    maxnb = int(max(1, nb.max() if B else 1))
    if max_blocks_per_seq is None:
        max_blocks_per_seq = maxnb
    assert max_blocks_per_seq >= maxnb

    # ---- logical page ids ------------------------------------------------
    table = np.full((B, max_blocks_per_seq), -1, dtype=np.int64)
    next_id = 0
    shared_first = {}
    shared_pages = np.zeros(B, dtype=np.int64)
    if session_of is not None:
        session_of = np.asarray(session_of)
        prefix_len = np.asarray(prefix_len, dtype=np.int64)
        for b in range(B):
            s = int(session_of[b])
            ns = int(prefix_len[b] // PAGE)
            assert prefix_len[b] <= lens[b] - (1 if append else 0)
            if s not in shared_first:
                shared_first[s] = (next_id, ns, int(prefix_len[b]), b)
                next_id += ns
            first, ns0, p0, _ = shared_first[s]
            assert ns0 == ns and p0 == int(prefix_len[b]), "prefix length differs inside a session"
            table[b, :ns] = np.arange(first, first + ns)
            shared_pages[b] = ns
    for b in range(B):
        npriv = int(nb[b] - shared_pages[b])
        table[b, shared_pages[b]:nb[b]] = np.arange(next_id, next_id + npriv)
        next_id += npriv
    n_used = next_id
    num_pages = n_used + spare_pages

    # ---- physical placement ------------------------------------------------
    if permute:
        perm = _rng(seed, _TAG_PERM).permutation(num_pages).astype(np.int64)
    else:
        perm = np.arange(num_pages, dtype=np.int64)
    block_table = np.where(table >= 0, perm[np.clip(table, 0, None)], -1).astype(np.int32)

    valid = np.zeros(num_pages, dtype=np.int32)
    for b in range(B):
        n = int(nb[b])
        if n == 0:
            continue
        cnt = np.minimum(PAGE, lens[b] - PAGE * np.arange(n)).astype(np.int32)
        phys = block_table[b, :n]
        valid[phys] = np.maximum(valid[phys], cnt)

    # tokens actually stored before the call: with a staged append the last token of each
    # sequence is not in the pool yet (fp8 scales are taken over the stored tokens only)
    stored = valid
    if append:
        stored = valid.copy()
        for b in range(B):
            if lens[b] > 0:
                last = block_table[b, (lens[b] - 1) // PAGE]
                stored[last] = min(stored[last], (lens[b] - 1) % PAGE)

    # ---- draws ---------------------------------------------------------------
    q = f32_to_bf16_bits(_rng(seed, _TAG_Q).standard_normal((B, Hq, d), dtype=np.float32))
    k_pages, k_scales = _draw_pool(seed, _TAG_K, num_pages, Hkv, d, kv_dtype, stored, threads)
    v_pages, v_scales = _draw_pool(seed, _TAG_V, num_pages, Hkv, d, kv_dtype, stored, threads)

    # prefix tails that do not fill a page: same values in every branch.  bf16: the tail's bytes are
    # copied from the session's first branch.  fp8: codes only mean something together with their
    # page's scale, so every branch gets the codes AND scales of the whole page of the session's
    # longest branch (its scale covers a superset of each branch's own tokens in that page; slots a
    # shorter branch does not own are poisoned below like any other slot past a sequence's end).
    if session_of is not None:
        for b in range(B):
            s_id = int(session_of[b])
            _, ns, p, b0 = shared_first[s_id]
            tail = p % PAGE
            if not tail:
                continue
            if kv_dtype == "bf16":
                if b != b0:
                    src, dst = block_table[b0, ns], block_table[b, ns]
                    k_pages[dst, :, :tail] = k_pages[src, :, :tail]
                    v_pages[dst, :, :tail] = v_pages[src, :, :tail]
            else:
                members = np.nonzero(session_of == s_id)[0]
                bsrc = int(members[np.argmax(lens[members])])
                if b != bsrc:
                    src, dst = block_table[bsrc, ns], block_table[b, ns]
                    k_pages[dst], v_pages[dst] = k_pages[src], v_pages[src]
                    k_scales[dst], v_scales[dst] = k_scales[src], v_scales[src]

    wl = Workload(
        name=name, batch=B, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, kv_dtype=kv_dtype,
        scale=float(np.float32(scale)), num_pages=num_pages, max_blocks_per_seq=int(max_blocks_per_seq),
        max_context_len=int(max(1, lens.max() if B else 1)), q=q, k_pages=k_pages, v_pages=v_pages,
        block_table=block_table, context_lens=lens.astype(np.int32), k_scales=k_scales, v_scales=v_scales,
        seed=seed, valid_slots=valid,
    )
    uniq = int(valid.astype(np.int64).sum())
    wl.unique_tokens = uniq
    if session_of is not None:
        change = np.nonzero(np.diff(session_of))[0] + 1
        assert len(set(session_of.tolist())) == len(change) + 1, "sequences of a session must be consecutive"
        wl.group_start = np.concatenate([[0], change, [B]]).astype(np.int32)
        wl.shared_len = (shared_pages * PAGE).astype(np.int32)

    if append:
        assert session_of is None or kv_dtype == "bf16"
        rows = np.nonzero(lens > 0)[0]
        r = _rng(seed, _TAG_APPEND)
        wl.k_new = f32_to_bf16_bits(r.standard_normal((len(rows), Hkv, d), dtype=np.float32))
        wl.v_new = f32_to_bf16_bits(r.standard_normal((len(rows), Hkv, d), dtype=np.float32))
        wl.seq_ids = rows.astype(np.int32)
        wl.positions = (lens[rows] - 1).astype(np.int32)

    if poison:
        nan = BF16_NAN_BITS if kv_dtype == "bf16" else E4M3FN_NAN_BITS
        slot = np.arange(PAGE)
        partial = np.nonzero(valid < PAGE)[0]
        for p in partial:
            k_pages[p, :, valid[p]:] = nan
            v_pages[p, :, valid[p]:] = nan
        if k_scales is not None:
            k_scales[stored == 0] = np.nan
            v_scales[stored == 0] = np.nan
        if append:
            for b, pos in zip(wl.seq_ids, wl.positions):
                p = block_table[b, pos // PAGE]
                k_pages[p, :, pos % PAGE] = nan
                v_pages[p, :, pos % PAGE] = nan
        del slot
    return wl


def draw_extra_pool(wl: Workload, seed: int):
    """A second K/V pool of the same shape with independent values (same table).

    Used to rotate the benchmark over several pools so that no cache level can
    hold the working set between iterations.  bf16 pools keep the poison of the
    original; fp8 pools come with their own scales.
    """
    k, ks = _draw_pool(seed, _TAG_K, wl.num_pages, wl.num_kv_heads, wl.head_dim, wl.kv_dtype, wl.valid_slots, 8)
    v, vs = _draw_pool(seed, _TAG_V, wl.num_pages, wl.num_kv_heads, wl.head_dim, wl.kv_dtype, wl.valid_slots, 8)
    return k, v, ks, vs


CONFIG_NAMES = {
    0: "tiny paged decode",
    1: "7B-shaped rollout step",
    2: "long-horizon agent step",
    3: "partial-rollout / branching mix",
    4: "large-batch decode, fp8 KV",
}


_CONFIG_SHAPES = {  # (Hq, Hkv, d, kv_dtype)
    0: (8, 2, 64, "bf16"),
    1: (28, 4, 128, "bf16"),
    2: (64, 8, 128, "bf16"),
    3: (32, 8, 128, "bf16"),
    4: (64, 8, 128, "fp8"),
}


def config_lengths(idx: int, seed: int = 0):
    """Context lengths of workload `idx` (and, for the branching mix, the
    session of each sequence and its shared prefix length)."""
    r = _rng(seed, _TAG_LENS)
    if idx == 0:
        return r.integers(1, 512, size=4, endpoint=True), None, None
    if idx == 1:
        return r.integers(1024, 8192, size=64, endpoint=True), None, None
    if idx == 2:
        lens = np.rint(np.exp(r.normal(math.log(16384.0), 1.0, size=32))).astype(np.int64)
        return np.clip(lens, 2048, 65536), None, None
    if idx == 3:
        nsess, nbr = 16, 16
        prefix = r.integers(2048, 16384, size=nsess, endpoint=True)
        suffix = r.integers(64, 4096, size=nsess * nbr, endpoint=True)
        session_of = np.repeat(np.arange(nsess), nbr)
        prefix_len = prefix[session_of]
        return prefix_len + suffix + 1, session_of, prefix_len  # +1: the token the append writes
    if idx == 4:
        return r.integers(512, 4096, size=1024, endpoint=True), None, None
    raise ValueError(f"no config {idx}")


def make_config(idx: int, seed: int = 0, append: Optional[bool] = None, threads=None, batch: Optional[int] = None):
    """The five benchmark workloads.  `batch` (optional) keeps only the first
    `batch` sequences, for bounded CPU timing samples and tests.  The branching
    mix stages its one-token append by default; the others on request."""
    lens, session_of, prefix_len = config_lengths(idx, seed)
    if batch is not None:
        lens = lens[:batch]
        if session_of is not None:
            session_of, prefix_len = session_of[:batch], prefix_len[:batch]
    Hq, Hkv, d, dt = _CONFIG_SHAPES[idx]
    if append is None:
        append = idx == 3
    return build_paged(CONFIG_NAMES[idx], lens, Hq, Hkv, d, dt, seed=seed, session_of=session_of,
                       prefix_len=prefix_len, append=append, threads=threads)


def make_custom(lens, Hq, Hkv, d, kv_dtype="bf16", seed=0, **kw):
    """Small ad-hoc workloads for tests."""
    return build_paged("custom", lens, Hq, Hkv, d, kv_dtype, seed=seed, **kw)

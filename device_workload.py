"""Device-side holder for one decode workload: uploads host arrays into torch
tensors once, sizes the workspace, and forwards to the C ABI.  No arithmetic
happens here; torch is used for device memory and streams only.
"""
from __future__ import annotations

import numpy as np
import torch

import paper_2508_11553_amd as sd


def _to_dev(a: np.ndarray, device) -> torch.Tensor:
    """numpy -> device tensor with the same bytes (uint16 travels as int16)."""
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device, non_blocking=False)


class DeviceWorkload:
    """Anything with the fields of workloads.Workload can be uploaded."""

    def __init__(self, wl, device="cuda:0", chunk_tokens: int = 0, upload_pools: bool = True,
                 balance_for_batch: bool = False):
        """chunk_tokens = 0 leaves the chunk to the library; balance_for_batch asks it for the chunk that
        fits this batch's token count (which a scheduler knows on the host) instead of the shape-only guess."""
        self.wl = wl
        self.device = torch.device(device)
        self.shape = sd.Shape(
            batch=wl.batch, num_q_heads=wl.num_q_heads, num_kv_heads=wl.num_kv_heads, head_dim=wl.head_dim,
            page_size=wl.page_size, num_pages=wl.num_pages, max_blocks_per_seq=wl.max_blocks_per_seq,
            kv_dtype=sd.SD_FP8_E4M3 if wl.kv_dtype == "fp8" else sd.SD_BF16,
            max_context_len=wl.max_context_len, chunk_tokens=chunk_tokens)
        if balance_for_batch and not chunk_tokens:
            self.shape.chunk_tokens = sd.chunk_for_batch(self.shape, int(wl.unique_tokens))
        self.scale = float(wl.scale)
        self.q = _to_dev(wl.q, self.device)
        self.block_table = _to_dev(wl.block_table, self.device)
        self.context_lens = _to_dev(wl.context_lens, self.device)
        self.k_pages = self.v_pages = self.k_scales = self.v_scales = None
        if upload_pools:
            self.set_pool(wl.k_pages, wl.v_pages, wl.k_scales, wl.v_scales)
        self.k_new = self.v_new = self.seq_ids = self.positions = None
        self.T = 0
        if getattr(wl, "k_new", None) is not None:
            self.k_new, self.v_new = _to_dev(wl.k_new, self.device), _to_dev(wl.v_new, self.device)
            self.seq_ids, self.positions = _to_dev(wl.seq_ids, self.device), _to_dev(wl.positions, self.device)
            self.T = int(wl.k_new.shape[0])
            # the same rows as ranges of one token each, for the fp8 append
            self.range_row0 = _to_dev(np.arange(self.T + 1, dtype=np.int32), self.device)
            # and as one row per sequence in batch order (zeros where nothing is staged), for the call that appends and attends
            if wl.k_new.dtype == np.uint16 and wl.kv_dtype == "bf16":
                full_k = np.zeros((wl.batch,) + wl.k_new.shape[1:], np.uint16)
                full_v = full_k.copy()
                full_k[wl.seq_ids], full_v[wl.seq_ids] = wl.k_new, wl.v_new
                self.k_new_rows, self.v_new_rows = _to_dev(full_k, self.device), _to_dev(full_v, self.device)
        self.group_start = self.shared_len = None
        self.num_groups = self.max_group_size = self.max_shared_len = 0
        if getattr(wl, "group_start", None) is not None:
            self.group_start, self.shared_len = _to_dev(wl.group_start, self.device), _to_dev(wl.shared_len, self.device)
            self.num_groups = int(len(wl.group_start) - 1)
            self.max_group_size = int(np.diff(wl.group_start).max())
            self.max_shared_len = int(wl.shared_len.max())
        self.out = torch.empty((wl.batch, wl.num_q_heads, wl.head_dim), dtype=torch.float32, device=self.device)
        self.ws_bytes = sd.workspace_bytes(self.shape)
        self.workspace = torch.empty(max(self.ws_bytes, 256), dtype=torch.uint8, device=self.device)

    def set_pool(self, k_pages, v_pages, k_scales=None, v_scales=None):
        """Upload (numpy) or adopt (torch) a K/V pool."""
        up = lambda a: a if a is None or isinstance(a, torch.Tensor) else _to_dev(a, self.device)
        self.k_pages, self.v_pages = up(k_pages), up(v_pages)
        self.k_scales, self.v_scales = up(k_scales), up(v_scales)

    def chunk_tokens(self) -> int:
        return sd.chunk_tokens(self.shape)

    def append(self, stream=None):
        if self.shape.kv_dtype == sd.SD_FP8_E4M3:
            sd.kv_append_fp8(self.shape, self.k_new, self.v_new, self.seq_ids, self.positions, self.range_row0,
                             self.T, 1, self.k_pages, self.v_pages, self.k_scales, self.v_scales, self.block_table,
                             stream)
            return
        sd.kv_append(self.shape, self.k_new, self.v_new, self.seq_ids, self.positions, self.T,
                     self.k_pages, self.v_pages, self.block_table, stream)

    def attend(self, stream=None, timer=None, out=None):
        out = self.out if out is None else out
        sd.paged_decode_attention(self.shape, self.q, self.k_pages, self.v_pages, self.k_scales, self.v_scales,
                                  self.block_table, self.context_lens, self.scale, out, self.workspace,
                                  self.ws_bytes, stream, timer)
        return out

    def append_and_attend(self, stream=None, timer=None, out=None):
        """One call: the staged newest tokens (one per sequence, in batch order) go into the pool and are attended."""
        out = self.out if out is None else out
        sd.paged_decode_attention_append(self.shape, self.q, self.k_new_rows, self.v_new_rows, self.k_pages, self.v_pages,
                                         self.block_table, self.context_lens, self.scale, out, self.workspace,
                                         self.ws_bytes, stream, timer)
        return out

    def attend_prefix(self, stream=None, timer=None, out=None):
        """Shared-prefix aware call (needs the workload's group_start / shared_len)."""
        out = self.out if out is None else out
        sd.paged_decode_attention_prefix(self.shape, self.q, self.k_pages, self.v_pages, self.k_scales, self.v_scales,
                                         self.block_table, self.context_lens, self.group_start, self.shared_len,
                                         self.num_groups, self.max_group_size, self.max_shared_len, self.scale, out,
                                         self.workspace, self.ws_bytes, stream, timer)
        return out

    def attend_prefill(self, q_rows, q_start, stream=None, timer=None):
        """Causal attention of the query rows q_rows ([rows][Hq][d] bf16 bits, numpy) split by q_start ([B+1])."""
        q_start = np.asarray(q_start, dtype=np.int32)
        q_dev, qs_dev = _to_dev(q_rows, self.device), _to_dev(q_start, self.device)
        rows = int(q_rows.shape[0])
        out = torch.zeros((rows, self.wl.num_q_heads, self.wl.head_dim), dtype=torch.float32, device=self.device)
        max_q = int(np.diff(q_start).max()) if len(q_start) > 1 else 0
        sd.paged_prefill_attention(self.shape, q_dev, qs_dev, rows, max_q, self.k_pages, self.v_pages, self.k_scales,
                                   self.v_scales, self.block_table, self.context_lens, self.scale, out, stream, timer)
        return out

    def pools_to_host(self):
        """Pool bytes back as numpy arrays of the workload's dtype."""
        k, v = self.k_pages.cpu().numpy(), self.v_pages.cpu().numpy()
        if k.dtype == np.int16:
            k, v = k.view(np.uint16), v.view(np.uint16)
        return k, v

"""ctypes binding: same names as the C ABI, argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libseamdecode.so")
_lib = None

SD_BF16 = 0
SD_FP8_E4M3 = 1


class SeamDecodeError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} (code {code}, hip {load().sd_last_hip_error()})")


class Shape(ctypes.Structure):
    """Mirror of sd_shape."""
    _fields_ = [
        ("batch", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("page_size", ctypes.c_int32),
        ("num_pages", ctypes.c_int32),
        ("max_blocks_per_seq", ctypes.c_int32),
        ("kv_dtype", ctypes.c_int32),
        ("max_context_len", ctypes.c_int32),
        ("chunk_tokens", ctypes.c_int32),
    ]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libseamdecode.so (built beforehand by build.py); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2508_11553_amd.build` "
            "(hipcc, --offload-arch=gfx950). There is no fallback path.")
    L = ctypes.CDLL(_LIB_PATH)
    vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
    sp = ctypes.POINTER(Shape)
    L.sd_version.restype = ctypes.c_int
    L.sd_version.argtypes = []
    L.sd_strerror.restype = ctypes.c_char_p
    L.sd_strerror.argtypes = [ctypes.c_int]
    L.sd_last_hip_error.restype = ctypes.c_int
    L.sd_last_hip_error.argtypes = []
    L.sd_chunk_tokens.restype = ctypes.c_int
    L.sd_chunk_tokens.argtypes = [sp]
    L.sd_chunk_for_batch.restype = ctypes.c_int
    L.sd_chunk_for_batch.argtypes = [sp, ctypes.c_int64]
    L.sd_workspace_bytes.restype = sz
    L.sd_workspace_bytes.argtypes = [sp]
    L.kv_append.restype = ctypes.c_int
    L.kv_append.argtypes = [sp, vp, vp, vp, vp, i32, vp, vp, vp, vp]
    L.paged_decode_attention.restype = ctypes.c_int
    L.paged_decode_attention.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, sz, vp]
    L.paged_decode_attention_append.restype = ctypes.c_int
    L.paged_decode_attention_append.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, sz, vp, vp]
    L.paged_decode_attention_static.restype = ctypes.c_int
    L.paged_decode_attention_static.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp]
    L.paged_decode_attention_timed.restype = ctypes.c_int
    L.paged_decode_attention_timed.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, f32, vp, vp, sz, vp, vp]
    L.kv_append_fp8.restype = ctypes.c_int
    L.kv_append_fp8.argtypes = [sp, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
    L.paged_decode_attention_prefix.restype = ctypes.c_int
    L.paged_decode_attention_prefix.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp, vp, sz,
                                                vp, vp]
    L.kv_copy_pages.restype = ctypes.c_int
    L.kv_copy_pages.argtypes = [sp, vp, vp, i32, vp, vp, vp, vp, vp]
    L.paged_prefill_attention.restype = ctypes.c_int
    L.paged_prefill_attention.argtypes = [sp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, f32, vp, vp, vp]
    L.sd_validate_tables.restype = ctypes.c_int
    L.sd_validate_tables.argtypes = [sp, vp, vp, vp, vp]
    L.sd_validate_groups.restype = ctypes.c_int
    L.sd_validate_groups.argtypes = [sp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
    L.sd_timer_create.restype = vp
    L.sd_timer_create.argtypes = [i32]
    L.sd_timer_destroy.restype = None
    L.sd_timer_destroy.argtypes = [vp]
    L.sd_timer_reset.restype = None
    L.sd_timer_reset.argtypes = [vp]
    L.sd_timer_read.restype = ctypes.c_int
    L.sd_timer_read.argtypes = [vp, vp, vp, i32]
    L.sd_range_parts.restype = ctypes.c_int
    L.sd_range_parts.argtypes = [i32, i32, i32, i32, vp, i32]
    L.sd_probe_sink_words.restype = sz
    L.sd_probe_sink_words.argtypes = [sp]
    L.sd_probe_read.restype = ctypes.c_int
    L.sd_probe_read.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, vp]
    _lib = L
    return L


def version() -> int:
    return int(load().sd_version())


def strerror(code: int) -> str:
    return load().sd_strerror(int(code)).decode()


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, a raw int address, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch

        return int(torch.cuda.current_stream().cuda_stream) or None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


def _check(rc: int, what: str):
    if rc != 0:
        raise SeamDecodeError(rc, what)


def chunk_tokens(shape: Shape) -> int:
    rc = int(load().sd_chunk_tokens(ctypes.byref(shape)))
    if rc <= 0:
        raise SeamDecodeError(rc, "sd_chunk_tokens")
    return rc


def chunk_for_batch(shape: Shape, total_tokens: int) -> int:
    rc = int(load().sd_chunk_for_batch(ctypes.byref(shape), int(total_tokens)))
    if rc <= 0:
        raise SeamDecodeError(rc, "sd_chunk_for_batch")
    return rc


def workspace_bytes(shape: Shape) -> int:
    return int(load().sd_workspace_bytes(ctypes.byref(shape)))


def kv_append(shape: Shape, k_new, v_new, seq_ids, positions, T: int, k_pages, v_pages, block_table, stream=None):
    rc = load().kv_append(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(seq_ids), _ptr(positions), int(T),
                          _ptr(k_pages), _ptr(v_pages), _ptr(block_table), _stream(stream))
    _check(rc, "kv_append")


def kv_append_fp8(shape: Shape, k_new, v_new, range_seq, range_start, range_row0, num_ranges: int,
                  max_range_len: int, k_pages, v_pages, k_scales, v_scales, block_table, stream=None):
    rc = load().kv_append_fp8(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(range_seq), _ptr(range_start),
                              _ptr(range_row0), int(num_ranges), int(max_range_len), _ptr(k_pages), _ptr(v_pages),
                              _ptr(k_scales), _ptr(v_scales), _ptr(block_table), _stream(stream))
    _check(rc, "kv_append_fp8")


class KernelTimer:
    """Owns an sd_timer; pass it to paged_decode_attention(timer=...)."""

    def __init__(self, max_calls: int):
        self._h = load().sd_timer_create(int(max_calls))
        if not self._h:
            raise SeamDecodeError(-4, "sd_timer_create")
        self.max_calls = int(max_calls)

    def reset(self):
        load().sd_timer_reset(self._h)

    def read(self):
        """-> (split_ms[], merge_ms[]) python lists; waits for the recorded events."""
        a = (ctypes.c_float * self.max_calls)()
        b = (ctypes.c_float * self.max_calls)()
        n = int(load().sd_timer_read(self._h, a, b, self.max_calls))
        if n < 0:
            raise SeamDecodeError(n, "sd_timer_read")
        return list(a[:n]), list(b[:n])

    def close(self):
        if self._h:
            load().sd_timer_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def paged_decode_attention(shape: Shape, q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens,
                           scale: float, out, workspace, workspace_nbytes: int, stream=None,
                           timer: Optional[KernelTimer] = None):
    L = load()
    if timer is None:
        rc = L.paged_decode_attention(ctypes.byref(shape), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(k_scales),
                                      _ptr(v_scales), _ptr(block_table), _ptr(context_lens), float(scale),
                                      _ptr(out), _ptr(workspace), int(workspace_nbytes), _stream(stream))
    else:
        rc = L.paged_decode_attention_timed(ctypes.byref(shape), _ptr(q), _ptr(k_pages), _ptr(v_pages),
                                            _ptr(k_scales), _ptr(v_scales), _ptr(block_table), _ptr(context_lens),
                                            float(scale), _ptr(out), _ptr(workspace), int(workspace_nbytes),
                                            _stream(stream), timer._h)
    _check(rc, "paged_decode_attention")


def paged_decode_attention_append(shape: Shape, q, k_new, v_new, k_pages, v_pages, block_table, context_lens,
                                  scale: float, out, workspace, workspace_nbytes: int, stream=None,
                                  timer: Optional[KernelTimer] = None):
    rc = load().paged_decode_attention_append(ctypes.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_pages),
                                              _ptr(v_pages), _ptr(block_table), _ptr(context_lens), float(scale),
                                              _ptr(out), _ptr(workspace), int(workspace_nbytes), _stream(stream),
                                              timer._h if timer is not None else None)
    _check(rc, "paged_decode_attention_append")


def paged_decode_attention_static(shape: Shape, q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens,
                                  scale: float, out, stream=None):
    rc = load().paged_decode_attention_static(ctypes.byref(shape), _ptr(q), _ptr(k_pages), _ptr(v_pages),
                                              _ptr(k_scales), _ptr(v_scales), _ptr(block_table), _ptr(context_lens),
                                              float(scale), _ptr(out), _stream(stream))
    _check(rc, "paged_decode_attention_static")


def paged_decode_attention_prefix(shape: Shape, q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens,
                                  group_start, shared_len, num_groups: int, max_group_size: int,
                                  max_shared_len: int, scale: float, out, workspace, workspace_nbytes: int,
                                  stream=None, timer: Optional[KernelTimer] = None):
    rc = load().paged_decode_attention_prefix(
        ctypes.byref(shape), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(k_scales), _ptr(v_scales), _ptr(block_table),
        _ptr(context_lens), _ptr(group_start), _ptr(shared_len), int(num_groups), int(max_group_size),
        int(max_shared_len), float(scale), _ptr(out), _ptr(workspace), int(workspace_nbytes), _stream(stream),
        timer._h if timer is not None else None)
    _check(rc, "paged_decode_attention_prefix")


def kv_copy_pages(shape: Shape, src_pages, dst_pages, num_copies: int, k_pages, v_pages, k_scales=None, v_scales=None,
                  stream=None):
    rc = load().kv_copy_pages(ctypes.byref(shape), _ptr(src_pages), _ptr(dst_pages), int(num_copies), _ptr(k_pages),
                              _ptr(v_pages), _ptr(k_scales), _ptr(v_scales), _stream(stream))
    _check(rc, "kv_copy_pages")


def paged_prefill_attention(shape: Shape, q, q_start, total_q: int, max_q_len: int, k_pages, v_pages, k_scales,
                            v_scales, block_table, context_lens, scale: float, out, stream=None,
                            timer: Optional[KernelTimer] = None):
    rc = load().paged_prefill_attention(
        ctypes.byref(shape), _ptr(q), _ptr(q_start), int(total_q), int(max_q_len), _ptr(k_pages), _ptr(v_pages),
        _ptr(k_scales), _ptr(v_scales), _ptr(block_table), _ptr(context_lens), float(scale), _ptr(out),
        _stream(stream), timer._h if timer is not None else None)
    _check(rc, "paged_prefill_attention")


def validate_tables(shape: Shape, block_table, context_lens, report, stream=None):
    rc = load().sd_validate_tables(ctypes.byref(shape), _ptr(block_table), _ptr(context_lens), _ptr(report),
                                   _stream(stream))
    _check(rc, "sd_validate_tables")


def validate_groups(shape: Shape, block_table, context_lens, group_start, shared_len, num_groups: int,
                    max_group_size: int, max_shared_len: int, report, stream=None):
    rc = load().sd_validate_groups(ctypes.byref(shape), _ptr(block_table), _ptr(context_lens), _ptr(group_start),
                                   _ptr(shared_len), int(num_groups), int(max_group_size), int(max_shared_len),
                                   _ptr(report), _stream(stream))
    _check(rc, "sd_validate_groups")


def probe_read(shape: Shape, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, sink, stream=None):
    rc = load().sd_probe_read(ctypes.byref(shape), _ptr(k_pages), _ptr(v_pages), _ptr(k_scales), _ptr(v_scales),
                              _ptr(block_table), _ptr(context_lens), _ptr(sink), _stream(stream))
    _check(rc, "sd_probe_read")


def range_parts(first_tile: int, end_tile: int, line_tiles: int, tiles_per_range: int):
    """sd_range_parts: the ranges that still hold a part of the sequence occupying tiles [first_tile, end_tile)."""
    cap = max(1, (line_tiles + tiles_per_range - 1) // max(1, tiles_per_range))
    buf = (ctypes.c_int * cap)()
    n = load().sd_range_parts(first_tile, end_tile, line_tiles, tiles_per_range, buf, cap)
    _check(min(n, 0), "sd_range_parts")
    return list(buf[:n])


def probe_sink_words(shape: Shape) -> int:
    return int(load().sd_probe_sink_words(ctypes.byref(shape)))

"""ctypes loader for the CPU oracle (oracle.c).

TEST INFRASTRUCTURE ONLY.  Import this from tests, from the smoke check and
from the benchmark's CPU-baseline leg; the product package never does.
Arguments are plain numpy arrays in the layout the workload generator
documents; nothing here does arithmetic.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_SRC = [os.path.join(_HERE, "oracle.c"), os.path.join(_HERE, "oracle_attention_impl.h")]
_lib = None

KV_CODE = {"bf16": 0, "fp8": 1}


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (OpenMP) if the library is missing or stale."""
    stale = force or not os.path.exists(_SO) or any(os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _SO, _SRC[0], "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_SO)
        L.oracle_bf16_to_float.restype = ctypes.c_float
        L.oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
        L.oracle_e4m3fn_to_float.restype = ctypes.c_float
        L.oracle_e4m3fn_to_float.argtypes = [ctypes.c_uint8]
        L.oracle_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    assert a.dtype == dtype, (a.dtype, dtype)
    return a


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def e4m3fn_to_float(code: int) -> float:
    return float(lib().oracle_e4m3fn_to_float(int(code)))


def bf16_to_float(bits: int) -> float:
    return float(lib().oracle_bf16_to_float(int(bits)))


def _common(q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, kv_dtype):
    kvd = np.uint8 if kv_dtype == "fp8" else np.uint16
    q = _c(q, np.uint16)
    k_pages, v_pages = _c(k_pages, kvd), _c(v_pages, kvd)
    k_scales, v_scales = _c(k_scales, np.float32), _c(v_scales, np.float32)
    block_table, context_lens = _c(block_table, np.int32), _c(context_lens, np.int32)
    if kv_dtype == "fp8":
        assert k_scales is not None and v_scales is not None
    B, Hq, d = q.shape
    Hkv = k_pages.shape[1]
    assert k_pages.shape[2] == 16 and k_pages.shape[3] == d and v_pages.shape == k_pages.shape
    assert block_table.shape[0] == B and context_lens.shape == (B,)
    return q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, B, Hq, Hkv, d


def attend_rows(q, k_pages, v_pages, block_table, context_lens, scale, rows_bh,
                k_scales=None, v_scales=None, kv_dtype="bf16", precision="f64"):
    """Attention output for the listed (b, h) rows -> [n_rows][d]."""
    q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, B, Hq, Hkv, d = _common(
        q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, kv_dtype)
    rows = np.ascontiguousarray(np.asarray(rows_bh, dtype=np.int32).reshape(-1, 2))
    real = np.float64 if precision == "f64" else np.float32
    out = np.zeros((rows.shape[0], d), dtype=real)
    fn = getattr(lib(), f"oracle_attend_rows_{precision}")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(block_table.shape[1]),
            ctypes.c_int(KV_CODE[kv_dtype]), _p(q), _p(k_pages), _p(v_pages), _p(k_scales), _p(v_scales),
            _p(block_table), _p(context_lens), ctypes.c_float(scale), _p(rows), ctypes.c_int(rows.shape[0]),
            _p(out))
    if rc:
        raise MemoryError("oracle_attend_rows failed")
    return out


def paged_decode_attention(q, k_pages, v_pages, block_table, context_lens, scale,
                           k_scales=None, v_scales=None, kv_dtype="bf16", precision="f64"):
    """Attention output for every (b, h) -> [B][Hq][d]."""
    q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, B, Hq, Hkv, d = _common(
        q, k_pages, v_pages, k_scales, v_scales, block_table, context_lens, kv_dtype)
    real = np.float64 if precision == "f64" else np.float32
    out = np.zeros((B, Hq, d), dtype=real)
    fn = getattr(lib(), f"oracle_paged_decode_attention_{precision}")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d),
            ctypes.c_int(block_table.shape[1]), ctypes.c_int(KV_CODE[kv_dtype]), _p(q), _p(k_pages),
            _p(v_pages), _p(k_scales), _p(v_scales), _p(block_table), _p(context_lens),
            ctypes.c_float(scale), _p(out))
    if rc:
        raise MemoryError("oracle_paged_decode_attention failed")
    return out


def partial(q, k_pages, v_pages, block_table, scale, b, h, t0, t1,
            k_scales=None, v_scales=None, kv_dtype="bf16", precision="f64"):
    """(m, l, acc[d]) of row (b, h) over tokens [t0, t1)."""
    kvd = np.uint8 if kv_dtype == "fp8" else np.uint16
    q, k_pages, v_pages = _c(q, np.uint16), _c(k_pages, kvd), _c(v_pages, kvd)
    k_scales, v_scales = _c(k_scales, np.float32), _c(v_scales, np.float32)
    block_table = _c(block_table, np.int32)
    _, Hq, d = q.shape
    Hkv = k_pages.shape[1]
    real, creal = (np.float64, ctypes.c_double) if precision == "f64" else (np.float32, ctypes.c_float)
    m, l = creal(0), creal(0)
    acc = np.zeros(d, dtype=real)
    fn = getattr(lib(), f"oracle_partial_{precision}")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(block_table.shape[1]),
            ctypes.c_int(KV_CODE[kv_dtype]), _p(q), _p(k_pages), _p(v_pages), _p(k_scales), _p(v_scales),
            _p(block_table), ctypes.c_float(scale), ctypes.c_int(b), ctypes.c_int(h), ctypes.c_int(t0),
            ctypes.c_int(t1), ctypes.byref(m), ctypes.byref(l), _p(acc))
    if rc:
        raise MemoryError("oracle_partial failed")
    return m.value, l.value, acc


def combine(m, l, acc, precision="f64"):
    """Merge partial results of one row: m[n], l[n], acc[n][d] -> out[d]."""
    real = np.float64 if precision == "f64" else np.float32
    m = np.ascontiguousarray(m, dtype=real)
    l = np.ascontiguousarray(l, dtype=real)
    acc = np.ascontiguousarray(acc, dtype=real)
    n, d = acc.shape
    out = np.zeros(d, dtype=real)
    fn = getattr(lib(), f"oracle_combine_{precision}")
    fn.restype = None
    fn(ctypes.c_int(n), ctypes.c_int(d), _p(m), _p(l), _p(acc), _p(out))
    return out


def kv_append(k_new, v_new, seq_ids, positions, k_pages, v_pages, block_table):
    """In-place append of rows [T][Hkv][d] into the pools (numpy arrays)."""
    assert k_pages.flags.c_contiguous and v_pages.flags.c_contiguous and k_pages.flags.writeable
    k_new, v_new = np.ascontiguousarray(k_new), np.ascontiguousarray(v_new)
    assert k_new.dtype == k_pages.dtype and v_new.dtype == v_pages.dtype
    seq_ids, positions = _c(seq_ids, np.int32), _c(positions, np.int32)
    block_table = _c(block_table, np.int32)
    T, Hkv, d = k_new.shape
    assert k_pages.shape[1] == Hkv and k_pages.shape[3] == d
    fn = lib().oracle_kv_append
    fn.restype = None
    fn(ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(block_table.shape[1]),
       ctypes.c_int(k_pages.dtype.itemsize), _p(k_new), _p(v_new), _p(seq_ids), _p(positions),
       ctypes.c_int(T), _p(k_pages), _p(v_pages), _p(block_table))


def kv_copy_pages(src_pages, dst_pages, k_pages, v_pages, k_scales=None, v_scales=None):
    """In-place copy of whole pages src -> dst (K, V, and the scales of fp8 pools)."""
    assert k_pages.flags.c_contiguous and v_pages.flags.c_contiguous and k_pages.flags.writeable
    src_pages, dst_pages = _c(src_pages, np.int32), _c(dst_pages, np.int32)
    assert len(src_pages) == len(dst_pages)
    num_pages, Hkv, _, d = k_pages.shape
    fn = lib().oracle_kv_copy_pages
    fn.restype = None
    fn(ctypes.c_int(num_pages), ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(k_pages.dtype.itemsize),
       _p(src_pages), _p(dst_pages), ctypes.c_int(len(src_pages)), _p(k_pages), _p(v_pages),
       _p(k_scales) if k_scales is not None else None, _p(v_scales) if v_scales is not None else None)


def float_to_e4m3fn(y: float) -> int:
    f = lib().oracle_float_to_e4m3fn
    f.restype = ctypes.c_uint8
    f.argtypes = [ctypes.c_float]
    return int(f(float(y)))


def kv_append_fp8(k_new, v_new, range_seq, range_start, range_row0, k_pages, v_pages, k_scales, v_scales, block_table):
    """In-place quantising append of row ranges (bf16 rows [T][Hkv][d]) into fp8 pools and their scales."""
    k_new, v_new = _c(k_new, np.uint16), _c(v_new, np.uint16)
    range_seq, range_start, range_row0 = _c(range_seq, np.int32), _c(range_start, np.int32), _c(range_row0, np.int32)
    block_table = _c(block_table, np.int32)
    for a, t in ((k_pages, np.uint8), (v_pages, np.uint8), (k_scales, np.float32), (v_scales, np.float32)):
        assert a.dtype == t and a.flags.c_contiguous and a.flags.writeable
    T, Hkv, d = k_new.shape
    assert range_row0.shape[0] == range_seq.shape[0] + 1 and int(range_row0[-1]) <= T
    fn = lib().oracle_kv_append_fp8
    fn.restype = None
    fn(ctypes.c_int(Hkv), ctypes.c_int(d), ctypes.c_int(block_table.shape[1]), _p(k_new), _p(v_new), _p(range_seq),
       _p(range_start), _p(range_row0), ctypes.c_int(range_seq.shape[0]), _p(k_pages), _p(v_pages), _p(k_scales),
       _p(v_scales), _p(block_table))


def paged_prefill_attention(q, q_start, k_pages, v_pages, block_table, context_lens, scale,
                            k_scales=None, v_scales=None, kv_dtype="bf16", precision="f64"):
    """Causal attention of several query rows per sequence: q [rows][Hq][d], q_start [B+1] -> [rows][Hq][d]."""
    kvd = np.uint8 if kv_dtype == "fp8" else np.uint16
    q, k_pages, v_pages = _c(q, np.uint16), _c(k_pages, kvd), _c(v_pages, kvd)
    k_scales, v_scales = _c(k_scales, np.float32), _c(v_scales, np.float32)
    q_start, block_table, context_lens = _c(q_start, np.int32), _c(block_table, np.int32), _c(context_lens, np.int32)
    rows, Hq, d = q.shape
    B = context_lens.shape[0]
    assert q_start.shape == (B + 1,) and int(q_start[-1]) == rows
    real = np.float64 if precision == "f64" else np.float32
    out = np.zeros((rows, Hq, d), dtype=real)
    fn = getattr(lib(), f"oracle_paged_prefill_attention_{precision}")
    fn.restype = ctypes.c_int
    rc = fn(ctypes.c_int(B), ctypes.c_int(Hq), ctypes.c_int(k_pages.shape[1]), ctypes.c_int(d),
            ctypes.c_int(block_table.shape[1]), ctypes.c_int(KV_CODE[kv_dtype]), _p(q), _p(q_start), _p(k_pages),
            _p(v_pages), _p(k_scales), _p(v_scales), _p(block_table), _p(context_lens), ctypes.c_float(scale), _p(out))
    if rc:
        raise MemoryError("oracle_paged_prefill_attention failed")
    return out

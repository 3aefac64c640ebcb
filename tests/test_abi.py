"""Host-side checks of the C ABI: run without a GPU (no kernel is launched)."""
import ctypes
import os
import re

import pytest

import paper_2508_11553_amd as sd
from paper_2508_11553_amd import build as sd_build

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "seamdecode.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(sd.lib_path()):
        sd_build.build()
    return sd.load()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\(", src)
    return sorted({n for n in names if n not in ("defined",)})


def good_shape(**over):
    f = dict(batch=4, num_q_heads=8, num_kv_heads=2, head_dim=64, page_size=16, num_pages=100,
             max_blocks_per_seq=32, kv_dtype=sd.SD_BF16, max_context_len=512, chunk_tokens=0)
    f.update(over)
    return sd.Shape(**f)


def test_library_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"kv_append", "paged_decode_attention", "sd_workspace_bytes", "sd_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in seamdecode.h but not exported"


def test_version_and_error_strings(lib):
    assert sd.version() >= 100
    seen = {sd.strerror(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and "unknown" in sd.strerror(-99)


def test_shape_struct_matches_header():
    src = open(HEADER).read()
    body = re.search(r"typedef struct \{(.*?)\} sd_shape;", src, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"int32_t\s+(\w+);", body)
    assert fields == [f[0] for f in sd.Shape._fields_]
    assert ctypes.sizeof(sd.Shape) == 4 * len(fields)


def test_workspace_size_is_positive_and_monotone(lib):
    a = sd.workspace_bytes(good_shape())
    b = sd.workspace_bytes(good_shape(max_context_len=512, max_blocks_per_seq=64, batch=8))
    assert 0 < a <= b   # the one-launch path's scratch depends on the machine's size, not on the batch
    c = sd.workspace_bytes(good_shape(head_dim=128))
    assert c > a
    # one chunk's worth of (m, l, acc) per row at least
    assert a >= 4 * 8 * (64 + 2) * 4
    assert sd.workspace_bytes(good_shape(chunk_tokens=128)) >= a
    # two partial slots per wave of the largest grid (512 workgroups), 4 query heads each
    assert a >= 2 * 4 * 512 * 4 * (64 + 2) * 4


@pytest.mark.parametrize("over,code", [
    (dict(page_size=32), -1),
    (dict(num_q_heads=7), -1),
    (dict(head_dim=96), -2),
    (dict(num_q_heads=130, num_kv_heads=2), -2),   # 65 query heads per KV head: more than 4 blocks of 16
    (dict(kv_dtype=7), -1),
    (dict(max_context_len=513), -1),
    (dict(chunk_tokens=100), -1),
    (dict(batch=-1), -1),
])
def test_bad_shapes_are_rejected_on_the_host(lib, over, code):
    s = good_shape(**over)
    assert lib.sd_chunk_tokens(ctypes.byref(s)) == code
    assert sd.workspace_bytes(s) == 0
    rc = lib.paged_decode_attention(ctypes.byref(s), 16, 16, 16, None, None, 16, 16, 1.0, 16, 16, 1 << 30, None)
    assert rc == code


def test_null_and_misaligned_pointers_are_rejected_before_any_launch(lib):
    s = good_shape()
    ws = sd.workspace_bytes(s)
    args = [16, 32, 48, None, None, 64, 80, 1.0, 96, 112, ws, None]
    for i in (0, 1, 2, 5, 6, 8, 9):
        bad = list(args); bad[i] = None
        assert lib.paged_decode_attention(ctypes.byref(s), *bad) == -1
        bad[i] = 24  # 8-byte aligned only
        assert lib.paged_decode_attention(ctypes.byref(s), *bad) == -1
    short = list(args); short[10] = ws - 1
    assert lib.paged_decode_attention(ctypes.byref(s), *short) == -3
    s8 = good_shape(kv_dtype=sd.SD_FP8_E4M3, head_dim=128)
    args8 = list(args); args8[10] = sd.workspace_bytes(s8)
    assert lib.paged_decode_attention(ctypes.byref(s8), *args8) == -1  # fp8 needs scales
    assert lib.sd_chunk_tokens(ctypes.byref(good_shape(kv_dtype=sd.SD_FP8_E4M3))) > 0    # fp8 with d=64
    assert lib.kv_append(ctypes.byref(s), None, 16, 16, 16, 3, 16, 16, 16, None) == -1
    assert lib.kv_append(ctypes.byref(s), 16, 16, 16, 16, -1, 16, 16, 16, None) == -1
    assert lib.kv_append(ctypes.byref(s8), 16, 16, 16, 16, 3, 16, 16, 16, None) == -2


def test_prefill_arguments_are_checked_on_the_host(lib):
    s = good_shape()
    args = [16, 32, 8, 8, 48, 64, None, None, 80, 96, 1.0, 112, None, None]
    for i in (0, 1, 4, 5, 8, 9, 11):
        bad = list(args); bad[i] = None
        assert lib.paged_prefill_attention(ctypes.byref(s), *bad) == -1
        bad[i] = 24
        assert lib.paged_prefill_attention(ctypes.byref(s), *bad) == -1
    neg = list(args); neg[2] = -1
    assert lib.paged_prefill_attention(ctypes.byref(s), *neg) == -1
    none = list(args); none[2] = 0
    assert lib.paged_prefill_attention(ctypes.byref(s), *none) == 0   # no query rows: nothing to do
    s8 = good_shape(kv_dtype=sd.SD_FP8_E4M3, head_dim=128)
    assert lib.paged_prefill_attention(ctypes.byref(s8), *args) == -1  # fp8 needs scales


def test_copy_pages_arguments_are_checked_on_the_host(lib):
    s = good_shape()
    assert lib.kv_copy_pages(ctypes.byref(s), None, None, 0, None, None, None, None, None) == 0
    assert lib.kv_copy_pages(ctypes.byref(s), 16, 32, -1, 48, 64, None, None, None) == -1
    for i in range(2):
        for j in (0, 1, 3, 4):
            args = [16, 32, 2, 48, 64, None, None, None]
            args[j] = (None, 24)[i]
            assert lib.kv_copy_pages(ctypes.byref(s), *args) == -1
    s8 = good_shape(kv_dtype=sd.SD_FP8_E4M3, head_dim=128)
    assert lib.kv_copy_pages(ctypes.byref(s8), 16, 32, 2, 48, 64, None, None, None) == -1  # fp8 pools come with scales


def test_chunk_for_batch_is_a_bounded_monotone_multiple_of_128(lib):
    lib.sd_chunk_for_batch.argtypes = [ctypes.c_void_p, ctypes.c_int64]
    s = good_shape(batch=64, max_blocks_per_seq=512, max_context_len=8192)
    prev = 0
    for total in (0, 1000, 10_000, 100_000, 300_000, 1_000_000, 10**9):
        c = lib.sd_chunk_for_batch(ctypes.byref(s), total)
        assert c % 128 == 0 and 128 <= c <= 8192 and c >= prev
        prev = c
    assert prev == 8192                                   # a huge batch: the cap, which is also the longest sequence
    short = good_shape(batch=4096, max_blocks_per_seq=64, max_context_len=1000)
    assert lib.sd_chunk_for_batch(ctypes.byref(short), 4096 * 800) == 1024   # covers every sequence: one chunk each
    assert lib.sd_chunk_for_batch(ctypes.byref(s), -1) == -1
    assert lib.sd_chunk_for_batch(None, 5) == -1


def test_empty_calls_are_noops(lib):
    s = good_shape(batch=0)
    assert lib.paged_decode_attention(ctypes.byref(s), None, None, None, None, None, None, None, 1.0, None, None, 0, None) == 0
    assert lib.kv_append(ctypes.byref(good_shape()), None, None, None, None, 0, None, None, None, None) == 0


def test_shapes_beyond_the_scratch_array_are_refused(lib):
    """Rejected on the host before any HIP call; nothing is enqueued."""
    s = sd.Shape(batch=8192, num_q_heads=64, num_kv_heads=8, head_dim=128, page_size=16, num_pages=16,
                 max_blocks_per_seq=512, kv_dtype=sd.SD_BF16, max_context_len=8192, chunk_tokens=1024)
    assert sd.workspace_bytes(s) > 48 << 20
    rc = sd.load().paged_decode_attention_static(ctypes.byref(s), 16, 16, 16, None, None, 16, 16, 1.0, 16, None)
    assert rc == -3


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2508_11553_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        binding.load()

"""libseamdecode: paged decode attention for MI355X (gfx950).

Thin ctypes binding over the C ABI in include/seamdecode.h.  Every step of the
decode path runs in the HIP kernels of libseamdecode.so; Python only marshals
pointers.  torch supplies device memory and streams.  There is no CPU
fallback: if the shared library is missing, loading raises.
"""
from .binding import (  # noqa: F401
    SD_BF16,
    SD_FP8_E4M3,
    SeamDecodeError,
    Shape,
    KernelTimer,
    chunk_for_batch,
    chunk_tokens,
    kv_append,
    kv_append_fp8,
    kv_copy_pages,
    lib_path,
    load,
    paged_decode_attention,
    paged_decode_attention_append,
    paged_decode_attention_prefix,
    paged_decode_attention_static,
    paged_prefill_attention,
    probe_read,
    range_parts,
    strerror,
    validate_groups,
    validate_tables,
    version,
    workspace_bytes,
)

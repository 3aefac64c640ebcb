"""Seeded synthetic inputs for paged decode attention.

This package only draws random numbers, rounds them to the storage formats
(bf16, OCP fp8 e4m3fn) and lays them out in a paged KV pool.  It contains no
attention arithmetic and is the one module that both the CPU oracle's tests
and the HIP path's tests read their inputs from.
"""
from .formats import (  # noqa: F401
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    f32_to_e4m3fn_bits,
    BF16_NAN_BITS,
    E4M3FN_NAN_BITS,
    E4M3FN_MAX,
)
from .gen import (  # noqa: F401
    Workload,
    CONFIG_NAMES,
    make_config,
    config_lengths,
    make_custom,
    build_paged,
)

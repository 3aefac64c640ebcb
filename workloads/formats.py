"""Storage-format encoders used when drawing inputs.

bf16 is the upper half of an IEEE binary32 word; OCP fp8 e4m3fn is
1 sign / 4 exponent (bias 7) / 3 mantissa bits with no infinities, one NaN
code per sign (0x7f / 0xff) and a largest finite magnitude of 448.
Encoders only: decoding for checking purposes lives with whoever checks.
"""
import numpy as np

BF16_NAN_BITS = np.uint16(0x7FC0)
E4M3FN_NAN_BITS = np.uint8(0x7F)
E4M3FN_MAX = 448.0


def f32_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    out = (r >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = BF16_NAN_BITS
    return out


def bf16_bits_to_f32(b):
    """uint16 bf16 bit patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_e4m3fn_bits(x):
    """float32 array -> uint8 e4m3fn codes: round-to-nearest-even, saturating
    at +-448, never producing a NaN code for finite input."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    sign = (x.view(np.uint32) >> np.uint32(24)).astype(np.uint8) & np.uint8(0x80)
    a = np.minimum(np.abs(x), np.float32(E4M3FN_MAX))
    # normal range (>= 2^-6): keep 3 mantissa bits of the binary32 word, RNE
    u = a.view(np.uint32)
    r = u + (np.uint32(0x7FFFF) + ((u >> np.uint32(20)) & np.uint32(1)))
    normal = ((r >> np.uint32(20)).astype(np.int32) - (120 << 3))
    # subnormal range (< 2^-6): multiples of 2^-9; rint is round-half-even
    sub = np.rint(a * np.float32(512.0)).astype(np.int32)
    code = np.where(a < np.float32(2.0 ** -6), sub, normal)
    code = np.clip(code, 0, 0x7E).astype(np.uint8)
    return code | sign

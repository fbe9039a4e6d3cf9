"""bfloat16 storage helpers (numpy has no bf16 dtype; buffers are uint16 bit patterns).

bf16 is the upper half of an IEEE-754 binary32, so decoding is exact and encoding is
one round-to-nearest-even step on the dropped 16 bits.
"""
import numpy as np


def f32_to_bf16_bits(x):
    """Round float32 values to bf16 (nearest, ties to even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(bits):
    """Exact decode of bf16 bit patterns to float32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(bits):
    """Exact decode of bf16 bit patterns to float64."""
    return bf16_bits_to_f32(bits).astype(np.float64)

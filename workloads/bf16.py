"""bfloat16 <-> float32 conversion on the host (numpy has no bfloat16 type).

bfloat16 is the upper 16 bits of an IEEE-754 binary32 value. Rounding a
binary32 to bfloat16 uses round-to-nearest, ties-to-even on the dropped 16
bits. Only finite inputs are produced by the generators, so NaN handling is a
plain quieting of the payload.
"""
import numpy as np


def f32_to_bf16_bits(x):
    """Round float32 (or anything castable) to bfloat16; return the uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    bits = (rounded >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        bits = np.where(nan, np.uint16(0x7FC0), bits)
    return bits


def bf16_bits_to_f32(bits):
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x):
    """Values of x after one rounding to bfloat16, returned as float32."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))

"""bfloat16 storage helpers (format conversion only: round-to-nearest-even)."""
import numpy as np


def f32_to_bf16_bits(a):
    """float32 array -> uint16 array of bfloat16 bit patterns (RNE, NaN kept quiet)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    with np.errstate(over="ignore"):
        rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out.reshape(a.shape)


def bf16_bits_to_f32(b):
    """uint16 bfloat16 bit patterns -> float32 array (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def round_to_bf16(a):
    """float32 array -> float32 array holding only bfloat16-representable values."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))

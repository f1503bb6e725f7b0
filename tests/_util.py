"""Helpers shared by the test modules (format conversion and error metrics only)."""
import numpy as np
import torch

from et_inputs import bf16_bits_to_f32, f32_to_bf16_bits


def bits_to_dev(bits, device="cuda:0"):
    """uint16 bf16 bit patterns (numpy) -> torch.bfloat16 tensor on the device."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.view(torch.bfloat16).to(device)


def dev_to_bits(t):
    """torch.bfloat16 tensor -> uint16 bit patterns (numpy)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def dev_to_f64(t):
    if t.dtype == torch.bfloat16:
        return bf16_bits_to_f32(dev_to_bits(t)).astype(np.float64)
    return t.detach().cpu().numpy().astype(np.float64)


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def bf16_ulp_distance(bits_a, bits_b):
    """Distance in bf16 steps between two arrays of bit patterns (same-sign finite values)."""
    def key(b):
        b = b.astype(np.int32)
        return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)
    return np.abs(key(np.asarray(bits_a)) - key(np.asarray(bits_b)))


def f64_to_bits(a):
    return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))

"""Input-side helpers for the tests: bf16 <-> fp32 bit handling in numpy.

Nothing of the method's arithmetic lives here (no FP8, no scales, no sums).
"""
import numpy as np


def f32_to_bf16_bits(a):
    """Round-to-nearest-even fp32 -> bf16 storage (uint16).  Finite inputs."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = u + 0x7FFF + lsb
    return (u >> 16).astype(np.uint16).reshape(a.shape)


def bf16_bits_to_f64(h):
    h = np.ascontiguousarray(h, dtype=np.uint16)
    return (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64).reshape(h.shape)


def all_bf16_patterns():
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def finite_mask(h):
    return (h & 0x7F80) != 0x7F80

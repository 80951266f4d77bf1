"""Helpers shared by the GPU parity tests (no method arithmetic)."""
import numpy as np


def rel_err(got, ref):
    """Per-tensor relative error: max|got - ref| / max|ref| (elementwise relative
    error is meaningless at near-zero gradient entries)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def to_bf16_bits(a):
    """float32 -> bf16 bit pattern (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return (((u + 0x7FFF + ((u >> 16) & 1)) >> 16) & 0xFFFF).astype(np.uint16)


def from_bf16_bits(b):
    return (b.astype(np.uint32) << 16).view(np.float32)

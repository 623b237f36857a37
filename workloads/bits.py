"""Storage-format helpers: bf16 bit patterns <-> fp32 / fp64 (exact widenings,
one round-to-nearest-even narrowing).  No arithmetic of the layer lives here."""
import numpy as np


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (round-to-nearest-even) and return the 16-bit
    patterns as uint16.  Inputs are finite by construction (normal draws)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor (uint16 = bf16 bits, or float32) to fp64."""
    if a.dtype == np.uint16:
        return f32_from_bf16_bits(a).astype(np.float64)
    return np.asarray(a, dtype=np.float64)

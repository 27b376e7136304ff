"""Storage-dtype helpers for the oracle (test infrastructure only).

The method's state lives in fp32 or bf16 buffers; the oracle computes in fp64 on the
values those buffers hold.  bf16 is carried as uint16 bit patterns because NumPy has
no bf16 type.  Rounding is IEEE round-to-nearest-even, done directly from fp64 (one
rounding).  bf16 subnormals are outside every workload's value range and are flushed
to signed zero here.
"""
import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Decode bf16 bit patterns (uint16) exactly to float64."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 to the nearest bf16 (ties to even); returns uint16 bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    u = x.view(np.uint64)
    # bf16 keeps 7 explicit mantissa bits; fp64 has 52 -> drop 45 with RNE.
    drop = np.uint64(45)
    lsb = (u >> drop) & np.uint64(1)
    rounded = (u + np.uint64((1 << 44) - 1) + lsb) >> drop << drop
    y = rounded.view(np.float64)
    tiny = np.abs(y) < 2.0 ** -126
    y = np.where(tiny, np.copysign(0.0, x), y)
    y32 = y.astype(np.float32)            # exact: y has an 8-bit significand
    return (y32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Value (as float64) that a buffer of `dtype` ("f32" | "bf16") holds after storing x."""
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f64(f64_to_bf16_bits(x))
    raise ValueError(dtype)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers at |x| (normal range)."""
    ax = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)

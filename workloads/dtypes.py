"""Storage-type helpers for the synthetic inputs (NumPy has no bfloat16).

A tensor in a 16-bit type is carried as its uint16 bit patterns; the float64
array of the values those bits denote is what the CPU oracle is given, and the
bits are what is copied into device memory.
"""
from __future__ import annotations

import numpy as np

F32, BF16, F16 = 0, 1, 2
NAMES = {F32: "f32", BF16: "bf16", F16: "f16"}
ITEMSIZE = {F32: 4, BF16: 2, F16: 2}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def quantize(values: np.ndarray, dtype: int):
    """Round float64 `values` to `dtype`.

    Returns (storage, exact) where `storage` is what goes to the device
    (float32 array, or uint16 bit patterns for the 16-bit types) and `exact`
    is the float64 array of the stored values.
    """
    v32 = np.asarray(values, dtype=np.float64).astype(np.float32)
    if dtype == F32:
        return v32, v32.astype(np.float64)
    if dtype == BF16:
        bits = f32_to_bf16_bits(v32)
        return bits, bf16_bits_to_f64(bits)
    if dtype == F16:
        h = np.asarray(values, dtype=np.float64).astype(np.float16)
        return h.view(np.uint16).copy(), h.astype(np.float64)
    raise ValueError(f"unknown dtype {dtype}")


def storage_to_f64(storage: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == F32:
        return np.asarray(storage, dtype=np.float32).astype(np.float64)
    if dtype == BF16:
        return bf16_bits_to_f64(storage)
    if dtype == F16:
        return np.ascontiguousarray(storage, dtype=np.uint16).view(np.float16).astype(np.float64)
    raise ValueError(f"unknown dtype {dtype}")

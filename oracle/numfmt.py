"""Decode stored 16/32-bit floating-point arrays to float64 (oracle side).

bfloat16 has no numpy type; it is carried as uint16 bit patterns whose value is
the float32 with those bits in its upper half (IEEE-754 binary32 truncated to
its top 16 bits).
"""
import numpy as np

F32, F16, BF16 = 0, 1, 2


def to_f64(x: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == F32:
        assert x.dtype == np.float32
        return x.astype(np.float64)
    if dtype == F16:
        assert x.dtype == np.float16
        return x.astype(np.float64)
    if dtype == BF16:
        assert x.dtype == np.uint16
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown dtype code {dtype}")


def storage_dtype(dtype: int):
    return {F32: np.float32, F16: np.float16, BF16: np.uint16}[dtype]

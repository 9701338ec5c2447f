"""Distance in units in the last place between bit patterns (test helper).

A pattern is mapped to an integer that preserves numeric order (+0 and -0 map
to the same integer), so the distance between two finite values is the number
of representable values between them.
"""
import numpy as np


def ordered_f32(x: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.int64)
    return np.where(b & 0x80000000, -(b & 0x7FFFFFFF), b)


def ordered_u16(bits: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.int64)
    return np.where(b & 0x8000, -(b & 0x7FFF), b)


def ulp_dist_f32(a, b) -> np.ndarray:
    return np.abs(ordered_f32(a) - ordered_f32(b))


def ulp_dist_u16(a, b) -> np.ndarray:
    return np.abs(ordered_u16(a) - ordered_u16(b))


def is_nan_lp(bits: np.ndarray, dtype: int) -> np.ndarray:
    """dtype 0 = bf16, 1 = fp16."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == 0:
        return ((bits & 0x7F80) == 0x7F80) & ((bits & 0x007F) != 0)
    return ((bits & 0x7C00) == 0x7C00) & ((bits & 0x03FF) != 0)


def max_ulp_report(name, a, b):
    d = ulp_dist_f32(a, b)
    mx = int(d.max()) if d.size else 0
    hist = {int(k): int((d == k).sum()) for k in np.unique(d)[:8]}
    return f"{name}: max ulp {mx}, histogram {hist}"

"""Materialisation rounding used by the oracle's bf16 precision contract."""
import numpy as np


def identity(x):
    return x


def round_bf16(x):
    """Round float64 -> float32 -> bfloat16 (round-to-nearest-even), return float64.

    bfloat16 is the upper 16 bits of an IEEE binary32; RNE adds 0x7FFF plus the
    lowest kept bit before truncating.  Going through float32 first mirrors a
    device that holds fp32 accumulators and converts them on store.
    """
    f = np.ascontiguousarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(x))


def round_f32(x):
    """Round float64 -> float32 (round-to-nearest-even), return float64."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)

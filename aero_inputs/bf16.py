"""bfloat16 / binary16 / 8-bit float storage for generated inputs (bit patterns in ``uint16`` / ``uint8`` arrays)."""
import numpy as np


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (round-to-nearest-even), return the uint16 bits.

    Inputs are finite by construction (Gaussian draws), so NaN handling is not needed.
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def f32_to_f16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to IEEE binary16 (round-to-nearest-even), return the uint16 bits."""
    return np.ascontiguousarray(x, dtype=np.float32).astype(np.float16).view(np.uint16)


def f32_to_f8e4m3_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the 8-bit float with 4 exponent and 3 mantissa bits (no infinities, largest
    finite value 448) by round-to-nearest-even; magnitudes beyond 448 go to 448.  Returns the uint8 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.arange(127)                                  # the non-negative finite patterns, ascending in value
    e, m = codes >> 3, codes & 7
    grid = np.where(e == 0, m * 2.0 ** -9, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))
    a = np.abs(x).astype(np.float64)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, 126)
    lo = np.clip(hi - 1, 0, 126)
    d_lo, d_hi = a - grid[lo], grid[hi] - a
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0)) | (lo == hi)
    code = np.where(take_hi, hi, lo).astype(np.uint8)
    code = np.where(a > 448.0, np.uint8(126), code)
    return (code | (np.signbit(x).astype(np.uint8) << np.uint8(7))).astype(np.uint8)

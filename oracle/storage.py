"""16-bit storage of feature tables, written out (test infrastructure).

A table kept in bfloat16 or IEEE half halves the bytes an aggregation gathers.  The stored value
is DEFINED as the float32 value rounded to nearest, ties to even, in the target format; the
aggregation then runs on exactly those values.  (A variant outside the paper's fp32 results: its
error is that of the rounding, not of the arithmetic.)

  bf16: the upper 16 bits of the float32 pattern after adding the rounding bias
        0x7FFF + (bit 16), NaNs kept NaN (quiet), overflow rounds to infinity as in IEEE
  fp16: IEEE binary16, with subnormals and overflow to infinity
"""
from __future__ import annotations

import numpy as np

FORMATS = {"bf16": 1, "fp16": 2}


def store(x, fmt: str) -> np.ndarray:
    """float32 array -> uint16 array of stored patterns."""
    x = np.ascontiguousarray(x, np.float32)
    if fmt == "fp16":
        with np.errstate(over="ignore"):
            return x.astype(np.float16).view(np.uint16)
    assert fmt == "bf16"
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    quiet = ((bits >> 16) | 0x0040).astype(np.uint16)          # keep sign and payload top bits, set the quiet bit
    return np.where(nan, quiet, rounded)


def load(u16, fmt: str) -> np.ndarray:
    """uint16 patterns -> the float32 values they stand for (exact)."""
    u16 = np.ascontiguousarray(u16, np.uint16)
    if fmt == "fp16":
        return u16.view(np.float16).astype(np.float32)
    assert fmt == "bf16"
    return (u16.astype(np.uint32) << 16).view(np.float32)

"""Storage-type rounding used on oracle inputs -- TEST INFRASTRUCTURE ONLY.

The paper computes in fp32 only (Section 5.3, SGEMM).  This build also takes
bf16 and fp16 operands; the oracle consumes values that were first rounded to
the operand type with round-to-nearest-even, so that a comparison against it
isolates accumulation and output rounding.

bf16 is the upper 16 bits of an IEEE binary32 (1 sign, 8 exponent, 7 fraction
bits); rounding is done on the bit pattern.  fp16 uses numpy's IEEE binary16.

Pins (tests/test_oracle_rounding.py): every one of the 65536 bf16 patterns
survives a round trip; constructed midpoints go to the even neighbour; values
just above/below a midpoint go up/down; overflow goes to infinity.
"""
from __future__ import annotations

import numpy as np


def f32_to_bf16_bits(x) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns uint16 patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    keep_lsb = (u >> 16) & 1          # parity of the part that is kept
    rounded = (u + 0x7FFF + keep_lsb) >> 16
    out = (rounded & 0xFFFF).astype(np.uint16)
    nan = np.isnan(x)
    if np.any(nan):
        # keep NaNs NaN (the increment could carry a NaN payload into the exponent)
        out = np.where(nan, ((u >> 16) | 0x0040).astype(np.uint16), out)
    return out.reshape(x.shape)


def bf16_bits_to_f32(bits) -> np.ndarray:
    """Exact widening of bf16 patterns (uint16) to fp32."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def f32_to_f16_bits(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    with np.errstate(over="ignore"):
        return x.astype(np.float16).view(np.uint16).reshape(x.shape)


def f16_bits_to_f32(bits) -> np.ndarray:
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return b.view(np.float16).astype(np.float32).reshape(b.shape)


def round_to(dtype: str, x):
    """(bits, values): storage pattern and its exact fp32 value for `dtype`.

    For "f32" the pattern is the uint32 view and the value is x itself.
    """
    if dtype == "f32":
        x = np.ascontiguousarray(x, dtype=np.float32)
        return x.view(np.uint32), x
    if dtype == "bf16":
        b = f32_to_bf16_bits(x)
        return b, bf16_bits_to_f32(b)
    if dtype == "f16":
        b = f32_to_f16_bits(x)
        return b, f16_bits_to_f32(b)
    raise ValueError(dtype)


def bits_to_f32(dtype: str, bits) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(bits, dtype=np.uint32).view(np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(bits)
    if dtype == "f16":
        return f16_bits_to_f32(bits)
    raise ValueError(dtype)

"""Error measures the parity tests gate on -- TEST INFRASTRUCTURE ONLY.

The accuracy targets are "max relative error 1e-5 (fp32) / 2e-2 (bf16, fp16)
against the fp64 result".  A strictly element-wise relative error is not a
usable gate: an output that is small only because large terms cancelled has an
absolute error set by the size of the terms, not of the result.  The gate used
here divides by max(|ref_ij|, rms(ref)) per operator; the strict element-wise,
norm-wise and backward (relative to sum_k |a||b|) figures are returned beside
it.  `order_free_bound` is the rigorous ceiling any fp32-accumulate summation
order must sit under.

Pins (tests/test_oracle_compare.py, tests/test_oracle_rounding.py): `errors`
against hand-worked gate / strict / normwise / backward figures, including a
cancellation case and the floors a mean or a maximum would give instead of the
root mean square; `order_free_bound` from both sides: fp32 accumulation of the
exact products in ascending, descending, pairwise and shuffled order passes, a
constructed sequential sum comes within 5 % of it, and a dropped product, fp16
accumulation, products rounded to bf16 and a twice-rounded result are rejected.
"""
from __future__ import annotations

import numpy as np

TOL = {"f32": 1e-5, "bf16": 2e-2, "f16": 2e-2}

# unit roundoff of the output format (round to nearest): 2^-p for p significand bits
# (fp32: 24, fp16: 11, bf16: 8 = 7 stored + 1 implicit)
_U_OUT = {"f32": 2.0 ** -24, "bf16": 2.0 ** -8, "f16": 2.0 ** -11}
# half the spacing of the output format's subnormal numbers: the absolute rounding error of an
# output below the smallest normal number (fp16: 2^-14), which u * |value| does not cover
_HALF_SUBNORMAL = {"f32": 2.0 ** -150, "bf16": 2.0 ** -134, "f16": 2.0 ** -25}


def errors(c, ref, mag=None):
    c = np.asarray(c, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(c - ref)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    floor = np.maximum(np.abs(ref), rms)
    out = {
        "gate": float(np.max(diff / np.where(floor > 0, floor, 1.0))) if ref.size else 0.0,
        "normwise": float(np.max(diff) / max(float(np.max(np.abs(ref))), 1e-300)) if ref.size else 0.0,
        "max_abs": float(np.max(diff)) if ref.size else 0.0,
    }
    with np.errstate(divide="ignore", invalid="ignore"):
        strict = np.where(np.abs(ref) > 0, diff / np.abs(ref), 0.0)
    out["strict"] = float(np.max(strict)) if ref.size else 0.0
    if mag is not None:
        mag = np.asarray(mag, dtype=np.float64)
        with np.errstate(divide="ignore", invalid="ignore"):
            bw = np.where(mag > 0, diff / mag, 0.0)
        out["backward"] = float(np.max(bw)) if ref.size else 0.0
    return out


def order_free_bound(ref, mag, K: int, dtype: str):
    """|c - ref| <= gamma*mag + max(u_out*(|ref| + gamma*mag), half the subnormal spacing) for fp32
    accumulation of K exactly representable products in any order, followed by one rounding to
    the output format (relative error u_out in the normal range, absolute error of half a
    subnormal step below it).  gamma = (K+2)*2^-24 (first-order, slightly inflated)."""
    gamma = (K + 2) * 2.0 ** -24
    ref = np.abs(np.asarray(ref, dtype=np.float64))
    mag = np.asarray(mag, dtype=np.float64)
    acc = gamma * mag
    return acc + np.maximum(_U_OUT[dtype] * (ref + acc) * 1.0000001, _HALF_SUBNORMAL[dtype]) + 1e-300

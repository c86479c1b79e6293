"""The paper's ternary quantizers, written out literally (TEST INFRASTRUCTURE ONLY).

Section 4.1: normalise by the step size, saturate, round with bankers rounding.

    weights / real-valued activations (Eq. 8, unified as Eq. 9):
        Q^w(p) = round(clip(p / alpha1, -1, 0)) + round(clip(p / alpha2, 0, 1))     in {-1, 0, +1}
    non-negative (ReLU) activations (Eq. 10, reading the misprinted parenthesis as
    clip((p - alpha1) / alpha2, 0, 1)):
        Q^a(p) = round(clip(p / alpha1, 0, 1)) + round(clip((p - alpha1) / alpha2, 0, 1))   in {0, 1, 2}

The rounding decides an integer from floating point, so it is taken in the precision
the HIP kernel works in: every operation below is a single-precision IEEE operation
(numpy float32 arithmetic, round-half-to-even).  Level index = Q^w + 1, or Q^a.

NaN.  Eq. 8-10 are defined on real numbers; a NaN is outside their domain, and the level
set {-1,0,+1} / {0,1,2} (first constraint of Section 3.3) has no member for it.  Reading:
a NaN is an invalid input in the same sense as a level index outside {0,1,2} -- it takes the
VALUE 0 (Q^w = 0, Q^a = 0) and is counted (count_invalid).  The value is assigned explicitly
below; no floating-point NaN is ever converted to an integer.
No code is shared with the HIP path (which pre-computes exact thresholds instead of
dividing).
"""
from __future__ import annotations

import numpy as np

SYM, RELU = 0, 1


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def _finite_part(p: np.ndarray):
    """(is_nan mask, p with every NaN replaced by 0.0 so that the formulas below see numbers only)."""
    nan = np.isnan(p)
    return nan, np.where(nan, np.float32(0), p).astype(np.float32)


def _values(q: np.ndarray, nan: np.ndarray) -> np.ndarray:
    """Quantizer output as int8 with the value 0 wherever the input was a NaN."""
    return np.where(nan, np.int8(0), q.astype(np.int8)).astype(np.int8)


def count_invalid(p) -> int:
    """Inputs outside the quantizers' domain (NaN)."""
    return int(np.isnan(_f32(p)).sum())


def quantize_weight(p, alpha1, alpha2) -> np.ndarray:
    """Eq. 9 in float32; returns values in {-1, 0, +1} as int8."""
    nan, p = _finite_part(_f32(p))
    a1, a2 = np.float32(alpha1), np.float32(alpha2)
    with np.errstate(over="ignore"):
        neg = np.rint(np.clip(p / a1, np.float32(-1), np.float32(0)))
        pos = np.rint(np.clip(p / a2, np.float32(0), np.float32(1)))
    return _values(neg + pos, nan)


def quantize_weight_piecewise(p, alpha1, alpha2) -> np.ndarray:
    """Eq. 8 (the two-case form) in float32."""
    nan, p = _finite_part(_f32(p))
    a1, a2 = np.float32(alpha1), np.float32(alpha2)
    with np.errstate(over="ignore"):
        neg = np.rint(np.clip(p / a1, np.float32(-1), np.float32(0)))
        pos = np.rint(np.clip(p / a2, np.float32(0), np.float32(1)))
    return _values(np.where(p < 0, neg, pos), nan)


def quantize_relu_act(p, alpha1, alpha2) -> np.ndarray:
    """Eq. 10 in float32; returns values in {0, 1, 2} as int8."""
    nan, p = _finite_part(_f32(p))
    a1, a2 = np.float32(alpha1), np.float32(alpha2)
    with np.errstate(over="ignore"):
        first = np.rint(np.clip(p / a1, np.float32(0), np.float32(1)))
        second = np.rint(np.clip((p - a1) / a2, np.float32(0), np.float32(1)))
    return _values(first + second, nan)


def levels_from_floats(p, role_is_weight: bool, act_mode: int, alpha1, alpha2) -> np.ndarray:
    """Level indices in {0,1,2} as the packer must see them (Algorithm 1, step 1)."""
    if role_is_weight or act_mode == SYM:
        return (quantize_weight(p, alpha1, alpha2) + 1).astype(np.int8)
    return quantize_relu_act(p, alpha1, alpha2)

"""Layer-chaining epilogue, composed from the oracle's pieces (TEST INFRASTRUCTURE ONLY).

Supplementary S1: batch normalisation is folded into the layer (one scale and one
bias per output channel), ReLU and the skip connection are fused, and the result is
quantized and packed as the next layer's input.  In float32, one rounding per
operation, in this order:

    f = scale[c] * float(C) ; f = f + bias[c] ; f = f + skip ; f = max(f, 0)
    level = activation quantizer of the next layer applied to f   (oracle/quantizer.py)

The paper does not say what ReLU does to a NaN; the reading taken is the IEEE 754 maximum
of two numbers, which returns the operand that is not a NaN: max(NaN, 0) = 0.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

from . import quantizer, scale_epilogue


def chain_epilogue(C: np.ndarray, scale: np.ndarray, bias: Optional[np.ndarray], skip: Optional[np.ndarray],
                   relu: bool, out_act_mode: int, alpha1: float, alpha2: float) -> Tuple[np.ndarray, np.ndarray]:
    """C: int32 NHWC conv result.  Returns (f float32 NHWC, levels int8 NHWC)."""
    f = scale_epilogue(C, scale, bias, channel_is_row=False)
    if skip is not None:
        f = (f + np.asarray(skip, dtype=np.float32)).astype(np.float32)
    if relu:
        f = np.fmax(f, np.float32(0))
    levels = quantizer.levels_from_floats(f, False, out_act_mode, alpha1, alpha2)
    return f, levels

"""Layer-chaining epilogue, composed from the oracle's pieces (TEST INFRASTRUCTURE ONLY).

Supplementary S1: batch normalisation is folded into the layer (one scale and one
bias per output channel), ReLU and the skip connection are fused, and the result is
quantized and packed as the next layer's input.  In float32, one rounding per
operation, in this order:

    f = scale[c] * float(C) ; f = f + bias[c] ; f = f + skip ; f = max(f, 0)
    level = activation quantizer of the next layer applied to f   (oracle/quantizer.py)

The paper does not say what ReLU does to a NaN.  Reading: ReLU is max(f, 0) as the deep-learning
frameworks the paper trains in define it, where a NaN operand gives a NaN (the fp32 output f shows
it to the caller); the quantizer then treats that NaN as its module documents (the value 0).
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
        f = np.maximum(f, np.float32(0))     # NaN stays NaN
    levels = quantizer.levels_from_floats(f, False, out_act_mode, alpha1, alpha2)
    return f, levels

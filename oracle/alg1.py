"""The paper's fast ternary inner product, step by step (TEST INFRASTRUCTURE ONLY).

Where ``fatnn_oracle.c`` is the plain definition, this module walks through the
method in the paper's own order and notation -- Table 1's codec, Eq. 4 (xnor),
Eq. 5 (switch), Eq. 6 (mask), Eq. 7 (TM), Eq. 3 and Algorithm 1 (pack four
values per unsigned char, accumulate popcount(TM), subtract N).  It exists so
the definition can be pinned against the method as printed, and the method
against Tables 1 and 2.  Small inputs only (pure Python loops).
"""
from __future__ import annotations

from typing import Iterable, List, Sequence

import numpy as np

# Table 1: value -> codec.  The value 0 has two spellings.
CODEC_OF_VALUE = {-1: (0b00,), 0: (0b01, 0b10), +1: (0b11,)}
AUXI_FIELD = 0b01          # auxi of Section 3.3 (Eq. 5): the fixed field with codec 01
AUXI_BYTE = 0b01010101     # the same constant replicated over the four fields of a byte


def popcount(x: int) -> int:
    return bin(x).count("1")


def decode_field(c: int) -> int:
    """Table 1: popcount(codec) = data + 1."""
    return popcount(c & 0b11) - 1


def tm(x_c: int, y_c: int, width_bits: int = 8) -> int:
    """Ternary multiplication of two packed codec words (Eq. 4-7).

    y_c is the operand that supplies the mask (the weights, end of Section 3.3).
    """
    full = (1 << width_bits) - 1
    auxi = 0
    for f in range(width_bits // 2):
        auxi |= AUXI_FIELD << (2 * f)
    xnor = ~(x_c ^ y_c) & full                                         # Eq. 4
    switch = ((y_c >> 1) & auxi) | ((y_c << 1) & ~auxi & full)         # Eq. 5
    mask = switch ^ y_c                                                # Eq. 6
    return (mask & auxi) | (~mask & full & xnor)                       # Eq. 7


def mask_of(y_c: int, width_bits: int = 8) -> int:
    full = (1 << width_bits) - 1
    auxi = 0
    for f in range(width_bits // 2):
        auxi |= AUXI_FIELD << (2 * f)
    switch = ((y_c >> 1) & auxi) | ((y_c << 1) & ~auxi & full)
    return switch ^ y_c


def pack_bytes(codecs: Sequence[int]) -> List[int]:
    """Algorithm 1, step 1: four 2-bit fields per unsigned char.

    A ragged tail is filled with the value 0 (codec 01) in both operands, so each
    filler slot adds popcount(TM) = 1 and the matching 1 is removed again by
    subtracting the padded length -- the reading taken for N not a multiple of 4.
    """
    out = []
    n = len(codecs)
    for i in range(0, n, 4):
        byte = 0
        for j in range(4):
            c = codecs[i + j] if i + j < n else 0b01
            byte |= (c & 0b11) << (2 * j)
        out.append(byte)
    return out


def inner_product_codecs(x_codecs: Sequence[int], y_codecs: Sequence[int]) -> int:
    """Algorithm 1, step 2 and Eq. 3: z = sum popcount(TM(w_hat[i], a_hat[i])) - N."""
    if len(x_codecs) != len(y_codecs):
        raise ValueError("length mismatch")
    a_hat = pack_bytes(x_codecs)
    w_hat = pack_bytes(y_codecs)
    acc = 0
    for i in range(len(w_hat)):
        acc += popcount(tm(a_hat[i], w_hat[i]))
    n_padded = 4 * len(w_hat)
    return acc - n_padded


def codec_of_level(level: int, zero_spelling: int = 0b01) -> int:
    """Level index (= popcount of the codec) -> codec, with a chosen spelling of 0."""
    if level == 0:
        return 0b00
    if level == 1:
        return zero_spelling
    if level == 2:
        return 0b11
    raise ValueError("level outside {0,1,2}")


def inner_product_levels(lw: Iterable[int], la: Iterable[int], act_mode: int = 0) -> int:
    """Ternary inner product of two level vectors through Algorithm 1.

    act_mode 1 (ReLU, activation values {0,1,2}): the kernel still sees the
    codecs of la - 1 and the fixed constant "sum of the weights" is added
    afterwards (second constraint, Section 3.3).
    """
    lw = [int(v) for v in lw]
    la = [int(v) for v in la]
    z = inner_product_codecs([codec_of_level(v) for v in la], [codec_of_level(v) for v in lw])
    if act_mode == 1:
        z += sum(v - 1 for v in lw)
    return z


def gemm_levels(Lw: np.ndarray, La: np.ndarray, act_mode: int = 0) -> np.ndarray:
    M, N = Lw.shape[0], La.shape[0]
    C = np.zeros((M, N), dtype=np.int32)
    for m in range(M):
        for n in range(N):
            C[m, n] = inner_product_levels(Lw[m], La[n], act_mode)
    return C


def inner_product_xnor_only(x_codecs: Sequence[int], y_codecs: Sequence[int]) -> int:
    """Eq. 3 with TM replaced by the plain xnor of Eq. 4, i.e. without the zero-operand fix of
    Eq. 5-7 (the ablation of Table 4).  Wrong exactly on the bold rows of Table 2."""
    if len(x_codecs) != len(y_codecs):
        raise ValueError("length mismatch")
    acc = 0
    for xc, yc in zip(x_codecs, y_codecs):
        acc += popcount(~(xc ^ yc) & 0b11)
    return acc - len(x_codecs)


def gemm_xnor_only(Lw: np.ndarray, La: np.ndarray) -> np.ndarray:
    M, N = Lw.shape[0], La.shape[0]
    C = np.zeros((M, N), dtype=np.int32)
    for m in range(M):
        yw = [codec_of_level(int(v)) for v in Lw[m]]
        for n in range(N):
            C[m, n] = inner_product_xnor_only([codec_of_level(int(v)) for v in La[n]], yw)
    return C

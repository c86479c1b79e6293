"""CPU oracle (TEST INFRASTRUCTURE ONLY).

Thin ctypes wrapper around ``fatnn_oracle.c`` -- the plain integer definition of
the ternary GEMM / convolution that the paper's fast inner product (Section 3.3,
Eq. 3) reaches exactly.  Only tests, ``__graft_entry__.smoke()`` and
``bench.py``'s ``cpu_baseline`` leg may import this package; it shares nothing
with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fatnn_oracle.c")
_LIB = os.path.join(_HERE, "libfatnn_oracle.so")

SYM, RELU = 0, 1
BASIS_TERNARY, BASIS_UNIFORM = 0, 1

_lib: Optional[ctypes.CDLL] = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32p, i8p, fp = ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p
        lib.oracle_ternary_gemm.argtypes = [i8p, i8p, i64, i64, i64, ctypes.c_int, i32p]
        lib.oracle_ternary_conv2d.argtypes = [i8p, i8p] + [i64] * 9 + [ctypes.c_int, i32p]
        lib.oracle_twobit_gemm.argtypes = [i8p, i8p, i64, i64, i64, ctypes.c_int, i32p]
        lib.oracle_binary_gemm.argtypes = [i8p, i8p, i64, i64, i64, i32p]
        lib.oracle_scale_epilogue.argtypes = [i32p, i64, i64, ctypes.c_int, fp, fp, fp]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
        lib.oracle_set_num_threads.restype = None
        _lib = lib
    return _lib


def _i8(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.int8:
        raise TypeError("levels must be int8")
    return a


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the C loops use from now on (timing only; results do not depend on it)."""
    _load().oracle_set_num_threads(int(n))


def ternary_gemm(Lw: np.ndarray, La: np.ndarray, act_mode: int = SYM) -> np.ndarray:
    """C[m][n] = sum_k (Lw[m][k]-1) * val(La[n][k]);  Lw [M][K], La [N][K] -> int32 [M][N]."""
    Lw, La = _i8(Lw), _i8(La)
    M, K = Lw.shape
    N, K2 = La.shape
    if K != K2:
        raise ValueError("K mismatch")
    C = np.empty((M, N), dtype=np.int32)
    rc = _load().oracle_ternary_gemm(Lw.ctypes.data, La.ctypes.data, M, N, K, act_mode, C.ctypes.data)
    if rc != 0:
        raise ValueError("level outside {0,1,2}")
    return C


def ternary_conv2d(Lw: np.ndarray, Lx: np.ndarray, stride: int = 1, pad: int = 1,
                   act_mode: int = RELU) -> np.ndarray:
    """Lw [Cout][R][S][Cin], Lx [B][H][W][Cin] -> int32 [B][Ho][Wo][Cout], zero padding."""
    Lw, Lx = _i8(Lw), _i8(Lx)
    Cout, R, S, Cin = Lw.shape
    B, H, W, Cin2 = Lx.shape
    if Cin != Cin2:
        raise ValueError("Cin mismatch")
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    Y = np.empty((B, Ho, Wo, Cout), dtype=np.int32)
    rc = _load().oracle_ternary_conv2d(Lw.ctypes.data, Lx.ctypes.data, B, Cin, H, W, Cout, R, S,
                                       stride, pad, act_mode, Y.ctypes.data)
    if rc != 0:
        raise ValueError("level outside {0,1,2}")
    return Y


def twobit_gemm(Qw: np.ndarray, Qa: np.ndarray, basis: int = BASIS_TERNARY) -> np.ndarray:
    """Eq. 2 with two bits per operand, as the integer dot product of the coded values."""
    Qw, Qa = _i8(Qw), _i8(Qa)
    M, K = Qw.shape
    N, K2 = Qa.shape
    if K != K2:
        raise ValueError("K mismatch")
    C = np.empty((M, N), dtype=np.int32)
    rc = _load().oracle_twobit_gemm(Qw.ctypes.data, Qa.ctypes.data, M, N, K, basis, C.ctypes.data)
    if rc != 0:
        raise ValueError("code outside {0,1,2,3}")
    return C


def binary_gemm(Bw: np.ndarray, Ba: np.ndarray) -> np.ndarray:
    """Eq. 1 as the integer dot product of +-1 vectors given as bits 0 / 1."""
    Bw, Ba = _i8(Bw), _i8(Ba)
    M, K = Bw.shape
    N, K2 = Ba.shape
    if K != K2:
        raise ValueError("K mismatch")
    C = np.empty((M, N), dtype=np.int32)
    if _load().oracle_binary_gemm(Bw.ctypes.data, Ba.ctypes.data, M, N, K, C.ctypes.data) != 0:
        raise ValueError("bit outside {0,1}")
    return C


def scale_epilogue(C: np.ndarray, scale: np.ndarray, bias: Optional[np.ndarray], channel_is_row: bool) -> np.ndarray:
    """Cf = scale[ch] * float(C) (+ bias[ch]) in fp32, one rounding per operation."""
    C2 = np.ascontiguousarray(C, dtype=np.int32)
    shape = C2.shape
    if channel_is_row:
        C2 = C2.reshape(shape[0], -1)
    else:
        C2 = C2.reshape(-1, shape[-1])
    scale = np.ascontiguousarray(scale, dtype=np.float32)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    Cf = np.empty(C2.shape, dtype=np.float32)
    _load().oracle_scale_epilogue(C2.ctypes.data, C2.shape[0], C2.shape[1], 1 if channel_is_row else 0,
                                  scale.ctypes.data, None if b is None else b.ctypes.data, Cf.ctypes.data)
    return Cf.reshape(shape)

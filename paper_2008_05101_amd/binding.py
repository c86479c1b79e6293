"""ctypes binding of include/fatnn.h.  Argument marshalling only: every step of the
path (packing, multiply-accumulate, epilogue) runs in the HIP kernels.  torch is
used for device memory and the current stream, nothing else."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfatnn.so")

WEIGHT, ACT = 0, 1
SYM, RELU = 0, 1
ROWMAJOR_K, NHWC, OHWI, OIHW, NCHW = 0, 1, 2, 3, 4
BASIS_TERNARY, BASIS_UNIFORM, BASIS_XNOR_ONLY = 0, 1, 2
X_PLAIN, X_BORDERED, X_BORDERED1 = 0, 1, 2

EXPORTS = [
    "fatnn_words_per_row", "fatnn_packed_bytes", "fatnn_weight_consts_offset",
    "fatnn_weight_interleaved_offset", "fatnn_pack_ternary", "fatnn_bordered_act_bytes",
    "fatnn_pack_ternary_bordered", "fatnn_pack_twobit_bordered", "fatnn_quantize_pack",
    "fatnn_quantize_pack_bordered", "fatnn_bordered_act_init", "fatnn_ternary_conv2d_chain",
    "fatnn_ternary_gemm", "fatnn_ternary_conv2d", "fatnn_pack_twobit", "fatnn_twobit_gemm",
    "fatnn_twobit_conv2d", "fatnn_binary_packed_bytes", "fatnn_pack_binary", "fatnn_binary_gemm",
    "fatnn_gemm_workspace_bytes", "fatnn_gemm_workspace_init", "fatnn_ternary_gemm_ws", "fatnn_twobit_gemm_ws",
    "fatnn_binary_gemm_ws", "fatnn_noalloc_scratch_bytes", "fatnn_ternary_gemm_noalloc",
    "fatnn_time_next_launch", "fatnn_set_tuning", "fatnn_level_status",
    "fatnn_probe_scratch_bytes", "fatnn_probe_valu", "fatnn_probe_hbm", "fatnn_status_str", "fatnn_version",
]


class FatnnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_str(status)} (status {status})")


_lib: Optional[ctypes.CDLL] = None


def lib() -> ctypes.CDLL:
    """Loads libfatnn.so; fails loudly if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2008_05101_amd.build` "
                "(there is no CPU fallback)")
        l = ctypes.CDLL(LIB_PATH)
        vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        l.fatnn_words_per_row.argtypes = [i64]
        l.fatnn_words_per_row.restype = i64
        l.fatnn_packed_bytes.argtypes = [i32, i64, i64]
        l.fatnn_packed_bytes.restype = sz
        l.fatnn_weight_consts_offset.argtypes = [i64, i64]
        l.fatnn_weight_consts_offset.restype = sz
        l.fatnn_weight_interleaved_offset.argtypes = [i64, i64]
        l.fatnn_weight_interleaved_offset.restype = sz
        dims4 = ctypes.POINTER(i64)
        l.fatnn_pack_ternary.argtypes = [vp, i32, dims4, i32, vp, sz, vp, vp]
        l.fatnn_pack_twobit.argtypes = [vp, i32, dims4, i32, vp, sz, vp, vp]
        l.fatnn_ternary_gemm.argtypes = [vp, vp, i64, i64, i64, i32, vp, i64, vp, vp, vp, i64, vp]
        l.fatnn_ternary_conv2d.argtypes = [vp, vp, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp, vp,
                                           vp, vp]
        l.fatnn_bordered_act_bytes.argtypes = [i64, i64, i64, i64, i32]
        l.fatnn_bordered_act_bytes.restype = sz
        l.fatnn_pack_ternary_bordered.argtypes = [vp, dims4, i32, i32, vp, sz, vp, vp]
        l.fatnn_pack_twobit_bordered.argtypes = [vp, dims4, i32, vp, sz, vp, vp]
        f32 = ctypes.c_float
        l.fatnn_quantize_pack.argtypes = [vp, i32, dims4, i32, i32, f32, f32, vp, sz, vp, vp]
        l.fatnn_quantize_pack_bordered.argtypes = [vp, dims4, i32, i32, f32, f32, vp, sz, vp, vp]
        l.fatnn_bordered_act_init.argtypes = [vp, sz, i64, i64, i64, i64, i32, i32, vp]
        l.fatnn_ternary_conv2d_chain.argtypes = [vp, vp, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp,
                                                 vp, i32, f32, f32, i32, i32, vp, sz, vp, vp]
        l.fatnn_twobit_gemm.argtypes = [vp, vp, i64, i64, i64, i32, vp, i64, vp]
        l.fatnn_twobit_conv2d.argtypes = [vp, vp, i32, i64, i64, i64, i64, i64, i32, i32, i32, i32, i32, vp, vp]
        l.fatnn_binary_packed_bytes.argtypes = [i64, i64]
        l.fatnn_binary_packed_bytes.restype = sz
        l.fatnn_pack_binary.argtypes = [vp, i64, i64, vp, sz, vp, vp]
        l.fatnn_binary_gemm.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp]
        l.fatnn_time_next_launch.argtypes = [vp, vp]
        l.fatnn_set_tuning.argtypes = [i32, i32, i32, i32, i32]
        l.fatnn_gemm_workspace_bytes.restype = sz
        l.fatnn_gemm_workspace_init.argtypes = [vp, sz, vp]
        l.fatnn_ternary_gemm_ws.argtypes = [vp, vp, i64, i64, i64, i32, vp, i64, vp, vp, vp, i64, vp, sz, vp]
        l.fatnn_noalloc_scratch_bytes.restype = sz
        l.fatnn_ternary_gemm_noalloc.argtypes = [vp, vp, i64, i64, i64, i32, vp, i64, vp, vp, vp, i64, vp]
        l.fatnn_twobit_gemm_ws.argtypes = [vp, vp, i64, i64, i64, i32, vp, i64, vp, sz, vp]
        l.fatnn_binary_gemm_ws.argtypes = [vp, vp, i64, i64, i64, vp, i64, vp, sz, vp]
        l.fatnn_level_status.argtypes = [i64]
        l.fatnn_probe_scratch_bytes.restype = sz
        l.fatnn_probe_valu.argtypes = [i32, i32, i32, vp, sz, ctypes.POINTER(i64), vp]
        l.fatnn_probe_hbm.argtypes = [i32, vp, vp, sz, vp, sz, vp]
        l.fatnn_status_str.argtypes = [i32]
        l.fatnn_status_str.restype = ctypes.c_char_p
        l.fatnn_version.restype = i32
        _lib = l
    return _lib


def status_str(status: int) -> str:
    return lib().fatnn_status_str(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise FatnnError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype: torch.dtype, what: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{what} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{what} must be {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def pack_binary(bits: torch.Tensor, out: Optional[torch.Tensor] = None,
                n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    bits = _dev(bits, torch.int8, "bits")
    rows, K = bits.shape
    if out is None:
        out = torch.empty(max(int(lib().fatnn_binary_packed_bytes(rows, K)), 16), dtype=torch.uint8,
                          device=bits.device)
    chk = _LevelCheck(check_levels, n_invalid, bits.device)
    n_invalid = chk.counter
    _check(lib().fatnn_pack_binary(_ptr(bits), rows, K, _ptr(out), out.numel(), _ptr(n_invalid), _stream()),
           "fatnn_pack_binary")
    chk.finish("fatnn_pack_binary")
    return out


def binary_gemm(Wb: torch.Tensor, Ab: torch.Tensor, M: int, N: int, K: int,
                out: Optional[torch.Tensor] = None, workspace="auto") -> torch.Tensor:
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=Wb.device)
    ldc = out.stride(0) if out.dim() == 2 and M > 0 else N
    ws = _ws(workspace, Wb.device)
    _check(lib().fatnn_binary_gemm_ws(_ptr(Wb), _ptr(Ab), M, N, K, _ptr(out), max(ldc, N), _ptr(ws),
                                      0 if ws is None else ws.numel(), _stream()), "fatnn_binary_gemm_ws")
    return out


def set_tuning(conv_kernel: int = -1, stream_wps: int = -1, seven_pixel_groups: int = -1,
               gemm_even_share: int = -1, gemm_deepk: int = -1) -> None:
    """fatnn_set_tuning: process-wide measurement switches; -1 keeps a value."""
    _check(lib().fatnn_set_tuning(conv_kernel, stream_wps, seven_pixel_groups, gemm_even_share, gemm_deepk),
           "fatnn_set_tuning")


_workspaces = {}


def gemm_workspace(device, nbytes: Optional[int] = None) -> torch.Tensor:
    """A workspace for the *_gemm_ws calls: allocated by torch and initialised once per device (or a fresh
    one of `nbytes` bytes).  Calls that use the shared one must run on one stream at a time."""
    dev = torch.device(device)
    if dev.index is None:
        dev = torch.device("cuda", torch.cuda.current_device())
    if nbytes is None and dev in _workspaces:
        return _workspaces[dev]
    ws = torch.empty(int(lib().fatnn_gemm_workspace_bytes()) if nbytes is None else nbytes, dtype=torch.uint8, device=dev)
    _check(lib().fatnn_gemm_workspace_init(_ptr(ws), ws.numel(), _stream()), "fatnn_gemm_workspace_init")
    if nbytes is None:
        _workspaces[dev] = ws
    return ws


def _ws(workspace, device) -> Optional[torch.Tensor]:
    """workspace argument of the GEMM wrappers: "auto" = the device's shared one, None = none, or a tensor."""
    if isinstance(workspace, str):
        return gemm_workspace(device)
    return workspace


PROBE_PAIR_V, PROBE_PAIR_S, PROBE_BCNT, PROBE_BITOP3, PROBE_XOR, PROBE_PAIR_LDS = 0, 1, 2, 3, 4, 5
HBM_READ, HBM_WRITE, HBM_COPY = 0, 1, 2


def probe_scratch(device="cuda") -> torch.Tensor:
    """Scratch buffer the roofline probes need (its contents serve as operand bits)."""
    return torch.empty(int(lib().fatnn_probe_scratch_bytes()), dtype=torch.uint8, device=device).fill_(0x5A)


def probe_valu(kind: int, waves_per_simd: int, iters: int, scratch: torch.Tensor) -> int:
    """fatnn_probe_valu; returns the number of 32-bit lane-instructions the launch executes."""
    n = ctypes.c_int64(0)
    _check(lib().fatnn_probe_valu(kind, waves_per_simd, iters, _ptr(scratch), scratch.numel(), ctypes.byref(n),
                                  _stream()), "fatnn_probe_valu")
    return int(n.value)


def probe_hbm(kind: int, dst: Optional[torch.Tensor], src: Optional[torch.Tensor], nbytes: int,
              scratch: torch.Tensor) -> None:
    _check(lib().fatnn_probe_hbm(kind, _ptr(dst), _ptr(src), nbytes, _ptr(scratch), scratch.numel(), _stream()),
           "fatnn_probe_hbm")


class _LevelCheck:
    """check_levels=True of the packing wrappers: a zeroed device counter for the call, read back
    afterwards (this synchronises the stream) and turned into FATNN_ERR_LEVEL when it is not zero."""

    def __init__(self, enabled: bool, n_invalid: Optional[torch.Tensor], device):
        self.counter = n_invalid
        self.enabled = enabled
        self.before = 0
        if enabled:
            if n_invalid is None:
                self.counter = torch.zeros(1, dtype=torch.int32, device=device)
            else:
                self.before = int(n_invalid.item())

    def finish(self, where: str) -> None:
        if self.enabled:
            _check(lib().fatnn_level_status(int(self.counter.item()) - self.before), where)


def time_next_launch(start_event: Optional[int], stop_event: Optional[int]) -> None:
    """fatnn_time_next_launch: raw hipEvent_t handles (ints) or (None, None)."""
    _check(lib().fatnn_time_next_launch(start_event, stop_event), "fatnn_time_next_launch")


def words_per_row(K: int) -> int:
    return int(lib().fatnn_words_per_row(K))


def packed_bytes(role: int, rows: int, K: int) -> int:
    return int(lib().fatnn_packed_bytes(role, rows, K))


def weight_consts_offset(rows: int, K: int) -> int:
    return int(lib().fatnn_weight_consts_offset(rows, K))


def weight_interleaved_offset(rows: int, K: int) -> int:
    return int(lib().fatnn_weight_interleaved_offset(rows, K))


def _rows_k(layout: int, dims: Sequence[int]) -> Tuple[int, int]:
    d = list(dims)
    if layout == ROWMAJOR_K:
        return d[0], d[1]
    if layout == NHWC:
        return d[0] * d[1] * d[2], d[3]
    if layout == OHWI:
        return d[0], d[1] * d[2] * d[3]
    if layout == OIHW:
        return d[0], d[1] * d[2] * d[3]
    if layout == NCHW:
        return d[0] * d[2] * d[3], d[1]
    raise ValueError("unknown layout")


def _dims4(layout: int, levels: torch.Tensor):
    shape = list(levels.shape)
    if layout == ROWMAJOR_K:
        if len(shape) != 2:
            raise ValueError("ROWMAJOR_K wants a 2-D tensor")
        shape = shape + [1, 1]
    elif len(shape) != 4:
        raise ValueError("layout wants a 4-D tensor")
    return (ctypes.c_int64 * 4)(*shape), shape


def pack_ternary(levels: torch.Tensor, role: int, layout: int = ROWMAJOR_K,
                 out: Optional[torch.Tensor] = None, n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    """fatnn_pack_ternary: int8 level tensor -> packed plane words (uint8 buffer)."""
    levels = _dev(levels, torch.int8, "levels")
    dims, shape = _dims4(layout, levels)
    rows, K = _rows_k(layout, shape)
    nbytes = packed_bytes(role, rows, K) if K >= 1 else 0
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=levels.device)
    chk = _LevelCheck(check_levels, n_invalid, levels.device)
    n_invalid = chk.counter
    _check(lib().fatnn_pack_ternary(_ptr(levels), layout, dims, role, _ptr(out), out.numel(),
                                    _ptr(n_invalid), _stream()), "fatnn_pack_ternary")
    chk.finish("fatnn_pack_ternary")
    return out


def pack_twobit(codes: torch.Tensor, role: int = ACT, layout: int = ROWMAJOR_K,
                out: Optional[torch.Tensor] = None, n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    codes = _dev(codes, torch.int8, "codes")
    dims, shape = _dims4(layout, codes)
    rows, K = _rows_k(layout, shape)
    nbytes = packed_bytes(role, rows, K) if K >= 1 else 0
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=codes.device)
    chk = _LevelCheck(check_levels, n_invalid, codes.device)
    n_invalid = chk.counter
    _check(lib().fatnn_pack_twobit(_ptr(codes), layout, dims, role, _ptr(out), out.numel(), _ptr(n_invalid),
                                   _stream()), "fatnn_pack_twobit")
    chk.finish("fatnn_pack_twobit")
    return out


def bordered_act_bytes(B: int, H: int, W: int, C: int, border: int) -> int:
    return int(lib().fatnn_bordered_act_bytes(B, H, W, C, border))


def pack_ternary_bordered(levels: torch.Tensor, border: int, act_mode: int, out: Optional[torch.Tensor] = None,
                          n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    """fatnn_pack_ternary_bordered: NHWC int8 levels -> bordered packed activations."""
    levels = _dev(levels, torch.int8, "levels")
    if levels.dim() != 4:
        raise ValueError("levels must be NHWC")
    B, H, W, C = levels.shape
    dims = (ctypes.c_int64 * 4)(B, H, W, C)
    if out is None:
        out = torch.empty(max(bordered_act_bytes(B, H, W, C, border), 16), dtype=torch.uint8, device=levels.device)
    chk = _LevelCheck(check_levels, n_invalid, levels.device)
    n_invalid = chk.counter
    _check(lib().fatnn_pack_ternary_bordered(_ptr(levels), dims, border, act_mode, _ptr(out), out.numel(),
                                             _ptr(n_invalid), _stream()), "fatnn_pack_ternary_bordered")
    chk.finish("fatnn_pack_ternary_bordered")
    return out


def pack_twobit_bordered(codes: torch.Tensor, border: int, out: Optional[torch.Tensor] = None,
                         n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    codes = _dev(codes, torch.int8, "codes")
    if codes.dim() != 4:
        raise ValueError("codes must be NHWC")
    B, H, W, C = codes.shape
    dims = (ctypes.c_int64 * 4)(B, H, W, C)
    if out is None:
        out = torch.empty(max(bordered_act_bytes(B, H, W, C, border), 16), dtype=torch.uint8, device=codes.device)
    chk = _LevelCheck(check_levels, n_invalid, codes.device)
    n_invalid = chk.counter
    _check(lib().fatnn_pack_twobit_bordered(_ptr(codes), dims, border, _ptr(out), out.numel(), _ptr(n_invalid),
                                            _stream()), "fatnn_pack_twobit_bordered")
    chk.finish("fatnn_pack_twobit_bordered")
    return out


def quantize_pack(x: torch.Tensor, role: int, act_mode: int, alpha1: float, alpha2: float,
                  layout: int = ROWMAJOR_K, out: Optional[torch.Tensor] = None,
                  n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    """fatnn_quantize_pack: float32 tensor -> packed plane words through the paper's quantizer."""
    x = _dev(x, torch.float32, "x")
    dims, shape = _dims4(layout, x)
    rows, K = _rows_k(layout, shape)
    nbytes = packed_bytes(role, rows, K) if K >= 1 else 0
    if out is None:
        out = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=x.device)
    chk = _LevelCheck(check_levels, n_invalid, x.device)
    n_invalid = chk.counter
    _check(lib().fatnn_quantize_pack(_ptr(x), layout, dims, role, act_mode, alpha1, alpha2, _ptr(out), out.numel(),
                                     _ptr(n_invalid), _stream()), "fatnn_quantize_pack")
    chk.finish("fatnn_quantize_pack")
    return out


def quantize_pack_bordered(x: torch.Tensor, border: int, act_mode: int, alpha1: float, alpha2: float,
                           out: Optional[torch.Tensor] = None,
                           n_invalid: Optional[torch.Tensor] = None,
                          check_levels: bool = False) -> torch.Tensor:
    x = _dev(x, torch.float32, "x")
    if x.dim() != 4:
        raise ValueError("x must be NHWC")
    B, H, W, C = x.shape
    dims = (ctypes.c_int64 * 4)(B, H, W, C)
    if out is None:
        out = torch.empty(max(bordered_act_bytes(B, H, W, C, border), 16), dtype=torch.uint8, device=x.device)
    chk = _LevelCheck(check_levels, n_invalid, x.device)
    n_invalid = chk.counter
    _check(lib().fatnn_quantize_pack_bordered(_ptr(x), dims, border, act_mode, alpha1, alpha2, _ptr(out),
                                              out.numel(), _ptr(n_invalid), _stream()),
           "fatnn_quantize_pack_bordered")
    chk.finish("fatnn_quantize_pack_bordered")
    return out


def ternary_gemm(Wp: torch.Tensor, Ap: torch.Tensor, M: int, N: int, K: int, act_mode: int = SYM,
                 out: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                 bias: Optional[torch.Tensor] = None, out_f: Optional[torch.Tensor] = None,
                 want_int: bool = True, workspace="auto"):
    """fatnn_ternary_gemm_ws.  Returns (C int32 [M][N] or None, Cf fp32 [M][N] or None)."""
    if out is None and want_int:
        out = torch.empty((M, N), dtype=torch.int32, device=Wp.device)
    if scale is not None and out_f is None:
        out_f = torch.empty((M, N), dtype=torch.float32, device=Wp.device)
    ldc = out.stride(0) if out is not None and out.dim() == 2 and M > 0 else N
    ldcf = out_f.stride(0) if out_f is not None and out_f.dim() == 2 and M > 0 else N
    ws = _ws(workspace, Wp.device)
    _check(lib().fatnn_ternary_gemm_ws(_ptr(Wp), _ptr(Ap), M, N, K, act_mode, _ptr(out), max(ldc, N), _ptr(scale),
                                       _ptr(bias), _ptr(out_f), max(ldcf, N), _ptr(ws),
                                       0 if ws is None else ws.numel(), _stream()), "fatnn_ternary_gemm_ws")
    return out, out_f


def ternary_gemm_noalloc(Wp: torch.Tensor, Ap: torch.Tensor, M: int, N: int, K: int, act_mode: int,
                         out: Optional[torch.Tensor], scale: Optional[torch.Tensor] = None,
                         bias: Optional[torch.Tensor] = None, out_f: Optional[torch.Tensor] = None) -> None:
    """fatnn_ternary_gemm_noalloc: the caller brings every output; nothing is allocated here or in the library."""
    ldc = out.stride(0) if out is not None and out.dim() == 2 and M > 0 else N
    ldcf = out_f.stride(0) if out_f is not None and out_f.dim() == 2 and M > 0 else N
    _check(lib().fatnn_ternary_gemm_noalloc(_ptr(Wp), _ptr(Ap), M, N, K, act_mode, _ptr(out), max(ldc, N), _ptr(scale),
                                            _ptr(bias), _ptr(out_f), max(ldcf, N), _stream()),
           "fatnn_ternary_gemm_noalloc")


def _conv_out_hw(H: int, W: int, R: int, S: int, stride: int, pad: int) -> Tuple[int, int]:
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def ternary_conv2d(Wp: torch.Tensor, Xp: torch.Tensor, B: int, Cin: int, H: int, W: int, Cout: int,
                   R: int = 3, S: int = 3, stride: int = 1, pad: int = 1, act_mode: int = RELU,
                   out: Optional[torch.Tensor] = None, scale: Optional[torch.Tensor] = None,
                   bias: Optional[torch.Tensor] = None, out_f: Optional[torch.Tensor] = None,
                   want_int: bool = True, x_layout: int = X_PLAIN):
    """fatnn_ternary_conv2d.  Returns (Y int32 NHWC or None, Yf fp32 NHWC or None)."""
    Ho, Wo = _conv_out_hw(H, W, R, S, stride, pad)
    if out is None and want_int:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.int32, device=Wp.device)
    if scale is not None and out_f is None:
        out_f = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=Wp.device)
    _check(lib().fatnn_ternary_conv2d(_ptr(Wp), _ptr(Xp), x_layout, B, Cin, H, W, Cout, R, S, stride, pad, act_mode,
                                      _ptr(out), _ptr(scale), _ptr(bias), _ptr(out_f), _stream()),
           "fatnn_ternary_conv2d")
    return out, out_f


def bordered_act_init(B: int, H: int, W: int, C: int, border: int, act_mode: int,
                      out: Optional[torch.Tensor] = None, device=None) -> torch.Tensor:
    """Allocates (or takes) a bordered activation buffer and fills it with the value 0."""
    if out is None:
        out = torch.empty(max(bordered_act_bytes(B, H, W, C, border), 16), dtype=torch.uint8,
                          device=device if device is not None else "cuda")
    _check(lib().fatnn_bordered_act_init(_ptr(out), out.numel(), B, H, W, C, border, act_mode, _stream()),
           "fatnn_bordered_act_init")
    return out


def ternary_conv2d_chain(Wp: torch.Tensor, Xp: torch.Tensor, B: int, Cin: int, H: int, W: int, Cout: int,
                         R: int, S: int, stride: int, pad: int, act_mode: int, scale: torch.Tensor,
                         bias: Optional[torch.Tensor], skip: Optional[torch.Tensor], relu: bool,
                         alpha1: float, alpha2: float, out_act_mode: int, out_border: int, x_next: torch.Tensor,
                         out_f: Optional[torch.Tensor] = None, x_layout: int = X_BORDERED) -> torch.Tensor:
    """fatnn_ternary_conv2d_chain: conv + affine (+skip, ReLU) + next layer's quantizer + packing."""
    _check(lib().fatnn_ternary_conv2d_chain(_ptr(Wp), _ptr(Xp), x_layout, B, Cin, H, W, Cout, R, S, stride, pad, act_mode,
                                            _ptr(scale), _ptr(bias), _ptr(skip), 1 if relu else 0, alpha1, alpha2,
                                            out_act_mode, out_border, _ptr(x_next), x_next.numel(), _ptr(out_f),
                                            _stream()), "fatnn_ternary_conv2d_chain")
    return x_next


def twobit_gemm(Wp: torch.Tensor, Ap: torch.Tensor, M: int, N: int, K: int, basis: int = BASIS_TERNARY,
                out: Optional[torch.Tensor] = None, workspace="auto") -> torch.Tensor:
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32, device=Wp.device)
    ldc = out.stride(0) if out.dim() == 2 and M > 0 else N
    ws = _ws(workspace, Wp.device)
    _check(lib().fatnn_twobit_gemm_ws(_ptr(Wp), _ptr(Ap), M, N, K, basis, _ptr(out), max(ldc, N), _ptr(ws),
                                      0 if ws is None else ws.numel(), _stream()), "fatnn_twobit_gemm_ws")
    return out


def twobit_conv2d(Wp: torch.Tensor, Xp: torch.Tensor, B: int, Cin: int, H: int, W: int, Cout: int,
                  R: int = 3, S: int = 3, stride: int = 1, pad: int = 1, basis: int = BASIS_TERNARY,
                  out: Optional[torch.Tensor] = None, x_layout: int = X_PLAIN) -> torch.Tensor:
    Ho, Wo = _conv_out_hw(H, W, R, S, stride, pad)
    if out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.int32, device=Wp.device)
    _check(lib().fatnn_twobit_conv2d(_ptr(Wp), _ptr(Xp), x_layout, B, Cin, H, W, Cout, R, S, stride, pad, basis,
                                     _ptr(out), _stream()), "fatnn_twobit_conv2d")
    return out

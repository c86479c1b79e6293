"""CPU-only tests of the C-ABI boundary: the library loads, exports every symbol the
header declares, reports sizes, and turns bad arguments into status codes before any
GPU call (so all of this runs on a box with no GPU).  No compute is launched here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fatnn.h")

fatnn = pytest.importorskip("paper_2008_05101_amd")
from paper_2008_05101_amd import binding  # noqa: E402

OK, E_NULL, E_SHAPE, E_LEVEL, E_ALIGN, E_SIZE, E_UNSUP, E_HIP = 0, -1, -2, -3, -4, -5, -6, -7


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2008_05101_amd import build
        build.build(force=True)
    return fatnn.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fatnn_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in fatnn.h but not exported"
    assert sorted(binding.EXPORTS) == names


def test_header_cites_the_paper_for_every_entry_point():
    text = open(HEADER).read()
    for key in ("Algorithm 1", "Eq. 3", "Eq. 2", "Table 1", "Section 3.3", "Supplementary S1"):
        assert key in text


def test_sizes(lib):
    assert lib.fatnn_words_per_row(1) == 1
    assert lib.fatnn_words_per_row(32) == 1
    assert lib.fatnn_words_per_row(33) == 2
    assert lib.fatnn_words_per_row(4609) == 145
    assert lib.fatnn_words_per_row(0) == -1
    assert lib.fatnn_packed_bytes(fatnn.ACT, 64, 576) == 64 * 18 * 8
    assert lib.fatnn_packed_bytes(fatnn.ACT, 0, 576) == 0
    assert lib.fatnn_packed_bytes(7, 64, 576) == 0
    off = lib.fatnn_weight_consts_offset(37, 100)
    assert off % 256 == 0 and off >= 37 * 4 * 8
    ioff = lib.fatnn_weight_interleaved_offset(37, 100)
    assert ioff % 256 == 0 and ioff >= off + 37 * 8
    assert lib.fatnn_packed_bytes(fatnn.WEIGHT, 37, 100) == ioff + 64 * 4 * 8
    assert lib.fatnn_bordered_act_bytes(2, 5, 4, 64, 1) == (2 * 7 * 6 + 64) * 2 * 8
    assert lib.fatnn_bordered_act_bytes(2, 5, 4, 48, 1) == 0
    assert lib.fatnn_bordered_act_bytes(2, 5, 4, 64, 2) == 0


def test_status_strings(lib):
    seen = set()
    for code in range(0, -8, -1):
        s = lib.fatnn_status_str(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lib.fatnn_status_str(5).decode() == "unknown status"
    assert lib.fatnn_version() >= 100


def test_level_status_and_tuning_arguments(lib):
    assert lib.fatnn_level_status(0) == 0
    assert lib.fatnn_level_status(1) == -3 and lib.fatnn_level_status(1 << 40) == -3
    assert lib.fatnn_status_str(-3).decode() == "level outside {0,1,2}"
    assert lib.fatnn_set_tuning(-1, -1, -1, -1, -1) == 0            # keeps everything
    assert lib.fatnn_set_tuning(2, 0, 1, 0, 0) == -6
    assert lib.fatnn_set_tuning(0, 9, 1, 0, 0) == -6
    assert lib.fatnn_set_tuning(0, 0, 3, 0, 0) == -6
    assert lib.fatnn_set_tuning(0, 0, 1, 12, 0) == -6
    assert lib.fatnn_set_tuning(0, 0, 1, 0, 3) == -6
    assert lib.fatnn_set_tuning(0, 0, 1, 0, 0) == 0


def dims(*v):
    return (ctypes.c_int64 * 4)(*v)


FAKE = 0x10000      # never dereferenced: every call below fails (or returns) before a launch


def test_pack_argument_errors(lib):
    f = lib.fatnn_pack_ternary
    assert f(FAKE, fatnn.ROWMAJOR_K, None, fatnn.ACT, FAKE, 1 << 20, None, None) == E_NULL
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 0, 1, 1), fatnn.ACT, FAKE, 1 << 20, None, None) == E_SHAPE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(-1, 8, 1, 1), fatnn.ACT, FAKE, 1 << 20, None, None) == E_SHAPE
    assert f(FAKE, 99, dims(4, 8, 1, 1), fatnn.ACT, FAKE, 1 << 20, None, None) == E_UNSUP
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), 5, FAKE, 1 << 20, None, None) == E_UNSUP
    assert f(FAKE, fatnn.NHWC, dims(1, 4, 4, 48), fatnn.ACT, FAKE, 1 << 20, None, None) == E_UNSUP
    assert f(FAKE, fatnn.OHWI, dims(8, 3, 3, 0), fatnn.WEIGHT, FAKE, 1 << 20, None, None) == E_SHAPE
    assert f(None, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, FAKE, 1 << 20, None, None) == E_NULL
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, None, 1 << 20, None, None) == E_NULL
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, FAKE + 4, 1 << 20, None, None) == E_ALIGN
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, FAKE, 31, None, None) == E_SIZE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.WEIGHT, FAKE, 32, None, None) == E_SIZE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 1 << 25, 1, 1), fatnn.ACT, FAKE, 1 << 40, None, None) == E_SIZE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(1 << 32, 8, 1, 1), fatnn.ACT, FAKE, 1 << 40, None, None) == E_SIZE
    # nothing to pack is fine, whatever the pointers
    assert f(None, fatnn.ROWMAJOR_K, dims(0, 8, 1, 1), fatnn.ACT, None, 0, None, None) == OK
    g = lib.fatnn_pack_twobit
    assert g(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), 3, FAKE, 1 << 20, None, None) == E_UNSUP
    assert g(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, FAKE, 8, None, None) == E_SIZE


def test_bordered_pack_argument_errors(lib):
    f = lib.fatnn_pack_ternary_bordered
    big = 1 << 30
    assert f(FAKE, None, 1, 0, FAKE, big, None, None) == E_NULL
    assert f(FAKE, dims(2, 0, 4, 64), 1, 0, FAKE, big, None, None) == E_SHAPE
    assert f(FAKE, dims(2, 4, 4, 48), 1, 0, FAKE, big, None, None) == E_UNSUP
    assert f(FAKE, dims(2, 4, 4, 64), 2, 0, FAKE, big, None, None) == E_UNSUP
    assert f(FAKE, dims(2, 4, 4, 64), 1, 3, FAKE, big, None, None) == E_UNSUP
    assert f(None, dims(2, 4, 4, 64), 1, 0, FAKE, big, None, None) == E_NULL
    assert f(FAKE, dims(2, 4, 4, 64), 1, 0, None, big, None, None) == E_NULL
    assert f(FAKE + 8, dims(2, 4, 4, 64), 1, 0, FAKE, big, None, None) == E_ALIGN
    assert f(FAKE, dims(2, 4, 4, 64), 1, 0, FAKE, 100, None, None) == E_SIZE
    g = lib.fatnn_pack_twobit_bordered
    assert g(FAKE, dims(2, 4, 4, 64), 1, FAKE, 100, None, None) == E_SIZE


def test_quantize_pack_argument_errors(lib):
    f = lib.fatnn_quantize_pack
    f.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int64), ctypes.c_int, ctypes.c_int,
                  ctypes.c_float, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
    big = 1 << 30
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, 0.0, 1.0, FAKE, big, None, None) == E_SHAPE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, 1.0, -2.0, FAKE, big, None, None) == E_SHAPE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, float("nan"), 1.0, FAKE, big, None, None) == E_SHAPE
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, float("inf"), 1.0, FAKE, big, None, None) == E_SHAPE
    assert f(FAKE, fatnn.OIHW, dims(4, 32, 3, 3), fatnn.WEIGHT, 0, 1.0, 1.0, FAKE, big, None, None) == E_UNSUP
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), 9, 0, 1.0, 1.0, FAKE, big, None, None) == E_UNSUP
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 5, 1.0, 1.0, FAKE, big, None, None) == E_UNSUP
    assert f(None, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, 1.0, 1.0, FAKE, big, None, None) == E_NULL
    assert f(FAKE + 2, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, 1.0, 1.0, FAKE, big, None, None) == E_ALIGN
    assert f(FAKE, fatnn.ROWMAJOR_K, dims(4, 8, 1, 1), fatnn.ACT, 0, 1.0, 1.0, FAKE, 8, None, None) == E_SIZE
    assert f(None, fatnn.ROWMAJOR_K, dims(0, 8, 1, 1), fatnn.ACT, 0, 1.0, 1.0, None, 0, None, None) == OK
    g = lib.fatnn_quantize_pack_bordered
    assert g(FAKE, dims(2, 4, 4, 64), 1, 0, 1.0, 0.0, FAKE, big, None, None) == E_SHAPE
    assert g(FAKE, dims(2, 4, 4, 48), 1, 0, 1.0, 1.0, FAKE, big, None, None) == E_UNSUP
    assert g(FAKE, dims(2, 4, 4, 64), 1, 0, 1.0, 1.0, FAKE, 100, None, None) == E_SIZE


def test_gemm_argument_errors(lib):
    f = lib.fatnn_ternary_gemm
    a = (FAKE, FAKE)
    assert f(*a, -1, 4, 8, 0, FAKE, 4, None, None, None, 0, None) == E_SHAPE
    assert f(*a, 4, 4, 0, 0, FAKE, 4, None, None, None, 0, None) == E_SHAPE
    assert f(*a, 4, 4, (1 << 24) + 1, 0, FAKE, 4, None, None, None, 0, None) == E_SIZE
    assert f(*a, 4, 4, 8, 2, FAKE, 4, None, None, None, 0, None) == E_UNSUP
    assert f(*a, 4, 4, 8, 0, None, 4, None, None, None, 0, None) == E_NULL            # no output at all
    assert f(*a, 4, 4, 8, 0, None, 4, None, None, FAKE, 4, None) == E_NULL            # Cf without scale
    assert f(*a, 4, 4, 8, 0, FAKE, 3, None, None, None, 0, None) == E_SHAPE           # ldc < N
    assert f(*a, 4, 4, 8, 0, None, 0, FAKE, None, FAKE, 3, None) == E_SHAPE           # ldcf < N
    assert f(None, FAKE, 4, 4, 8, 0, FAKE, 4, None, None, None, 0, None) == E_NULL
    assert f(FAKE, None, 4, 4, 8, 0, FAKE, 4, None, None, None, 0, None) == E_NULL
    assert f(FAKE + 8, FAKE, 4, 4, 8, 0, FAKE, 4, None, None, None, 0, None) == E_ALIGN
    assert f(FAKE, FAKE, 4, 4, 8, 0, FAKE + 2, 4, None, None, None, 0, None) == E_ALIGN
    assert f(None, None, 0, 4, 8, 0, None, 4, None, None, None, 0, None) == OK          # empty problem
    assert f(None, None, 4, 0, 8, 0, None, 0, None, None, None, 0, None) == OK
    g = lib.fatnn_twobit_gemm
    assert g(*a, 4, 4, 8, 7, FAKE, 4, None) == E_UNSUP
    assert g(*a, 4, 4, 8, 0, None, 4, None) == E_NULL
    assert g(*a, 4, 4, 8, 0, FAKE, 2, None) == E_SHAPE
    assert g(*a, 4, 4, (1 << 20) + 1, 1, FAKE, 4, None) == E_SIZE                     # 9K must fit int32


def test_workspace_noalloc_and_probe_argument_errors(lib):
    assert lib.fatnn_gemm_workspace_bytes() == 65536 + 1024 * 2 * 64 * 32 * 3 * 4
    assert lib.fatnn_noalloc_scratch_bytes() == 65536 + 512 * 2 * 64 * 64 * 4
    assert lib.fatnn_probe_scratch_bytes() >= 4096 + 256 * 8 * 256 * 4
    big = lib.fatnn_gemm_workspace_bytes()
    init = lib.fatnn_gemm_workspace_init
    assert init(None, big, None) == E_NULL
    assert init(FAKE + 4, big, None) == E_ALIGN
    assert init(FAKE, 1000, None) == E_SIZE
    f = lib.fatnn_ternary_gemm_ws
    a = (FAKE, FAKE)
    assert f(*a, 4, 4, 8, 0, FAKE, 4, None, None, None, 0, FAKE + 8, big, None) == E_ALIGN      # workspace alignment
    assert f(*a, 4, 4, 0, 0, FAKE, 4, None, None, None, 0, FAKE, big, None) == E_SHAPE
    assert f(None, None, 0, 4, 8, 0, None, 4, None, None, None, 0, None, 0, None) == OK
    assert lib.fatnn_twobit_gemm_ws(*a, 4, 4, 8, 0, FAKE, 4, FAKE + 8, big, None) == E_ALIGN
    assert lib.fatnn_binary_gemm_ws(*a, 4, 4, 8, FAKE, 4, FAKE + 8, big, None) == E_ALIGN
    g = lib.fatnn_ternary_gemm_noalloc
    assert g(*a, 4, 4, 0, 0, FAKE, 4, None, None, None, 0, None) == E_SHAPE
    assert g(*a, 4, 4, 8, 3, FAKE, 4, None, None, None, 0, None) == E_UNSUP
    assert g(*a, 64 * 129, 64 * 128, 64, 0, FAKE, 64 * 128, None, None, None, 0, None) == E_SIZE  # > 16384 tiles
    assert g(*a, 4, 4, 8, 0, None, 4, None, None, None, 0, None) == E_NULL
    assert g(*a, 4, 4, 8, 0, FAKE, 3, None, None, None, 0, None) == E_SHAPE
    assert g(FAKE + 8, FAKE, 4, 4, 8, 0, FAKE, 4, None, None, None, 0, None) == E_ALIGN
    assert g(None, None, 0, 4, 8, 0, None, 4, None, None, None, 0, None) == OK
    pv = lib.fatnn_probe_valu
    sb = lib.fatnn_probe_scratch_bytes()
    assert pv(6, 4, 10, FAKE, sb, None, None) == E_UNSUP
    assert pv(0, 0, 10, FAKE, sb, None, None) == E_SHAPE
    assert pv(0, 9, 10, FAKE, sb, None, None) == E_SHAPE
    assert pv(0, 4, 0, FAKE, sb, None, None) == E_SHAPE
    assert pv(0, 4, 10, None, sb, None, None) == E_NULL
    assert pv(0, 4, 10, FAKE + 4, sb, None, None) == E_ALIGN
    assert pv(0, 4, 10, FAKE, 100, None, None) == E_SIZE
    ph = lib.fatnn_probe_hbm
    assert ph(3, FAKE, FAKE, 1 << 20, FAKE, sb, None) == E_UNSUP
    assert ph(2, FAKE, FAKE, 24, FAKE, sb, None) == E_SHAPE
    assert ph(0, None, None, 1 << 20, FAKE, sb, None) == E_NULL
    assert ph(1, None, FAKE, 1 << 20, FAKE, sb, None) == E_NULL
    assert ph(2, FAKE, FAKE + 8, 1 << 20, FAKE, sb, None) == E_ALIGN
    assert ph(2, FAKE, FAKE, 1 << 20, FAKE, 64, None) == E_SIZE


def test_binary_argument_errors(lib):
    f = lib.fatnn_pack_binary
    assert lib.fatnn_binary_packed_bytes(3, 65) == 3 * 2 * 8
    assert lib.fatnn_binary_packed_bytes(3, 0) == 0
    assert f(FAKE, 4, 0, FAKE, 1 << 20, None, None) == E_SHAPE
    assert f(None, 4, 8, FAKE, 1 << 20, None, None) == E_NULL
    assert f(FAKE, 4, 8, FAKE + 4, 1 << 20, None, None) == E_ALIGN
    assert f(FAKE, 4, 8, FAKE, 8, None, None) == E_SIZE
    assert f(None, 0, 8, None, 0, None, None) == OK
    g = lib.fatnn_binary_gemm
    assert g(FAKE, FAKE, 4, 4, 0, FAKE, 4, None) == E_SHAPE
    assert g(FAKE, FAKE, 4, 4, 8, None, 4, None) == E_NULL
    assert g(FAKE, FAKE, 4, 4, 8, FAKE, 3, None) == E_SHAPE
    assert g(FAKE, FAKE + 8, 4, 4, 8, FAKE, 4, None) == E_ALIGN
    assert g(None, None, 0, 4, 8, None, 4, None) == OK


def test_chain_argument_errors(lib):
    f = lib.fatnn_ternary_conv2d_chain
    f.argtypes = ([ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int] + [ctypes.c_int64] * 5 + [ctypes.c_int] * 5 +
                  [ctypes.c_void_p] * 3 + [ctypes.c_int, ctypes.c_float, ctypes.c_float, ctypes.c_int, ctypes.c_int,
                                           ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p])

    def call(xl=1, Cin=64, Cout=64, R=3, S=3, stride=1, pad=1, scale=FAKE, a1=1.0, a2=1.0, om=1, ob=1, Xn=FAKE,
             nbytes=1 << 30):
        return f(FAKE, FAKE, xl, 2, Cin, 8, 8, Cout, R, S, stride, pad, 1, scale, None, None, 1, a1, a2, om, ob, Xn,
                 nbytes, None, None)

    assert call(xl=0) == E_UNSUP              # needs a bordered input
    assert call(Cin=96) == E_UNSUP            # no streaming kernel for 3 channel words
    assert call(Cout=48) == E_UNSUP
    assert call(ob=2) == E_UNSUP
    assert call(om=4) == E_UNSUP
    assert call(a1=0.0) == E_SHAPE
    assert call(scale=None) == E_NULL
    assert call(Xn=None) == E_NULL
    assert call(nbytes=64) == E_SIZE
    g = lib.fatnn_bordered_act_init
    assert g(None, 1 << 20, 2, 4, 4, 64, 1, 0, None) == E_NULL
    assert g(FAKE, 16, 2, 4, 4, 64, 1, 0, None) == E_SIZE
    assert g(FAKE, 1 << 20, 2, 4, 4, 48, 1, 0, None) == E_UNSUP
    assert g(FAKE, 1 << 20, 2, 4, 4, 64, 1, 5, None) == E_UNSUP


def test_conv_argument_errors(lib):
    f = lib.fatnn_ternary_conv2d

    def call(Wp=FAKE, Xp=FAKE, xl=0, B=2, Cin=64, H=8, W=8, Cout=16, R=3, S=3, stride=1, pad=1, mode=0, Y=FAKE,
             scale=None, bias=None, Yf=None):
        return f(Wp, Xp, xl, B, Cin, H, W, Cout, R, S, stride, pad, mode, Y, scale, bias, Yf, None)

    assert call(Cin=0) == E_SHAPE
    assert call(H=0) == E_SHAPE
    assert call(B=-1) == E_SHAPE
    assert call(R=5, S=5) == E_UNSUP
    assert call(R=3, S=1) == E_UNSUP
    assert call(stride=3) == E_UNSUP
    assert call(pad=2) == E_UNSUP
    assert call(R=1, S=1, pad=1) == E_UNSUP
    assert call(Cin=48) == E_UNSUP
    assert call(mode=7) == E_UNSUP
    assert call(xl=3) == E_UNSUP
    assert call(H=1, W=1, pad=0) == E_SHAPE            # filter larger than the padded image
    assert call(Y=None) == E_NULL
    assert call(Y=None, Yf=FAKE) == E_NULL             # fp32 output without scale
    assert call(Wp=None) == E_NULL
    assert call(Xp=None) == E_NULL
    assert call(Xp=FAKE + 4) == E_ALIGN
    assert call(B=0, Y=None) == OK
    assert call(Cout=0, Y=None) == OK
    g = lib.fatnn_twobit_conv2d
    assert g(FAKE, FAKE, 0, 2, 64, 8, 8, 16, 3, 3, 1, 1, 1, FAKE, None) == E_UNSUP     # uniform basis has no zero
    assert g(FAKE, FAKE, 0, 2, 64, 8, 8, 16, 3, 3, 1, 1, 0, None, None) == E_NULL


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "does_not_exist", "libfatnn.so"))
    with pytest.raises(FileNotFoundError):
        binding.lib()


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2008_05101_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower(), f"{fn} mentions the oracle"
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for fn in files:
            if fn.endswith((".py", ".c")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "paper_2008_05101_amd" not in text and "libfatnn.so" not in text

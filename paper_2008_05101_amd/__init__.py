"""MI355X-native ternary GEMM / convolution (FATNN, arXiv 2008.05101, Section 3.3).

Thin Python binding over the C-ABI library ``libfatnn.so`` (HIP, gfx950 only).
Importing this package does not load the library; the first call does, and it
raises if the library has not been built (``python -m paper_2008_05101_amd.build``).
There is no CPU fallback.
"""
from .binding import (  # noqa: F401
    ACT, BASIS_TERNARY, BASIS_UNIFORM, BASIS_XNOR_ONLY, NCHW, NHWC, OHWI, OIHW, RELU, ROWMAJOR_K, SYM, WEIGHT, X_BORDERED, X_BORDERED1, X_PLAIN,
    FatnnError, binary_gemm, pack_binary, bordered_act_bytes, bordered_act_init, ternary_conv2d_chain, lib, pack_ternary, pack_ternary_bordered, pack_twobit, pack_twobit_bordered,
    packed_bytes, quantize_pack, quantize_pack_bordered, set_tuning, gemm_workspace, status_str, probe_scratch, probe_valu, probe_hbm,
    PROBE_PAIR_V, PROBE_PAIR_S, PROBE_BCNT, PROBE_BITOP3, PROBE_XOR, PROBE_PAIR_LDS, HBM_READ, HBM_WRITE, HBM_COPY, ternary_conv2d, ternary_gemm, ternary_gemm_noalloc, time_next_launch,
    twobit_conv2d, twobit_gemm, weight_consts_offset, weight_interleaved_offset, words_per_row,
)

"""The paper's complexity claim (Remark 1: the ternary inner product needs half the bit operations of the
conventional two-bit form, O(2N) against O(4N)) checked on the compiled kernels: instructions per K stage
of the tiled GEMM, counted in the assembly that hipcc emits for gfx950."""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2008_05101_amd", "csrc", "tgemm.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# one K stage of the 128x128 tile: 8 k-words x (8 x 8) accumulators per lane
KT, TM, TN = 8, 8, 8


@pytest.fixture(scope="module")
def kernels():
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "tgemm.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++20", "-ffp-contract=off", "-Xclang", "-target-feature",
               "-Xclang", "-packed-fp32-ops", "--cuda-device-only", "-S", "-o", out, SRC]
        subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
        text = open(out).read()
    bodies = {}
    for m in re.finditer(r"^(_ZN5fatnn\w*plane_gemm_kernelILi(\d)ELi2ELi2ELi8ELi8ELb0ELb0EE\w*):[^\n]*\n(.*?)s_endpgm", text,
                         re.S | re.M):
        bodies[int(m.group(2))] = m.group(3)
    return bodies


def count(body, mnemonic):
    return len(re.findall(r"^\s+" + mnemonic + r"\b", body, re.M))


def test_ternary_kernel_issues_one_logic_op_and_one_popcount_per_plane_word(kernels):
    body = kernels[0]                      # OP_TERNARY
    words = KT * TM * TN * 2               # plane words per lane and stage (hi and lo)
    assert count(body, "v_bitop3_b32") == words
    assert count(body, "v_bcnt_u32_b32") == words
    # nothing else does logic on the operands: no separate xor / and instructions
    assert count(body, "v_xor_b32_e32") + count(body, "v_xor_b32_e64") + count(body, "v_and_b32_e32") < 16


def test_two_bit_kernel_needs_twice_the_operations(kernels):
    ternary, twobit = kernels[0], kernels[1]   # OP_TWOBIT_TERNARY: Eq. 2 with two planes per operand
    logic3 = count(ternary, "v_bitop3_b32")
    pop3 = count(ternary, "v_bcnt_u32_b32")
    xors = count(twobit, "v_xor_b32_e32") + count(twobit, "v_xor_b32_e64")
    pop2 = count(twobit, "v_bcnt_u32_b32")
    pairs = KT * TM * TN
    assert pop2 == 4 * pairs and xors >= 4 * pairs and xors < 4 * pairs + 16
    assert pop2 == 2 * pop3 and 4 * pairs == 2 * logic3

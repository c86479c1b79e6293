"""The binary (Eq. 1) comparison kernel and the xnor-only ablation (Eq. 4 alone) against their oracles."""
import numpy as np
import pytest
import torch

import oracle
from oracle import alg1
from test_gpu_parity import dev, DEV

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 63), (65, 63, 64), (70, 130, 65), (130, 200, 1000), (200, 300, 4609)])
def test_binary_gemm_parity(M, N, K):
    rnd = np.random.default_rng(M + N + K)
    Bw = rnd.integers(0, 2, size=(M, K), dtype=np.int8)
    Ba = rnd.integers(0, 2, size=(N, K), dtype=np.int8)
    cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
    C = fatnn.binary_gemm(fatnn.pack_binary(dev(Bw), n_invalid=cnt), fatnn.pack_binary(dev(Ba)), M, N, K)
    assert np.array_equal(C.cpu().numpy(), oracle.binary_gemm(Bw, Ba))
    assert int(cnt.item()) == 0


def test_binary_pack_counts_invalid():
    b = np.array([[0, 1, 2, -1, 1, 0, 1, 1]], np.int8)
    cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
    buf = fatnn.pack_binary(dev(b), n_invalid=cnt)
    torch.cuda.synchronize()
    assert int(cnt.item()) == 2
    assert int(buf.cpu().numpy()[:4].view(np.uint32)[0]) == 0b11010010


def test_xnor_only_gemm_and_conv():
    rnd = np.random.default_rng(5)
    code = np.array([0, 1, 3], dtype=np.int8)
    Lw = rnd.integers(0, 3, size=(20, 100), dtype=np.int8)
    La = rnd.integers(0, 3, size=(30, 100), dtype=np.int8)
    C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(code[Lw])), fatnn.pack_twobit(dev(code[La])), 20, 30, 100,
                          fatnn.BASIS_XNOR_ONLY)
    assert np.array_equal(C.cpu().numpy(), alg1.gemm_xnor_only(Lw, La))
    # larger, through the closed form pinned on the CPU: true product + #(both operands zero)
    Lw = rnd.integers(0, 3, size=(130, 1000), dtype=np.int8)
    La = rnd.integers(0, 3, size=(257, 1000), dtype=np.int8)
    C = fatnn.twobit_gemm(fatnn.pack_twobit(dev(code[Lw])), fatnn.pack_twobit(dev(code[La])), 130, 257, 1000,
                          fatnn.BASIS_XNOR_ONLY)
    both_zero = (Lw == 1).astype(np.int64) @ (La == 1).astype(np.int64).T
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0) + both_zero)
    # convolution, both kernels: zero padding is a zero operand too (codec 01)
    Lw = rnd.integers(0, 3, size=(70, 3, 3, 128), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(2, 9, 8, 128), dtype=np.int8)
    Wp = fatnn.pack_twobit(dev(code[Lw]), fatnn.WEIGHT, fatnn.OHWI)
    Xb = fatnn.pack_twobit_bordered(dev(code[Lx]), 1)
    Xp = fatnn.pack_twobit(dev(code[Lx]), fatnn.ACT, fatnn.NHWC)
    Ys = fatnn.twobit_conv2d(Wp, Xb, 2, 128, 9, 8, 70, 3, 3, 1, 1, fatnn.BASIS_XNOR_ONLY, x_layout=fatnn.X_BORDERED)
    Yt = fatnn.twobit_conv2d(Wp, Xp, 2, 128, 9, 8, 70, 3, 3, 1, 1, fatnn.BASIS_XNOR_ONLY)
    assert torch.equal(Ys, Yt)
    wz = torch.from_numpy((Lw == 1).astype(np.float64)).permute(0, 3, 1, 2)
    xz = torch.nn.functional.pad(torch.from_numpy((Lx == 1).astype(np.float64)).permute(0, 3, 1, 2), (1, 1, 1, 1),
                                 value=1.0)
    both_zero = torch.nn.functional.conv2d(xz, wz).permute(0, 2, 3, 1).numpy().astype(np.int64)
    assert np.array_equal(Ys.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, 1, 1, 0) + both_zero)

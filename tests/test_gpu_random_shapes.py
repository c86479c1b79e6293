"""Seeded random shapes: every supported combination of filter, stride, padding, channel count and
activation mode drawn at random, GPU against the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from test_gpu_parity import conv_gpu, gemm_gpu, dev, DEV

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")


def draw_conv(rnd):
    R = int(rnd.choice([1, 3]))
    stride = int(rnd.choice([1, 2]))
    pad = int(rnd.choice([0, 1])) if R == 3 else 0
    Cin = int(rnd.choice([32, 64, 96, 128, 160, 256, 512]))
    Cout = int(rnd.integers(1, 200))
    H = int(rnd.integers(R, 20))
    W = int(rnd.integers(R, 30))
    B = int(rnd.integers(1, 5))
    return B, Cin, H, W, Cout, R, stride, pad


@pytest.mark.parametrize("seed", range(24))
def test_random_conv_shapes(seed):
    rnd = np.random.default_rng(1000 + seed)
    B, Cin, H, W, Cout, R, stride, pad = draw_conv(rnd)
    mode = int(rnd.integers(0, 2))
    bordered = bool(rnd.integers(0, 2))
    p = rnd.dirichlet([1.0, 1.0, 1.0])
    Lw = rnd.choice(3, size=(Cout, R, R, Cin), p=p).astype(np.int8)
    Lx = rnd.choice(3, size=(B, H, W, Cin), p=p[::-1]).astype(np.int8)
    scale = rnd.uniform(-2.0, 2.0, Cout).astype(np.float32)
    bias = rnd.standard_normal(Cout).astype(np.float32)
    Y, Yf = conv_gpu(Lw, Lx, stride, pad, mode, bordered=bordered, scale=dev(scale), bias=dev(bias))
    want = oracle.ternary_conv2d(Lw, Lx, stride, pad, mode)
    assert np.array_equal(Y.cpu().numpy(), want), (B, Cin, H, W, Cout, R, stride, pad, mode, bordered)
    assert np.array_equal(Yf.cpu().numpy(), oracle.scale_epilogue(want, scale, bias, False))


@pytest.mark.parametrize("seed", range(24))
def test_random_gemm_shapes(seed):
    rnd = np.random.default_rng(2000 + seed)
    M = int(rnd.integers(1, 400))
    N = int(rnd.integers(1, 400))
    K = int(rnd.choice([1, 7, 31, 32, 33, 64, 100, 255, 256, 257, 1000, 2049, 5000]))
    mode = int(rnd.integers(0, 2))
    p = rnd.dirichlet([1.0, 1.0, 1.0])
    Lw = rnd.choice(3, size=(M, K), p=p).astype(np.int8)
    La = rnd.choice(3, size=(N, K), p=p[::-1]).astype(np.int8)
    scale = rnd.uniform(-2.0, 2.0, M).astype(np.float32)
    # a padded, odd row pitch: the single-element store path of the epilogue
    big = torch.full((M, N + 3), -7, dtype=torch.int32, device=DEV)
    C, Cf = gemm_gpu(Lw, La, mode, out=big[:, :N], scale=dev(scale))
    want = oracle.ternary_gemm(Lw, La, mode)
    assert np.array_equal(C.cpu().numpy(), want), (M, N, K, mode)
    assert (big[:, N:] == -7).all()
    assert np.array_equal(Cf.cpu().numpy(), oracle.scale_epilogue(want, scale, None, True))

"""Parity of the HIP path (through the C ABI) against the CPU oracle, bit-exact in
int32; the fp32 scale epilogue within 1e-6 relative (bit-equal is expected: both
sides do one correctly rounded multiply and one add)."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")

DEV = "cuda:0"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


# ----------------------------------------------------------------------------- host-side decode (test only)
def decode_packed(buf: torch.Tensor, rows: int, K: int, role: int):
    """Packed plane words -> level indices, on the host.  Weights: (s, nm) planes."""
    Kw = (K + 31) // 32
    words = buf.cpu().numpy()[: rows * Kw * 8].view(np.uint32).reshape(rows, Kw, 2)
    bits = np.unpackbits(words.view(np.uint8).reshape(rows, Kw, 2, 4), axis=-1, bitorder="little")
    bits = bits.reshape(rows, Kw, 2, 32)
    px = bits[:, :, 0, :].reshape(rows, Kw * 32)
    py = bits[:, :, 1, :].reshape(rows, Kw * 32)
    if role == fatnn.ACT:
        lv = px.astype(np.int8) + py.astype(np.int8)           # hi + lo = popcount of the codec
        assert not np.any((px == 1) & (py == 0)), "activations must spell zero as 01"
    else:
        lv = np.where(py == 0, 1, np.where(px == 1, 2, 0)).astype(np.int8)
    return lv[:, :K], lv[:, K:]


def gemm_gpu(Lw, La, mode, **kw):
    M, K = Lw.shape
    N = La.shape[0]
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    return fatnn.ternary_gemm(Wp, Ap, M, N, K, mode, **kw)


def conv_gpu(Lw, Lx, stride, pad, mode, bordered=True, **kw):
    """bordered=True: activations packed with a physical ring of value-0 pixels (streaming
    kernel where the shape allows); False: plain pixel order (tiled implicit-GEMM kernel)."""
    Cout, R, S, Cin = Lw.shape
    B, H, W, _ = Lx.shape
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT, fatnn.OHWI)
    if bordered:
        Xp = fatnn.pack_ternary_bordered(dev(Lx), pad, mode)
        return fatnn.ternary_conv2d(Wp, Xp, B, Cin, H, W, Cout, R, S, stride, pad, mode,
                                    x_layout=fatnn.X_BORDERED, **kw)
    Xp = fatnn.pack_ternary(dev(Lx), fatnn.ACT, fatnn.NHWC)
    return fatnn.ternary_conv2d(Wp, Xp, B, Cin, H, W, Cout, R, S, stride, pad, mode, **kw)


# ----------------------------------------------------------------------------- packing
@pytest.mark.parametrize("K", [1, 5, 31, 32, 33, 48, 64, 100, 576, 4609])
@pytest.mark.parametrize("role", [0, 1])
def test_pack_roundtrip(K, role):
    rnd = np.random.default_rng(K * 2 + role)
    rows = 37
    L = rnd.integers(0, 3, size=(rows, K), dtype=np.int8)
    cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
    buf = fatnn.pack_ternary(dev(L), role, n_invalid=cnt)
    torch.cuda.synchronize()
    body, tail = decode_packed(buf, rows, K, role)
    assert np.array_equal(body, L)
    assert (tail == 1).all()            # tail slots hold the value 0
    assert int(cnt.item()) == 0
    if role == fatnn.WEIGHT:
        off = fatnn.weight_consts_offset(rows, K)
        consts = buf.cpu().numpy()[off: off + rows * 8].view(np.int32)
        assert np.array_equal(consts[:rows], (L != 1).sum(axis=1))
        assert np.array_equal(consts[rows:], (L == 2).sum(axis=1))


def test_pack_counts_invalid_levels_and_packs_them_as_zero():
    rnd = np.random.default_rng(9)
    L = rnd.integers(0, 3, size=(16, 96), dtype=np.int8)
    bad = [(0, 0, 3), (3, 17, -1), (7, 95, 77), (15, 40, -128), (15, 41, 4)]
    Lb = L.copy()
    for r, k, v in bad:
        Lb[r, k] = v
        L[r, k] = 1
    for role in (0, 1):
        cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
        buf = fatnn.pack_ternary(dev(Lb), role, n_invalid=cnt)
        torch.cuda.synchronize()
        assert int(cnt.item()) == len(bad)
        body, _ = decode_packed(buf, 16, 96, role)
        assert np.array_equal(body, L)


def test_check_levels_raises_err_level():
    """First constraint of Section 3.3: an input outside the level set is an error the binding can raise."""
    rnd = np.random.default_rng(19)
    L = rnd.integers(0, 3, size=(8, 64), dtype=np.int8)
    for role in (0, 1):
        fatnn.pack_ternary(dev(L), role, check_levels=True)                    # clean input: no error
    Lb = L.copy()
    Lb[2, 7] = 3
    with pytest.raises(fatnn.FatnnError) as e:
        fatnn.pack_ternary(dev(Lb), fatnn.ACT, check_levels=True)
    assert e.value.status == -3
    # a caller's own counter keeps counting; only this call's increment decides
    cnt = torch.full((1,), 5, dtype=torch.int32, device=DEV)
    fatnn.pack_ternary(dev(L), fatnn.ACT, n_invalid=cnt, check_levels=True)
    with pytest.raises(fatnn.FatnnError):
        fatnn.pack_ternary(dev(Lb), fatnn.WEIGHT, n_invalid=cnt, check_levels=True)
    assert int(cnt.item()) == 6
    x4 = rnd.integers(0, 3, size=(1, 4, 4, 32), dtype=np.int8)
    x4[0, 1, 2, 3] = -1
    with pytest.raises(fatnn.FatnnError):
        fatnn.pack_ternary_bordered(dev(x4), 1, fatnn.RELU, check_levels=True)
    xf = rnd.standard_normal((4, 64)).astype(np.float32)
    fatnn.quantize_pack(dev(xf), fatnn.ACT, fatnn.RELU, 0.7, 0.9, check_levels=True)
    xf[0, 0] = np.nan
    with pytest.raises(fatnn.FatnnError):
        fatnn.quantize_pack(dev(xf), fatnn.ACT, fatnn.RELU, 0.7, 0.9, check_levels=True)


def test_pack_layouts_agree():
    rnd = np.random.default_rng(10)
    w = rnd.integers(0, 3, size=(6, 3, 3, 64), dtype=np.int8)          # OHWI
    a = fatnn.pack_ternary(dev(w), fatnn.WEIGHT, fatnn.OHWI)
    b = fatnn.pack_ternary(dev(np.ascontiguousarray(w.transpose(0, 3, 1, 2))), fatnn.WEIGHT, fatnn.OIHW)
    nwords = 6 * (9 * 64 // 32) * 8                      # the alignment gap before the constants is not written
    off = fatnn.weight_consts_offset(6, 9 * 64)
    assert torch.equal(a[:nwords], b[:nwords])
    assert torch.equal(a[off:off + 6 * 8], b[off:off + 6 * 8])
    x = rnd.integers(0, 3, size=(2, 5, 7, 32), dtype=np.int8)          # NHWC
    a = fatnn.pack_ternary(dev(x), fatnn.ACT, fatnn.NHWC)
    b = fatnn.pack_ternary(dev(np.ascontiguousarray(x.transpose(0, 3, 1, 2))), fatnn.ACT, fatnn.NCHW)
    assert torch.equal(a, b)
    c = fatnn.pack_ternary(dev(x.reshape(-1, 32)), fatnn.ACT, fatnn.ROWMAJOR_K)
    assert torch.equal(a, c)


# ----------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M,N,K", [
    (1, 1, 1), (3, 5, 31), (64, 64, 32), (65, 63, 33), (7, 200, 65), (130, 70, 257),
    (128, 128, 256), (129, 257, 300), (200, 1000, 1000), (64, 1500, 96),
])
@pytest.mark.parametrize("mode", [0, 1])
def test_gemm_parity_small_and_ragged(M, N, K, mode):
    rnd = np.random.default_rng(M * 7 + N * 3 + K + mode)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    C, _ = gemm_gpu(Lw, La, mode)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, mode))


@pytest.mark.parametrize("M,N,K", [(2048, 2100, 96), (64, 70000, 64), (2100, 1100, 130), (4096, 8, 300),
                                   (8200, 8300, 40), (64, 1100000, 33)])
def test_gemm_parity_every_workgroup_shape(M, N, K):
    # from a few to more than 16 K tiles of 64x64: the 32x32, 64x64 and 128x128 workgroup shapes, and the
    # one-row-block case that stays on a small shape however many tiles there are
    rnd = np.random.default_rng(M + N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    C, _ = gemm_gpu(Lw, La, 1)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 1))


@pytest.mark.parametrize("M,N,K", [(64, 64, 2048), (130, 70, 2100), (200, 300, 2049), (512, 700, 2304), (9, 1000, 4609)])
@pytest.mark.parametrize("mode", [0, 1])
def test_gemm_parity_few_tiles_long_k(M, N, K, mode):
    # few tiles and a long K (the 32x32 workgroup tile, many K stages)
    rnd = np.random.default_rng(M + 3 * N + K + mode)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale = si.scale_vec(rnd, M)
    C, Cf = gemm_gpu(Lw, La, mode, scale=dev(scale))
    want = oracle.ternary_gemm(Lw, La, mode)
    assert np.array_equal(C.cpu().numpy(), want)
    assert np.array_equal(Cf.cpu().numpy(), oracle.scale_epilogue(want, scale, None, True))
    # the conventional two-bit form through the same workgroup shape
    code = np.array([0, 1, 3], np.int8)
    W2 = fatnn.pack_twobit(dev(code[Lw]), fatnn.WEIGHT)
    A2 = fatnn.pack_twobit(dev(code[La]), fatnn.ACT)
    C2 = fatnn.twobit_gemm(W2, A2, M, N, K, 0)
    assert np.array_equal(C2.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))


@pytest.mark.parametrize("M,N,K", [(3, 5, 100003), (70, 9, 262144 + 17), (2, 40, 1 << 20)])
def test_gemm_parity_very_long_k(M, N, K):
    # thousands of K stages per tile; all-(+1) rows and columns make the sums reach +-K and 2K
    rnd = np.random.default_rng(K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    Lw[0, :] = 2
    La[0, :] = 2
    La[1, :] = 0
    for mode in (0, 1):
        C, _ = gemm_gpu(Lw, La, mode)
        want = oracle.ternary_gemm(Lw, La, mode)
        assert np.array_equal(C.cpu().numpy(), want)
        assert want[0, 0] == (K if mode == 0 else 2 * K) and want[0, 1] == (-K if mode == 0 else 0)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 5, 7, 8, 9, 13, 16])
@pytest.mark.parametrize("mode", [0, 1])
def test_skinny_gemm_parity(N, mode):
    # (the matrix-vector kernel serves N <= 4, and N <= 8 with K < 2048; the rest goes to the K-splitting or tiled kernel)
    rnd = np.random.default_rng(N * 3 + mode)
    for M, K in [(1, 1), (5, 33), (130, 4609), (1027, 200), (70, 8200)]:
        Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
        La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
        scale = si.scale_vec(rnd, M)
        bias = si.bias_vec(rnd, M)
        big = torch.full((M, N + 3), -5, dtype=torch.int32, device=DEV)
        C, Cf = gemm_gpu(Lw, La, mode, out=big[:, :N], scale=dev(scale), bias=dev(bias))
        want = oracle.ternary_gemm(Lw, La, mode)
        assert np.array_equal(C.cpu().numpy(), want)
        assert (big[:, N:] == -5).all()
        assert np.array_equal(Cf.cpu().numpy(), oracle.scale_epilogue(want, scale, bias, True))


@pytest.mark.parametrize("mode", [0, 1])
def test_gemm_cfg1(mode):
    case = si.cfg1()
    Lw, La = case.make()
    C, _ = gemm_gpu(Lw, La, mode)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, mode))


def test_gemm_degenerate_operands():
    K = 777
    for lw, la, mode, want in [(2, 2, 0, K), (2, 0, 0, -K), (1, 2, 0, 0), (2, 1, 0, 0), (2, 2, 1, 2 * K),
                               (0, 2, 1, -2 * K), (2, 0, 1, 0)]:
        Lw = np.full((70, K), lw, np.int8)
        La = np.full((66, K), la, np.int8)
        C, _ = gemm_gpu(Lw, La, mode)
        assert (C.cpu().numpy() == want).all()


def test_gemm_accepts_the_other_spelling_of_zero():
    # Table 1 allows 10 as well as 01 for the value 0: hand-pack activations with 10.
    rnd = np.random.default_rng(12)
    M, N, K = 33, 40, 96
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    Ap = fatnn.pack_ternary(dev(La), fatnn.ACT)
    words = Ap.cpu().numpy().view(np.uint32).reshape(N, K // 32, 2).copy()
    hi, lo = words[:, :, 0], words[:, :, 1]
    zero = ~hi & lo
    flip = zero & np.uint32(0xA5A5F00F)          # respell some zeros as 10
    words[:, :, 0] = hi | flip
    words[:, :, 1] = lo & ~flip
    Ap2 = torch.from_numpy(words.view(np.uint8).reshape(-1)).to(DEV)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    C, _ = fatnn.ternary_gemm(Wp, Ap2, M, N, K, fatnn.SYM)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))


def test_gemm_empty_and_strided_output():
    Lw = np.ones((4, 40), np.int8)
    La = np.ones((0, 40), np.int8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT)
    Ap = torch.empty(16, dtype=torch.uint8, device=DEV)
    C, _ = fatnn.ternary_gemm(Wp, Ap, 4, 0, 40)
    assert C.shape == (4, 0)
    rnd = np.random.default_rng(1)
    Lw = rnd.integers(0, 3, size=(10, 70), dtype=np.int8)
    La = rnd.integers(0, 3, size=(20, 70), dtype=np.int8)
    big = torch.full((10, 32), -7, dtype=torch.int32, device=DEV)
    out = big[:, :20]
    gemm_gpu(Lw, La, 0, out=out)
    assert np.array_equal(out.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))
    assert (big[:, 20:] == -7).all()


def test_gemm_scale_epilogue():
    rnd = np.random.default_rng(14)
    M, N, K = 70, 90, 500
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale = si.scale_vec(rnd, M)
    bias = si.bias_vec(rnd, M)
    C = oracle.ternary_gemm(Lw, La, 1)
    for b in (None, bias):
        Ci, Cf = gemm_gpu(Lw, La, 1, scale=dev(scale), bias=None if b is None else dev(b))
        assert np.array_equal(Ci.cpu().numpy(), C)
        want = oracle.scale_epilogue(C, scale, b, channel_is_row=True)
        got = Cf.cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=1e-6, atol=0)
        assert np.array_equal(got, want)
    # fp32 only (no int32 output)
    Ci, Cf = gemm_gpu(Lw, La, 1, scale=dev(scale), want_int=False)
    assert Ci is None
    assert np.array_equal(Cf.cpu().numpy(), oracle.scale_epilogue(C, scale, None, True))


def test_gemm_operands_beyond_4_gib():
    """Packed operands larger than 4 GiB in either role (2^20 + 77 rows of K = 16416): the kernels address a
    tile's rows from a 64-bit tile base with 32-bit offsets, the packing kernels with 64-bit indices.  Outputs
    are compared with the oracle on columns / rows from both ends and the middle of the big operand."""
    M, N, K = 48, (1 << 20) + 77, 16384 + 32
    g = torch.Generator(device=DEV).manual_seed(5)
    La = torch.randint(0, 3, (N, K), dtype=torch.int8, device=DEV, generator=g)
    Lw = torch.randint(0, 3, (M, K), dtype=torch.int8, device=DEV, generator=g)
    Lw_h = Lw.cpu().numpy()
    pick = torch.from_numpy(np.concatenate([np.arange(0, 40), np.arange(N // 2 - 20, N // 2 + 20),
                                            np.arange(N - 100, N)])).to(DEV)
    La_h = La[pick].cpu().numpy()
    Ap = fatnn.pack_ternary(La, fatnn.ACT)
    assert Ap.numel() > (1 << 32)
    Wp = fatnn.pack_ternary(Lw, fatnn.WEIGHT)
    for mode in (0, 1):
        C, _ = fatnn.ternary_gemm(Wp, Ap, M, N, K, mode)
        assert np.array_equal(C[:, pick].cpu().numpy(), oracle.ternary_gemm(Lw_h, La_h, mode))
    del Ap, C
    Wbig = fatnn.pack_ternary(La, fatnn.WEIGHT)
    del La
    Asmall = fatnn.pack_ternary(Lw, fatnn.ACT)
    C, _ = fatnn.ternary_gemm(Wbig, Asmall, N, M, K, 0)
    assert np.array_equal(C[pick].cpu().numpy(), oracle.ternary_gemm(La_h, Lw_h, 0))
    del Wbig, C
    torch.cuda.empty_cache()


@pytest.mark.parametrize("bordered", [True, False])
def test_conv_output_beyond_4_gib(bordered):
    """A 1x1 convolution whose int32 output is 4.5 GB (batch 1400 of 56 x 56 x 64 -> 256): the streaming kernel
    addresses its output with 32-bit offsets, so the call must go to the tiled kernel (64-bit output
    addressing) whatever the input layout.  Three images are compared with the oracle."""
    B, Cin, Cout, H, W = 1400, 64, 256, 56, 56
    g = torch.Generator(device=DEV).manual_seed(9)
    Lx = torch.randint(0, 3, (B, H, W, Cin), dtype=torch.int8, device=DEV, generator=g)
    Lw = torch.randint(0, 3, (Cout, 1, 1, Cin), dtype=torch.int8, device=DEV, generator=g)
    Wp = fatnn.pack_ternary(Lw, fatnn.WEIGHT, fatnn.OHWI)
    if bordered:
        Xp = fatnn.pack_ternary_bordered(Lx, 0, 1)
        Y, _ = fatnn.ternary_conv2d(Wp, Xp, B, Cin, H, W, Cout, 1, 1, 1, 0, 1, x_layout=fatnn.X_BORDERED)
    else:
        Xp = fatnn.pack_ternary(Lx, fatnn.ACT, fatnn.NHWC)
        Y, _ = fatnn.ternary_conv2d(Wp, Xp, B, Cin, H, W, Cout, 1, 1, 1, 0, 1)
    assert Y.numel() * 4 > (1 << 32)
    Lw_h = Lw.cpu().numpy()
    for b in (0, 700, B - 1):
        want = oracle.ternary_conv2d(Lw_h, Lx[b:b + 1].cpu().numpy(), 1, 0, 1)
        assert np.array_equal(Y[b:b + 1].cpu().numpy(), want)
    del Y, Xp, Lx
    torch.cuda.empty_cache()


def unusual_coefficients(rnd, M):
    """Scale and bias vectors with negative, zero, denormal, huge, infinite and NaN entries."""
    scale = si.scale_vec(rnd, M)
    bias = si.bias_vec(rnd, M)
    scale[0:4] *= -1.0
    scale[4] = 0.0
    scale[5] = -0.0
    scale[6] = np.float32(1e-42)
    scale[7] = np.float32(3e38)
    scale[8] = np.inf
    scale[9] = -np.inf
    scale[10] = np.nan
    bias[6] = 0.0
    bias[8] = -np.inf
    bias[12] = np.inf
    bias[13] = np.nan
    bias[14] = np.float32(-3e38)
    return scale, bias


@pytest.mark.parametrize("M,N,K", [(70, 90, 500),         # tiled kernel
                                   (64, 3, 4608),         # matrix-vector kernel
                                   (96, 40, 4096),        # K-splitting kernel
                                   (128, 512, 8192)])     # even shares (hand-over before the epilogue)
def test_gemm_scale_epilogue_unusual_coefficients(M, N, K):
    """The fp32 epilogue is float32 multiply-then-add for every float it is given (the paper fixes one positive
    scale; the library does not check it): equal to the oracle bit for bit, NaN for NaN."""
    rnd = np.random.default_rng(M + N + K)
    Lw = rnd.integers(0, 3, size=(M, K), dtype=np.int8)
    La = rnd.integers(0, 3, size=(N, K), dtype=np.int8)
    scale, bias = unusual_coefficients(rnd, M)
    C = oracle.ternary_gemm(Lw, La, 0)
    with np.errstate(all="ignore"):
        want = oracle.scale_epilogue(C, scale, bias, channel_is_row=True)
    Ci, Cf = gemm_gpu(Lw, La, 0, scale=dev(scale), bias=dev(bias))
    assert np.array_equal(Ci.cpu().numpy(), C)
    assert np.array_equal(Cf.cpu().numpy(), want, equal_nan=True)


@pytest.mark.parametrize("bordered", [True, False])
def test_conv_scale_epilogue_unusual_coefficients(bordered):
    rnd = np.random.default_rng(31 + bordered)
    B, Cin, Cout, H, W = 2, 64, 64, 7, 9
    Lw = rnd.integers(0, 3, size=(Cout, 3, 3, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(B, H, W, Cin), dtype=np.int8)
    scale, bias = unusual_coefficients(rnd, Cout)
    Y = oracle.ternary_conv2d(Lw, Lx, 1, 1, 1)
    with np.errstate(all="ignore"):
        want = oracle.scale_epilogue(Y, scale, bias, channel_is_row=False)
    Yi, Yf = conv_gpu(Lw, Lx, 1, 1, 1, bordered=bordered, scale=dev(scale), bias=dev(bias))
    assert np.array_equal(Yi.cpu().numpy(), Y)
    assert np.array_equal(Yf.cpu().numpy(), want, equal_nan=True)


# ----------------------------------------------------------------------------- convolution
@pytest.mark.parametrize("Cin,Cout,H,W,R,stride,pad", [
    (32, 5, 6, 7, 3, 1, 1), (64, 64, 9, 9, 3, 1, 1), (64, 70, 12, 10, 3, 2, 1), (96, 33, 8, 8, 3, 1, 1),
    (64, 128, 14, 14, 1, 2, 0), (256, 64, 7, 9, 1, 1, 0), (32, 16, 5, 5, 3, 1, 0), (128, 130, 7, 7, 3, 1, 1),
    (256, 200, 9, 6, 3, 2, 1), (512, 64, 5, 5, 3, 1, 1), (512, 300, 6, 6, 1, 1, 0), (128, 1, 4, 4, 3, 1, 1),
    (64, 64, 1, 1, 1, 1, 0), (64, 64, 2, 1, 3, 1, 1), (128, 64, 30, 3, 3, 2, 1),
])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("bordered", [True, False])
def test_conv_parity_small(Cin, Cout, H, W, R, stride, pad, mode, bordered):
    rnd = np.random.default_rng(Cin + Cout + H + R + stride + mode)
    B = 3
    Lw = rnd.integers(0, 3, size=(Cout, R, R, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(B, H, W, Cin), dtype=np.int8)
    Y, _ = conv_gpu(Lw, Lx, stride, pad, mode, bordered=bordered)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, stride, pad, mode))


@pytest.mark.parametrize("Cin,Cout,H,W", [(256, 64, 7, 7), (256, 130, 9, 14), (512, 64, 7, 7), (512, 200, 5, 14),
                                          (256, 64, 3, 21), (128, 128, 6, 28), (128, 70, 7, 7)])
@pytest.mark.parametrize("mode", [0, 1])
def test_conv_parity_groups_of_seven(tuning, Cin, Cout, H, W, mode):
    """The seven-pixel-group kernels (normally chosen only for large batches) on small inputs."""
    tuning(seven_pixel_groups=2)
    rnd = np.random.default_rng(Cin + Cout + H + W + mode)
    Lw = rnd.integers(0, 3, size=(Cout, 3, 3, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(5, H, W, Cin), dtype=np.int8)
    scale = rnd.uniform(0.5, 1.5, Cout).astype(np.float32)
    bias = rnd.standard_normal(Cout).astype(np.float32)
    Y, Yf = conv_gpu(Lw, Lx, 1, 1, mode, bordered=True, scale=dev(scale), bias=dev(bias))
    want = oracle.ternary_conv2d(Lw, Lx, 1, 1, mode)
    assert np.array_equal(Y.cpu().numpy(), want)
    assert np.array_equal(Yf.cpu().numpy(), oracle.scale_epilogue(want, scale, bias, False))


@pytest.mark.parametrize("Cin,Cout,H,W,R,stride,pad", [(64, 70, 12, 10, 3, 2, 1), (128, 130, 7, 7, 3, 1, 1),
                                                       (64, 128, 14, 14, 1, 2, 0), (256, 64, 7, 9, 1, 1, 0)])
@pytest.mark.parametrize("mode", [0, 1])
def test_conv_bordered_input_on_the_tiled_kernel(tuning, Cin, Cout, H, W, R, stride, pad, mode):
    """The fallback that serves bordered inputs the streaming kernel cannot take (tensors of 4 GiB and
    more): the LDS-tiled kernel reading the bordered layout, forced here on small inputs."""
    tuning(conv_kernel=1)
    rnd = np.random.default_rng(Cin + Cout + H + R + stride + mode + 1)
    Lw = rnd.integers(0, 3, size=(Cout, R, R, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(3, H, W, Cin), dtype=np.int8)
    Y, _ = conv_gpu(Lw, Lx, stride, pad, mode, bordered=True)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, stride, pad, mode))


@pytest.mark.parametrize("Cin,Cout,H,W", [(128, 256, 9, 14), (128, 70, 14, 28), (256, 512, 6, 14), (256, 130, 14, 13)])
@pytest.mark.parametrize("mode", [0, 1])
def test_conv_stride2_groups_of_seven(tuning, Cin, Cout, H, W, mode):
    """Stride-2 3x3 layers with seven-pixel groups (output rows of 7: W = 13 or 14; 14: W = 28), forced on small inputs."""
    tuning(seven_pixel_groups=2)
    rnd = np.random.default_rng(Cin + Cout + H + W + mode)
    Lw = rnd.integers(0, 3, size=(Cout, 3, 3, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(4, H, W, Cin), dtype=np.int8)
    Y, _ = conv_gpu(Lw, Lx, 2, 1, mode, bordered=True)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, 2, 1, mode))


@pytest.mark.parametrize("Cout", [1, 64, 65, 256, 300, 512, 530])
@pytest.mark.parametrize("stride", [1, 2])
def test_conv_512_channels_wavefront_pairs(Cout, stride):
    """3x3 over 512 channels: two wavefronts per row block split K and meet in LDS once per group; the number of
    row blocks decides how many wavefronts of a workgroup are surplus."""
    rnd = np.random.default_rng(Cout + stride)
    Lw = rnd.integers(0, 3, size=(Cout, 3, 3, 512), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(3, 9, 11, 512), dtype=np.int8)
    scale = rnd.uniform(0.5, 1.5, Cout).astype(np.float32)
    for mode in (0, 1):
        Y, Yf = conv_gpu(Lw, Lx, stride, 1, mode, bordered=True, scale=dev(scale))
        want = oracle.ternary_conv2d(Lw, Lx, stride, 1, mode)
        assert np.array_equal(Y.cpu().numpy(), want)
        assert np.array_equal(Yf.cpu().numpy(), oracle.scale_epilogue(want, scale, None, False))


def test_bordered_pack_layout():
    rnd = np.random.default_rng(77)
    B, H, W, C = 2, 5, 4, 64
    Lx = rnd.integers(0, 3, size=(B, H, W, C), dtype=np.int8)
    plain = fatnn.pack_ternary(dev(Lx), fatnn.ACT, fatnn.NHWC).cpu().numpy().view(np.uint32).reshape(B, H, W, 2, 2)
    for mode, ring in ((0, (0, 0xFFFFFFFF)), (1, (0, 0))):
        buf = fatnn.pack_ternary_bordered(dev(Lx), 1, mode)
        assert buf.numel() == fatnn.bordered_act_bytes(B, H, W, C, 1)
        words = buf.cpu().numpy().view(np.uint32)
        body = words[: B * (H + 2) * (W + 2) * 4].reshape(B, H + 2, W + 2, 2, 2)
        assert np.array_equal(body[:, 1:-1, 1:-1], plain)
        mask = np.ones((H + 2, W + 2), bool)
        mask[1:-1, 1:-1] = False
        assert (body[:, mask][..., 0] == ring[0]).all() and (body[:, mask][..., 1] == ring[1]).all()
        slack = words[B * (H + 2) * (W + 2) * 4:].reshape(-1, 2)
        assert slack.shape[0] == 64 * 2 and (slack[:, 0] == ring[0]).all() and (slack[:, 1] == ring[1]).all()
    # border 0 = plain order plus slack
    b0 = fatnn.pack_ternary_bordered(dev(Lx), 0, 0).cpu().numpy().view(np.uint32)
    assert np.array_equal(b0[: plain.size], plain.reshape(-1))


def test_conv_cfg2_full_with_scale_epilogue():
    case = si.cfg2()
    Lw, Lx = case.make()
    scale, bias = case.make_scale_bias()
    Y, Yf = conv_gpu(Lw, Lx, 1, 1, case.act_mode, scale=dev(scale), bias=dev(bias))
    want = oracle.ternary_conv2d(Lw, Lx, 1, 1, case.act_mode)
    assert np.array_equal(Y.cpu().numpy(), want)
    wantf = oracle.scale_epilogue(want, scale, bias, channel_is_row=False)
    np.testing.assert_allclose(Yf.cpu().numpy(), wantf, rtol=1e-6, atol=0)
    assert np.array_equal(Yf.cpu().numpy(), wantf)
    Ys, _ = conv_gpu(Lw, Lx, 1, 1, fatnn.SYM)
    assert np.array_equal(Ys.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, 1, 1, 0))
    Yt, Ytf = conv_gpu(Lw, Lx, 1, 1, case.act_mode, bordered=False, scale=dev(scale), bias=dev(bias))
    assert np.array_equal(Yt.cpu().numpy(), want) and np.array_equal(Ytf.cpu().numpy(), wantf)


@pytest.mark.parametrize("layer", range(19))
@pytest.mark.parametrize("bordered", [True, False])
def test_conv_cfg3_layers_batch4(layer, bordered):
    case = si.cfg3(batch=4)[layer]
    Lw, Lx = case.make()
    Y, _ = conv_gpu(Lw, Lx, case.stride, case.pad, case.act_mode, bordered=bordered)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, case.stride, case.pad, case.act_mode))


@pytest.mark.parametrize("layer", range(19))
def test_conv_cfg3_layers_batch64_every_element(layer):
    # the launch configuration bench.py times: batch 64, bordered input, every output of every layer
    case = si.cfg3(batch=64)[layer]
    Lw, Lx = case.make()
    Y, _ = conv_gpu(Lw, Lx, case.stride, case.pad, case.act_mode)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, case.stride, case.pad, case.act_mode))


@pytest.mark.parametrize("layer", [1, 6, 12, 17])
def test_conv_cfg3_layers_batch64_tiled_kernel_every_element(layer):
    # the same through the LDS-tiled kernel's implicit-im2col front end (plain packed input)
    case = si.cfg3(batch=64)[layer]
    Lw, Lx = case.make()
    Y, _ = conv_gpu(Lw, Lx, case.stride, case.pad, case.act_mode, bordered=False)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, case.stride, case.pad, case.act_mode))


@pytest.mark.parametrize("idx", [0, 1])
def test_conv_cfg5_bottleneck_1x1_every_image(idx):
    case = si.cfg5_bottleneck()[idx]
    Lw, Lx = case.make()
    Y, _ = conv_gpu(Lw, Lx, 1, 0, case.act_mode)
    Y = Y.cpu().numpy()
    assert np.array_equal(Y, oracle.ternary_conv2d(Lw, Lx, 1, 0, case.act_mode))
    # a 1x1 convolution is the GEMM over pixels
    C, _ = gemm_gpu(Lw.reshape(case.Cout, case.Cin), Lx[:2].reshape(-1, case.Cin), case.act_mode)
    assert np.array_equal(C.cpu().numpy().T, Y[:2].reshape(-1, case.Cout))


# ----------------------------------------------------------------------------- the large and the ragged GEMMs
def test_gemm_cfg5_ragged_k4609_full():
    case = si.cfg5_ragged()
    Lw, La = case.make()
    C, _ = gemm_gpu(Lw, La, 0)
    assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))


def test_gemv_cfg5_full():
    case = si.cfg5_gemv()
    Lw, La = case.make()
    for mode in (0, 1):
        C, _ = gemm_gpu(Lw, La, mode)
        assert np.array_equal(C.cpu().numpy(), oracle.ternary_gemm(Lw, La, mode))


def test_gemm_cfg4_full_size_every_element():
    # 8192^3 on the seeded operands bench.py times; the oracle needs a few tens of seconds for all
    # 67 million outputs (it is cut into row blocks so that a progress line appears for each)
    case = si.cfg4()
    Lw, La = case.make()
    C, _ = gemm_gpu(Lw, La, 0)
    C = C.cpu().numpy()
    step = 1024
    for r0 in range(0, case.M, step):
        want = oracle.ternary_gemm(np.ascontiguousarray(Lw[r0:r0 + step]), La, 0)
        assert np.array_equal(C[r0:r0 + step], want), f"rows {r0}..{r0 + step - 1}"
        print(f"cfg4 rows {r0}..{r0 + step - 1} equal", flush=True)


# ----------------------------------------------------------------------------- conventional two-bit path
@pytest.mark.parametrize("M,N,K", [(3, 5, 31), (65, 63, 33), (130, 70, 257), (200, 300, 1000)])
@pytest.mark.parametrize("basis", [0, 1])
def test_twobit_gemm_parity(M, N, K, basis):
    rnd = np.random.default_rng(M + N + K + basis)
    Qw = rnd.integers(0, 4, size=(M, K), dtype=np.int8)
    Qa = rnd.integers(0, 4, size=(N, K), dtype=np.int8)
    Wp = fatnn.pack_twobit(dev(Qw))
    Ap = fatnn.pack_twobit(dev(Qa))
    C = fatnn.twobit_gemm(Wp, Ap, M, N, K, basis)
    assert np.array_equal(C.cpu().numpy(), oracle.twobit_gemm(Qw, Qa, basis))


def test_twobit_on_ternary_data_equals_ternary_path():
    case = si.cfg1()
    Lw, La = case.make()
    code = np.array([0, 1, 3], dtype=np.int8)
    Wp = fatnn.pack_twobit(dev(code[Lw]))
    Ap = fatnn.pack_twobit(dev(code[La]))
    C2 = fatnn.twobit_gemm(Wp, Ap, case.M, case.N, case.K, fatnn.BASIS_TERNARY)
    C3, _ = gemm_gpu(Lw, La, 0)
    assert torch.equal(C2, C3)
    assert np.array_equal(C2.cpu().numpy(), oracle.ternary_gemm(Lw, La, 0))


@pytest.mark.parametrize("R,stride,pad,Cin", [(3, 1, 1, 64), (3, 2, 1, 64), (1, 1, 0, 64), (3, 1, 1, 96), (3, 1, 1, 256),
                                              (3, 1, 1, 512), (3, 2, 1, 512), (1, 1, 0, 512)])
def test_twobit_conv_parity(R, stride, pad, Cin):
    rnd = np.random.default_rng(R + stride + Cin)
    Lw = rnd.integers(0, 3, size=(70, R, R, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(3, 10, 9, Cin), dtype=np.int8)
    code = np.array([0, 1, 3], dtype=np.int8)
    Wp = fatnn.pack_twobit(dev(code[Lw]), fatnn.WEIGHT, fatnn.OHWI)
    Xp = fatnn.pack_twobit(dev(code[Lx]), fatnn.ACT, fatnn.NHWC)
    Y = fatnn.twobit_conv2d(Wp, Xp, 3, Cin, 10, 9, 70, R, R, stride, pad)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, stride, pad, 0))
    Xb = fatnn.pack_twobit_bordered(dev(code[Lx]), pad)
    Yb = fatnn.twobit_conv2d(Wp, Xb, 3, Cin, 10, 9, 70, R, R, stride, pad, x_layout=fatnn.X_BORDERED)
    assert torch.equal(Y, Yb)

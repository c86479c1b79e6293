"""Layer-chaining epilogue (conv -> affine -> skip -> ReLU -> next quantizer -> packed bordered
input of the next layer) against the composed oracle; exact."""
import numpy as np
import pytest
import torch

import oracle
from oracle import chain as ochain
from test_gpu_parity import dev, DEV

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")


def decode_bordered(buf, B, H, W, C, border):
    """Bordered packed activations -> (levels of the interior NHWC, ring words, slack words)."""
    Cw = C // 32
    Hp, Wp = H + 2 * border, W + 2 * border
    words = buf.cpu().numpy().view(np.uint32)
    body = words[: B * Hp * Wp * Cw * 2].reshape(B, Hp, Wp, Cw, 2)
    slack = words[B * Hp * Wp * Cw * 2:].reshape(-1, 2)
    bits = np.unpackbits(body.view(np.uint8).reshape(B, Hp, Wp, Cw, 2, 4), axis=-1, bitorder="little")
    bits = bits.reshape(B, Hp, Wp, Cw, 2, 32)
    lv = (bits[..., 0, :].astype(np.int8) + bits[..., 1, :].astype(np.int8)).reshape(B, Hp, Wp, C)
    assert not np.any((bits[..., 0, :] == 1) & (bits[..., 1, :] == 0))
    mask = np.ones((Hp, Wp), bool)
    if border:
        mask[border:-border, border:-border] = False
        interior = lv[:, border:-border, border:-border]
    else:
        mask[:] = False
        interior = lv
    return interior, body[:, mask], slack


CASES = [
    # Cin, Cout, H, W, R, stride, pad, in_mode, out_mode, out_border, skip, relu
    (128, 128, 9, 8, 3, 1, 1, 1, 1, 1, False, False),
    (64, 64, 12, 12, 3, 1, 1, 1, 1, 1, True, True),
    (64, 128, 10, 10, 3, 2, 1, 1, 1, 1, False, True),
    (256, 96, 6, 7, 3, 1, 1, 0, 0, 1, True, False),
    (256, 64, 7, 5, 1, 1, 0, 1, 1, 0, True, True),
    (64, 256, 8, 8, 1, 2, 0, 1, 0, 1, False, False),
    (512, 128, 5, 5, 3, 1, 1, 1, 1, 1, True, True),
    (128, 32, 6, 6, 3, 1, 1, 1, 1, 0, False, True),
]


@pytest.mark.parametrize("Cin,Cout,H,W,R,stride,pad,in_mode,out_mode,out_border,use_skip,relu", CASES)
def test_chain_epilogue_exact(Cin, Cout, H, W, R, stride, pad, in_mode, out_mode, out_border, use_skip, relu):
    rnd = np.random.default_rng(Cin + Cout + H + R + stride)
    B = 3
    Lw = rnd.integers(0, 3, size=(Cout, R, R, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(B, H, W, Cin), dtype=np.int8)
    C = oracle.ternary_conv2d(Lw, Lx, stride, pad, in_mode)
    Ho, Wo = C.shape[1], C.shape[2]
    std = float(C.std()) + 1.0
    scale = (rnd.uniform(0.5, 1.5, Cout) / std).astype(np.float32)
    bias = (rnd.standard_normal(Cout) * 0.3).astype(np.float32)
    skip = (rnd.standard_normal((B, Ho, Wo, Cout)) * 0.5).astype(np.float32) if use_skip else None
    a1, a2 = 0.6, 0.8
    f_want, lv_want = ochain.chain_epilogue(C, scale, bias, skip, relu, out_mode, a1, a2)

    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT, fatnn.OHWI)
    Xp = fatnn.pack_ternary_bordered(dev(Lx), pad, in_mode)
    Xn = fatnn.bordered_act_init(B, Ho, Wo, Cout, out_border, out_mode, device=DEV)
    Yf = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=DEV)
    fatnn.ternary_conv2d_chain(Wp, Xp, B, Cin, H, W, Cout, R, R, stride, pad, in_mode, dev(scale), dev(bias),
                               None if skip is None else dev(skip), relu, a1, a2, out_mode, out_border, Xn, out_f=Yf)
    torch.cuda.synchronize()
    assert np.array_equal(Yf.cpu().numpy(), f_want)
    interior, ring, slack = decode_bordered(Xn, B, Ho, Wo, Cout, out_border)
    assert np.array_equal(interior, lv_want)
    zero_word = (0, 0xFFFFFFFF) if out_mode == 0 else (0, 0)
    assert (ring[..., 0] == zero_word[0]).all() and (ring[..., 1] == zero_word[1]).all()
    assert (slack[:, 0] == zero_word[0]).all() and (slack[:, 1] == zero_word[1]).all()
    # the chained buffer is byte-identical to packing the oracle's levels
    ref = fatnn.pack_ternary_bordered(dev(lv_want), out_border, out_mode)
    assert torch.equal(Xn, ref)


@pytest.mark.parametrize("Cin,Cout,H,W,use_skip", [(256, 256, 7, 7, True), (256, 96, 6, 14, False),
                                                   (512, 128, 7, 7, True), (512, 64, 4, 14, False),
                                                   (128, 128, 5, 28, True), (128, 96, 7, 7, False)])
def test_chain_epilogue_groups_of_seven(tuning, Cin, Cout, H, W, use_skip):
    """The chaining epilogue of the seven-pixel-group kernels (chosen by default only for large batches)."""
    tuning(seven_pixel_groups=2)
    test_chain_epilogue_exact(Cin, Cout, H, W, 3, 1, 1, 1, 1, 1, use_skip, True)


@pytest.mark.parametrize("relu", [True, False])
@pytest.mark.parametrize("out_mode", [0, 1])
def test_chain_epilogue_nan_and_inf_in_the_skip(relu, out_mode):
    rnd = np.random.default_rng(5 + relu + 2 * out_mode)
    B, Cin, Cout, H, W = 2, 64, 64, 6, 8
    Lw = rnd.integers(0, 3, size=(Cout, 3, 3, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(B, H, W, Cin), dtype=np.int8)
    C = oracle.ternary_conv2d(Lw, Lx, 1, 1, 1)
    scale = (rnd.uniform(0.5, 1.5, Cout) / (float(C.std()) + 1.0)).astype(np.float32)
    bias = (rnd.standard_normal(Cout) * 0.3).astype(np.float32)
    skip = (rnd.standard_normal((B, H, W, Cout)) * 0.5).astype(np.float32)
    flat = skip.reshape(-1)
    flat[rnd.choice(flat.size, 300, replace=False)] = np.nan
    flat[rnd.choice(flat.size, 100, replace=False)] = np.inf
    flat[rnd.choice(flat.size, 100, replace=False)] = -np.inf
    f_want, lv_want = ochain.chain_epilogue(C, scale, bias, skip, relu, out_mode, 0.6, 0.8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT, fatnn.OHWI)
    Xp = fatnn.pack_ternary_bordered(dev(Lx), 1, 1)
    Xn = fatnn.bordered_act_init(B, H, W, Cout, 1, out_mode, device=DEV)
    Yf = torch.empty((B, H, W, Cout), dtype=torch.float32, device=DEV)
    fatnn.ternary_conv2d_chain(Wp, Xp, B, Cin, H, W, Cout, 3, 3, 1, 1, 1, dev(scale), dev(bias), dev(skip), relu,
                               0.6, 0.8, out_mode, 1, Xn, out_f=Yf)
    torch.cuda.synchronize()
    assert np.array_equal(Yf.cpu().numpy(), f_want, equal_nan=True)
    interior, _, _ = decode_bordered(Xn, B, H, W, Cout, 1)
    assert np.array_equal(interior, lv_want)


@pytest.mark.parametrize("relu", [True, False])
@pytest.mark.parametrize("out_mode", [0, 1])
@pytest.mark.parametrize("with_f", [True, False])
def test_chain_epilogue_unusual_channel_coefficients(relu, out_mode, with_f):
    """Per-channel scale and bias that are negative, zero, denormal, huge, infinite or NaN (the paper fixes one
    positive scale per layer; the library takes whatever float it is given and must follow the float32
    definition of the epilogue for all of them), with and without the fp32 output."""
    rnd = np.random.default_rng(77 + relu + 2 * out_mode)
    B, Cin, Cout, H, W = 2, 64, 128, 5, 9
    Lw = rnd.integers(0, 3, size=(Cout, 3, 3, Cin), dtype=np.int8)
    Lx = rnd.integers(0, 3, size=(B, H, W, Cin), dtype=np.int8)
    C = oracle.ternary_conv2d(Lw, Lx, 1, 1, 1)
    scale = (rnd.uniform(0.5, 1.5, Cout) / (float(C.std()) + 1.0)).astype(np.float32)
    bias = (rnd.standard_normal(Cout) * 0.3).astype(np.float32)
    scale[0:8] *= -1.0
    scale[8:12] = 0.0
    scale[12:14] = -0.0
    scale[14] = np.float32(1e-42)              # denormal
    scale[15] = np.float32(3e38)               # products overflow
    scale[16] = np.inf
    scale[17] = -np.inf
    scale[18] = np.nan
    bias[20] = np.inf
    bias[21] = -np.inf
    bias[22] = np.nan
    bias[23] = np.float32(-3e38)
    bias[16] = -np.inf                         # inf - inf
    skip = (rnd.standard_normal((B, H, W, Cout)) * 0.5).astype(np.float32)
    bias[14] = 0.0
    skip[..., 14] = 0.0                        # the denormal products of channel 14 reach the output as they are
    with np.errstate(all="ignore"):
        f_want, lv_want = ochain.chain_epilogue(C, scale, bias, skip, relu, out_mode, 0.6, 0.8)
    Wp = fatnn.pack_ternary(dev(Lw), fatnn.WEIGHT, fatnn.OHWI)
    Xp = fatnn.pack_ternary_bordered(dev(Lx), 1, 1)
    Xn = fatnn.bordered_act_init(B, H, W, Cout, 1, out_mode, device=DEV)
    Yf = torch.empty((B, H, W, Cout), dtype=torch.float32, device=DEV) if with_f else None
    fatnn.ternary_conv2d_chain(Wp, Xp, B, Cin, H, W, Cout, 3, 3, 1, 1, 1, dev(scale), dev(bias), dev(skip), relu,
                               0.6, 0.8, out_mode, 1, Xn, out_f=Yf)
    torch.cuda.synchronize()
    if with_f:
        assert np.array_equal(Yf.cpu().numpy(), f_want, equal_nan=True)
    interior, _, _ = decode_bordered(Xn, B, H, W, Cout, 1)
    assert np.array_equal(interior, lv_want)


@pytest.mark.parametrize("Cin,Cout,H,W,use_skip", [(128, 256, 9, 14, True), (256, 512, 6, 14, False)])
def test_chain_epilogue_stride2_groups_of_seven(tuning, Cin, Cout, H, W, use_skip):
    tuning(seven_pixel_groups=2)
    test_chain_epilogue_exact(Cin, Cout, H, W, 3, 2, 1, 1, 1, 1, use_skip, True)


def test_two_layers_chained_equal_the_oracle_pipeline():
    rnd = np.random.default_rng(99)
    B, H, W = 4, 14, 14
    Lw1 = rnd.integers(0, 3, size=(128, 3, 3, 64), dtype=np.int8)
    Lw2 = rnd.integers(0, 3, size=(128, 3, 3, 128), dtype=np.int8)
    xf = np.abs(rnd.standard_normal((B, H, W, 64))).astype(np.float32)
    a_in, a_mid = (0.7, 0.8), (0.9, 1.1)
    # oracle pipeline
    from oracle import quantizer as oq
    Lx = oq.levels_from_floats(xf, False, 1, *a_in)
    C1 = oracle.ternary_conv2d(Lw1, Lx, 1, 1, 1)
    scale1 = (rnd.uniform(0.5, 1.5, 128) / (C1.std() + 1)).astype(np.float32)
    bias1 = (rnd.standard_normal(128) * 0.2).astype(np.float32)
    _, L1 = ochain.chain_epilogue(C1, scale1, bias1, None, True, 1, *a_mid)
    C2 = oracle.ternary_conv2d(Lw2, L1, 1, 1, 1)
    # GPU pipeline: quantize+pack -> conv with chaining epilogue -> conv
    Wp1 = fatnn.pack_ternary(dev(Lw1), fatnn.WEIGHT, fatnn.OHWI)
    Wp2 = fatnn.pack_ternary(dev(Lw2), fatnn.WEIGHT, fatnn.OHWI)
    X0 = fatnn.quantize_pack_bordered(dev(xf), 1, fatnn.RELU, *a_in)
    X1 = fatnn.bordered_act_init(B, H, W, 128, 1, fatnn.RELU, device=DEV)
    fatnn.ternary_conv2d_chain(Wp1, X0, B, 64, H, W, 128, 3, 3, 1, 1, fatnn.RELU, dev(scale1), dev(bias1), None, True,
                               *a_mid, fatnn.RELU, 1, X1)
    Y2, _ = fatnn.ternary_conv2d(Wp2, X1, B, 128, H, W, 128, 3, 3, 1, 1, fatnn.RELU, x_layout=fatnn.X_BORDERED)
    assert np.array_equal(Y2.cpu().numpy(), C2)


def test_chain_rejects_shapes_without_a_streaming_kernel():
    Wp = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    Xp = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    sc = torch.ones(64, device=DEV)
    Xn = torch.empty(1 << 16, dtype=torch.uint8, device=DEV)
    with pytest.raises(fatnn.FatnnError) as e:
        fatnn.ternary_conv2d_chain(Wp, Xp, 1, 96, 4, 4, 64, 3, 3, 1, 1, 0, sc, None, None, False, 1.0, 1.0, 0, 1, Xn)
    assert e.value.status == -6

"""Fused quantize-and-pack (Algorithm 1, step 1 as written) against the quantizer oracle
(Eq. 8-10 literally in float32).  Levels decide integers from floats, so both sides work in
float32; the comparison is exact, including inputs within a few ulps of every threshold."""
import numpy as np
import pytest
import torch

from oracle import quantizer as oq
from test_gpu_parity import decode_packed, dev, DEV

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")

ALPHAS = [(0.7, 0.9), (1.3, 0.2), (0.05, 2.5), (0.5, 0.25), (1.0, 1.0), (3.1415927, 0.33333334),
          # step sizes far from one: tiny, a second step below the first one's rounding unit, denormal, near overflow
          (1e-30, 3e-30), (1e30, 1e-30), (1e-40, 1e-40), (3e38, 3e38)]


def adversarial(rnd, n, a1, a2):
    """Random normals plus clouds of floats within +-8 ulps of every real-number threshold."""
    x = (rnd.standard_normal(n) * 1.5).astype(np.float32)
    with np.errstate(over="ignore"):              # a1 + a2 / 2 may round to +inf (step sizes near overflow)
        centres = np.array([-a1 / 2, a2 / 2, a1 / 2, a1 + a2 / 2, 0.0, -0.0, a1, a2], np.float32)
    pos = rnd.choice(n, size=min(n, 64 * len(centres)), replace=False)
    k = 0
    for c in centres:
        v = c
        cloud = [c]
        up, dn = c, c
        for _ in range(8):
            up = np.nextafter(up, np.float32(np.inf))
            dn = np.nextafter(dn, np.float32(-np.inf))
            cloud += [up, dn]
        for v in cloud:
            if k < len(pos):
                x[pos[k]] = v
                k += 1
    x[pos[-1]] = np.inf
    x[pos[-2]] = -np.inf
    return x


@pytest.mark.parametrize("a1,a2", ALPHAS)
@pytest.mark.parametrize("role,mode", [(0, 0), (1, 0), (1, 1)])
def test_quantize_pack_rowmajor_exact(a1, a2, role, mode):
    rnd = np.random.default_rng(int(a1 * 1000) + role * 7 + mode)
    for rows, K in [(37, 100), (16, 576), (5, 33), (3, 4609)]:
        x = adversarial(rnd, rows * K, a1, a2).reshape(rows, K)
        cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
        buf = fatnn.quantize_pack(dev(x), role, mode, a1, a2, n_invalid=cnt)
        torch.cuda.synchronize()
        body, tail = decode_packed(buf, rows, K, role)
        want = oq.levels_from_floats(x, role == fatnn.WEIGHT, mode, a1, a2)
        assert np.array_equal(body, want)
        assert (tail == 1).all()
        assert int(cnt.item()) == 0
        if role == fatnn.WEIGHT:
            off = fatnn.weight_consts_offset(rows, K)
            consts = buf.cpu().numpy()[off: off + rows * 8].view(np.int32)
            assert np.array_equal(consts[:rows], (want != 1).sum(axis=1))
            assert np.array_equal(consts[rows:], (want == 2).sum(axis=1))


def test_quantize_pack_equals_level_pack_of_the_oracle_levels():
    rnd = np.random.default_rng(3)
    a1, a2 = 0.6, 0.45
    x = adversarial(rnd, 64 * 9 * 64, a1, a2).reshape(64, 3, 3, 64)
    lv = oq.levels_from_floats(x, True, 0, a1, a2)
    a = fatnn.quantize_pack(dev(x), fatnn.WEIGHT, 0, a1, a2, layout=fatnn.OHWI)
    b = fatnn.pack_ternary(dev(lv), fatnn.WEIGHT, fatnn.OHWI)
    nwords = 64 * 18 * 8
    ioff = fatnn.weight_interleaved_offset(64, 576)
    coff = fatnn.weight_consts_offset(64, 576)
    assert torch.equal(a[:nwords], b[:nwords])
    assert torch.equal(a[coff:coff + 64 * 8], b[coff:coff + 64 * 8])
    assert torch.equal(a[ioff:], b[ioff:])


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("border", [0, 1])
def test_quantize_pack_bordered_equals_bordered_level_pack(mode, border):
    rnd = np.random.default_rng(11 + mode + border)
    a1, a2 = 0.8, 0.3
    x = adversarial(rnd, 3 * 9 * 7 * 64, a1, a2).reshape(3, 9, 7, 64)
    lv = oq.levels_from_floats(x, False, mode, a1, a2)
    a = fatnn.quantize_pack_bordered(dev(x), border, mode, a1, a2)
    b = fatnn.pack_ternary_bordered(dev(lv), border, mode)
    assert torch.equal(a, b)


def test_nan_is_counted_and_packed_as_zero():
    a1, a2 = 0.7, 0.9
    x = np.linspace(-2, 2, 4 * 64, dtype=np.float32).reshape(4, 64)
    x[1, 5] = np.nan
    x[3, 63] = np.nan
    for role, mode, zero_level in [(0, 0, 1), (1, 0, 1), (1, 1, 0)]:
        cnt = torch.zeros(1, dtype=torch.int32, device=DEV)
        buf = fatnn.quantize_pack(dev(x), role, mode, a1, a2, n_invalid=cnt)
        torch.cuda.synchronize()
        assert int(cnt.item()) == 2
        if role == fatnn.WEIGHT or mode == 0:
            body, _ = decode_packed(buf, 4, 64, role)
        else:
            words = buf.cpu().numpy()[: 4 * 2 * 8].view(np.uint32).reshape(4, 2, 2)
            bits = np.unpackbits(words.view(np.uint8).reshape(4, 2, 2, 4), axis=-1, bitorder="little").reshape(4, 2, 2, 32)
            body = (bits[:, :, 0, :] + bits[:, :, 1, :]).reshape(4, 64).astype(np.int8)
        assert body[1, 5] == zero_level and body[3, 63] == zero_level
        assert oq.count_invalid(x) == 2
        want = oq.levels_from_floats(x, role == fatnn.WEIGHT, mode, a1, a2)
        assert want[1, 5] == zero_level and want[3, 63] == zero_level
        assert np.array_equal(body, want)


def test_end_to_end_float_conv_through_quantizers():
    # floats -> (quantize+pack) -> ternary conv  ==  oracle conv on the oracle's levels
    import oracle
    rnd = np.random.default_rng(21)
    wf = (rnd.standard_normal((70, 3, 3, 64)) * 0.5).astype(np.float32)
    xf = np.abs(rnd.standard_normal((3, 10, 9, 64))).astype(np.float32)
    wa, xa = (0.5, 0.6), (0.7, 0.8)
    Wp = fatnn.quantize_pack(dev(wf), fatnn.WEIGHT, 0, *wa, layout=fatnn.OHWI)
    Xp = fatnn.quantize_pack_bordered(dev(xf), 1, fatnn.RELU, *xa)
    Y, _ = fatnn.ternary_conv2d(Wp, Xp, 3, 64, 10, 9, 70, 3, 3, 1, 1, fatnn.RELU, x_layout=fatnn.X_BORDERED)
    Lw = oq.levels_from_floats(wf, True, 0, *wa)
    Lx = oq.levels_from_floats(xf, False, 1, *xa)
    assert np.array_equal(Y.cpu().numpy(), oracle.ternary_conv2d(Lw, Lx, 1, 1, 1))

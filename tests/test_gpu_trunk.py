"""The ResNet-18-shaped ternary trunk (19 convolutions chained through the fused epilogue)
against the same data flow built from the oracle's pieces; exact in fp32 and in levels."""
import numpy as np
import pytest
import torch

import oracle
import synth_inputs as si
from oracle import chain as ochain
from oracle import quantizer as oq
from test_gpu_parity import dev, DEV
from test_gpu_chain import decode_bordered

pytestmark = pytest.mark.gpu

fatnn = pytest.importorskip("paper_2008_05101_amd")
from paper_2008_05101_amd import resnet_trunk as rt  # noqa: E402


def to_gpu_blocks(blocks):
    def cv(d):
        return rt.ConvParams(dev(d["levels"]), dev(d["scale"]), dev(d["bias"]), d["alpha"], d["stride"])
    return [rt.BlockParams(cv(b["conv1"]), cv(b["conv2"]), None if b["shortcut"] is None else cv(b["shortcut"]))
            for b in blocks]


def oracle_trunk(blocks, x, in_alpha):
    L = oq.levels_from_floats(x, False, 1, *in_alpha)
    f = x
    for b in blocks:
        c1, c2, sc = b["conv1"], b["conv2"], b["shortcut"]
        C1 = oracle.ternary_conv2d(c1["levels"], L, c1["stride"], 1, 1)
        _, Lmid = ochain.chain_epilogue(C1, c1["scale"], c1["bias"], None, True, 1, *c1["alpha"])
        skip = f
        if sc is not None:
            Cs = oracle.ternary_conv2d(sc["levels"], L, sc["stride"], 0, 1)
            skip = oracle.scale_epilogue(Cs, sc["scale"], sc["bias"], channel_is_row=False)
        C2 = oracle.ternary_conv2d(c2["levels"], Lmid, 1, 1, 1)
        f, L = ochain.chain_epilogue(C2, c2["scale"], c2["bias"], skip, True, 1, *c2["alpha"])
    return f, L


@pytest.mark.parametrize("batch,size", [(2, 56), (3, 24)])
def test_trunk_matches_oracle_pipeline(batch, size):
    blocks = si.trunk_params()
    x = si.trunk_input(batch, size)
    in_alpha = (0.6, 0.7)
    f_want, L_want = oracle_trunk(blocks, x, in_alpha)
    trunk = rt.Trunk(to_gpu_blocks(blocks), batch, size, in_alpha, device=DEV)
    seen = []
    f_got, p_got = trunk.forward(dev(x), before_conv=seen.append)
    torch.cuda.synchronize()
    assert sorted(seen) == list(range(19))
    assert np.array_equal(f_got.cpu().numpy(), f_want)
    interior, _, _ = decode_bordered(p_got, batch, f_want.shape[1], f_want.shape[2], 512, 1)
    assert np.array_equal(interior, L_want)
    # the levels are not degenerate (the synthetic scales keep all three levels in use)
    assert len(np.unique(L_want)) == 3
    assert trunk.macs == sum(c.macs() for c in si.cfg3(batch)) if size == 56 else True


def test_trunk_full_batch_every_image():
    # the launch configuration bench.py times (batch 64): the oracle pipeline runs all 64 images and
    # every fp32 output and every packed level of the last layer is compared
    blocks = si.trunk_params()
    batch = 64
    x = si.trunk_input(batch)
    in_alpha = (0.6, 0.7)
    trunk = rt.Trunk(to_gpu_blocks(blocks), batch, 56, in_alpha, device=DEV)
    f_got, p_got = trunk.forward(dev(x))
    f_got = f_got.cpu().numpy()
    interior, _, _ = decode_bordered(p_got, batch, 7, 7, 512, 1)
    f_want, L_want = oracle_trunk(blocks, x, in_alpha)
    assert np.array_equal(f_got, f_want)
    assert np.array_equal(interior, L_want)
    assert trunk.macs == sum(c.macs() for c in si.cfg3(batch))


def test_trunk_graph_replays_equal_eager_passes():
    """A captured pass replayed several times, with eager passes and synchronisations in between and a
    fresh input each time, gives the eager result bit for bit on every replay."""
    blocks = si.trunk_params()
    batch, size = 2, 24
    in_alpha = (0.6, 0.7)
    trunk = rt.Trunk(to_gpu_blocks(blocks), batch, size, in_alpha, device=DEV)
    x_static = dev(si.trunk_input(batch, size))
    graph = trunk.capture(x_static)
    rnd = np.random.default_rng(7)
    for rep in range(4):
        x_new = np.abs(rnd.standard_normal((batch, size, size, 64))).astype(np.float32) * (0.5 + rep)
        x_static.copy_(dev(x_new))
        f_e, p_e = trunk.forward(x_static)          # eager pass on the same buffers
        torch.cuda.synchronize()
        f_eager, p_eager = f_e.clone(), p_e.clone()
        f_e.zero_()
        p_e.zero_()                                  # make sure the replay really rewrites its outputs
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        f_g, p_g = trunk.graph_out
        assert torch.equal(f_g, f_eager)
        assert torch.equal(p_g, p_eager)
        assert float(f_eager.abs().sum()) > 0


def test_resnet34_shaped_trunk_matches_oracle_pipeline():
    """The deeper of the paper's two ImageNet networks (16 basic blocks, 35 ternary convolutions)."""
    blocks = si.trunk_params(34)
    assert len(blocks) == 16
    batch, size = 1, 24
    x = si.trunk_input(batch, size)
    in_alpha = (0.6, 0.7)
    f_want, L_want = oracle_trunk(blocks, x, in_alpha)
    trunk = rt.Trunk(to_gpu_blocks(blocks), batch, size, in_alpha, device=DEV)
    seen = []
    f_got, p_got = trunk.forward(dev(x), before_conv=seen.append)
    torch.cuda.synchronize()
    assert sorted(seen) == list(range(35))
    assert np.array_equal(f_got.cpu().numpy(), f_want)
    interior, _, _ = decode_bordered(p_got, batch, f_want.shape[1], f_want.shape[2], 512, 1)
    assert np.array_equal(interior, L_want)
    assert len(np.unique(L_want)) >= 2

"""A ResNet-18-shaped ternary trunk wired from the library's entry points.

Orchestration only: which kernel runs on which buffer.  Every arithmetic step -- the
input quantizer, the ternary convolutions, the folded batch-norm affine, the skip
addition, ReLU, re-quantisation and packing -- runs inside the HIP kernels
(fatnn_quantize_pack_bordered, fatnn_ternary_conv2d, fatnn_ternary_conv2d_chain).

Data flow of a basic block, as the paper's Supplementary S1 describes the deployed
network (high-precision skip connections, everything else fused into the
convolutions):

    x_packed --conv1 (3x3, stride s) --> affine, ReLU, quantize, pack --> mid_packed
    mid_packed --conv2 (3x3) --> affine, + skip, ReLU --> out_f32 (next skip)
                                                      \\-> quantize, pack --> out_packed
    skip = x_f32, or for a down-sampling block the fp32 output of a 1x1 stride-s
    convolution of x_packed (affine only)

The first convolution and the classifier of the network are not ternary in the paper
and are not part of the trunk.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, List, Optional, Sequence, Tuple

import torch

from . import binding as fb

# (Cin, Cout, stride) of the eight basic blocks after the stem (56x56 input, 64 channels)
RESNET18_BLOCKS: Tuple[Tuple[int, int, int], ...] = (
    (64, 64, 1), (64, 64, 1), (64, 128, 2), (128, 128, 1), (128, 256, 2), (256, 256, 1), (256, 512, 2), (512, 512, 1))


@dataclass
class ConvParams:
    """One ternary convolution: level tensor OHWI (int8), fp32 scale and bias per output
    channel, and the step sizes of the quantizer that its output feeds."""
    levels: torch.Tensor
    scale: torch.Tensor
    bias: torch.Tensor
    alpha: Tuple[float, float]
    stride: int


@dataclass
class BlockParams:
    conv1: ConvParams
    conv2: ConvParams
    shortcut: Optional[ConvParams]     # 1x1 stride-s convolution, or None for an identity skip


def conv_order(blocks: Sequence[BlockParams]) -> List[ConvParams]:
    """Convolutions in the order the layer list of the workload uses (conv1, conv2, shortcut)."""
    out = []
    for b in blocks:
        out += [b.conv1, b.conv2] + ([b.shortcut] if b.shortcut is not None else [])
    return out


class Trunk:
    """Packs the weights, allocates every buffer once, then `forward` only launches kernels."""

    def __init__(self, blocks: Sequence[BlockParams], batch: int, size: int, in_alpha: Tuple[float, float],
                 device: str = "cuda:0"):
        self.blocks = list(blocks)
        self.B, self.size, self.in_alpha, self.dev = batch, size, in_alpha, torch.device(device)
        self.packed = {}
        for cp in conv_order(self.blocks):
            self.packed[id(cp)] = fb.pack_ternary(cp.levels, fb.WEIGHT, fb.OHWI)
        B = batch
        cin0 = self.blocks[0].conv1.levels.shape[3]
        self.x0 = torch.empty(max(fb.bordered_act_bytes(B, size, size, cin0, 1), 16), dtype=torch.uint8,
                              device=self.dev)
        self.bufs = []
        hw = size
        for bp in self.blocks:
            cout = bp.conv1.levels.shape[0]
            hw_out = (hw + 2 - 3) // bp.conv1.stride + 1
            mid = fb.bordered_act_init(B, hw_out, hw_out, cout, 1, fb.RELU, device=self.dev)
            outp = fb.bordered_act_init(B, hw_out, hw_out, cout, 1, fb.RELU, device=self.dev)
            outf = torch.empty((B, hw_out, hw_out, cout), dtype=torch.float32, device=self.dev)
            skipf = (torch.empty((B, hw_out, hw_out, cout), dtype=torch.float32, device=self.dev)
                     if bp.shortcut is not None else None)
            self.bufs.append((mid, outp, outf, skipf, hw, hw_out))
            hw = hw_out
        self.macs = 0
        hw = size
        for bp in self.blocks:
            cout, _, _, cin = bp.conv1.levels.shape
            hw_out = (hw + 2 - 3) // bp.conv1.stride + 1
            n = B * hw_out * hw_out
            self.macs += n * cout * 9 * cin + n * cout * 9 * cout
            if bp.shortcut is not None:
                self.macs += n * cout * cin
            hw = hw_out

    def forward(self, x_f32: torch.Tensor, before_conv: Optional[Callable[[int], None]] = None):
        """x_f32: fp32 NHWC [B][size][size][C0], non-negative.  Returns (out_f32, out_packed) of the
        last block.  `before_conv(i)` is called before the i-th convolution launch (measurement)."""
        B = self.B
        fb.quantize_pack_bordered(x_f32, 1, fb.RELU, *self.in_alpha, out=self.x0)
        xp, xf = self.x0, x_f32
        k = 0
        for bp, (mid, outp, outf, skipf, hw, hw_out) in zip(self.blocks, self.bufs):
            cout, _, _, cin = bp.conv1.levels.shape
            c1, c2, sc = bp.conv1, bp.conv2, bp.shortcut
            # layer-list order inside a block: conv1, conv2, shortcut
            if before_conv:
                before_conv(k)
            fb.ternary_conv2d_chain(self.packed[id(c1)], xp, B, cin, hw, hw, cout, 3, 3, c1.stride, 1, fb.RELU,
                                    c1.scale, c1.bias, None, True, c1.alpha[0], c1.alpha[1], fb.RELU, 1, mid)
            skip = xf
            if sc is not None:
                if before_conv:
                    before_conv(k + 2)
                fb.ternary_conv2d(self.packed[id(sc)], xp, B, cin, hw, hw, cout, 1, 1, sc.stride, 0, fb.RELU,
                                  scale=sc.scale, bias=sc.bias, out_f=skipf, want_int=False,
                                  x_layout=fb.X_BORDERED1)
                skip = skipf
            if before_conv:
                before_conv(k + 1)
            fb.ternary_conv2d_chain(self.packed[id(c2)], mid, B, cout, hw_out, hw_out, cout, 3, 3, 1, 1, fb.RELU,
                                    c2.scale, c2.bias, skip, True, c2.alpha[0], c2.alpha[1], fb.RELU, 1, outp,
                                    out_f=outf)
            k += 3 if sc is not None else 2
            xp, xf = outp, outf
        return xf, xp

    def capture(self, x_static: torch.Tensor) -> "torch.cuda.CUDAGraph":
        """Records one forward pass on `x_static` into a HIP graph and returns it; `graph.replay()` then
        re-runs the 20 launches with one submission (at small batch the pass is launch-bound).  The caller
        refreshes `x_static` in place between replays; the outputs are the tensors `forward` returns.
        Only the library's own kernels are recorded (no memset nodes, no library reductions)."""
        self.forward(x_static)          # every one-time host query of the launchers happens outside the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.graph_out = self.forward(x_static)
        torch.cuda.synchronize()
        return graph

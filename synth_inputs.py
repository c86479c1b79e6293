"""Seeded synthetic inputs for the ternary GEMM / convolution hot path.

This module only draws random level tensors and names the workload shapes.  It
holds none of the method's arithmetic, so both the CPU oracle's tests and the
HIP path's tests can feed from it without sharing any computation.

Levels are int8 level indices l in {0,1,2}.  Weights always mean the value
l-1 in {-1,0,+1}.  Activations mean l-1 (symmetric mode) or l (ReLU mode,
values {0,1,2}; the paper's second constraint in Section 3.3).

The paper times ImageNet ResNet-18/34 layers with trained weights; neither the
data set nor the weights are needed for timing or bit-exactness of an integer
kernel that exploits no sparsity, so iid level tensors of the same shapes stand
in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 20080510 * 100

TENSOR_W, TENSOR_A, TENSOR_SCALE, TENSOR_BIAS = 0, 1, 2, 3

SYM, RELU = 0, 1


def rng_for(config: int, tensor_id: int, sub: int = 0) -> np.random.Generator:
    """Generator for one tensor of one workload (sub = layer index inside it)."""
    return np.random.Generator(np.random.PCG64(SEED_BASE + 10 * config + tensor_id + 1000 * sub))


def levels(rng: np.random.Generator, shape: Sequence[int], p: Sequence[float] = (1 / 3, 1 / 3, 1 / 3)) -> np.ndarray:
    """iid level indices in {0,1,2} with probabilities p[0], p[1], p[2]."""
    p = np.asarray(p, dtype=np.float64)
    p = p / p.sum()
    u = rng.random(size=tuple(shape), dtype=np.float32)
    out = (u >= np.float32(p[0])).astype(np.int8)
    out += (u >= np.float32(p[0] + p[1])).astype(np.int8)
    return out


def levels4(rng: np.random.Generator, shape: Sequence[int]) -> np.ndarray:
    """iid 2-bit codes in {0,1,2,3}, uniform."""
    return rng.integers(0, 4, size=tuple(shape), dtype=np.int8)


def scale_vec(rng: np.random.Generator, n: int) -> np.ndarray:
    return rng.uniform(0.5, 1.5, size=n).astype(np.float32)


def bias_vec(rng: np.random.Generator, n: int) -> np.ndarray:
    return rng.standard_normal(size=n).astype(np.float32)


def act_probs_zero_half(act_mode: int) -> Tuple[float, float, float]:
    """P(value 0) = 0.5, the two other values 0.25 each, as level probabilities."""
    return (0.5, 0.25, 0.25) if act_mode == RELU else (0.25, 0.5, 0.25)


@dataclass
class GemmCase:
    name: str
    M: int
    N: int
    K: int
    act_mode: int = SYM
    w_probs: Tuple[float, float, float] = (1 / 3, 1 / 3, 1 / 3)
    a_probs: Tuple[float, float, float] = (1 / 3, 1 / 3, 1 / 3)
    config: int = 0
    sub: int = 0

    def macs(self) -> int:
        return self.M * self.N * self.K

    def make(self) -> Tuple[np.ndarray, np.ndarray]:
        """(Lw [M][K], La [N][K]) int8 levels."""
        lw = levels(rng_for(self.config, TENSOR_W, self.sub), (self.M, self.K), self.w_probs)
        la = levels(rng_for(self.config, TENSOR_A, self.sub), (self.N, self.K), self.a_probs)
        return lw, la


@dataclass
class ConvCase:
    name: str
    B: int
    Cin: int
    H: int
    W: int
    Cout: int
    R: int = 3
    S: int = 3
    stride: int = 1
    pad: int = 1
    act_mode: int = RELU
    w_probs: Tuple[float, float, float] = (1 / 3, 1 / 3, 1 / 3)
    a_probs: Tuple[float, float, float] = (1 / 3, 1 / 3, 1 / 3)
    config: int = 0
    sub: int = 0

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def M(self) -> int:
        return self.Cout

    @property
    def N(self) -> int:
        return self.B * self.Ho * self.Wo

    @property
    def K(self) -> int:
        return self.R * self.S * self.Cin

    def macs(self) -> int:
        return self.M * self.N * self.K

    def make(self, batch: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
        """(Lw [Cout][R][S][Cin], Lx [B][H][W][Cin]) int8 levels (OHWI / NHWC)."""
        b = self.B if batch is None else batch
        lw = levels(rng_for(self.config, TENSOR_W, self.sub), (self.Cout, self.R, self.S, self.Cin), self.w_probs)
        lx = levels(rng_for(self.config, TENSOR_A, self.sub), (b, self.H, self.W, self.Cin), self.a_probs)
        return lw, lx

    def make_scale_bias(self) -> Tuple[np.ndarray, np.ndarray]:
        return (scale_vec(rng_for(self.config, TENSOR_SCALE, self.sub), self.Cout),
                bias_vec(rng_for(self.config, TENSOR_BIAS, self.sub), self.Cout))


# ---------------------------------------------------------------------------
# The five workloads
# ---------------------------------------------------------------------------

def cfg1() -> GemmCase:
    """Small single GEMM (oracle runs in well under a second)."""
    return GemmCase("cfg1_gemm_64x1024x576", 64, 1024, 576, SYM, config=1)


def cfg2(batch: int = 32) -> ConvCase:
    """ResNet-18-style 3x3 conv, 128->128 at 28x28, batch 32."""
    return ConvCase("cfg2_conv3x3_128_28", batch, 128, 28, 28, 128, 3, 3, 1, 1, RELU, config=2)


def cfg3(batch: int = 64) -> List[ConvCase]:
    """All ternary conv layers of a ResNet-18-shaped net (first conv, FC excluded)."""
    a = act_probs_zero_half(RELU)
    spec = []
    spec += [(64, 56, 64, 3, 1, 1)] * 4
    spec += [(64, 56, 128, 3, 2, 1), (128, 28, 128, 3, 1, 1), (64, 56, 128, 1, 2, 0)]
    spec += [(128, 28, 128, 3, 1, 1)] * 2
    spec += [(128, 28, 256, 3, 2, 1), (256, 14, 256, 3, 1, 1), (128, 28, 256, 1, 2, 0)]
    spec += [(256, 14, 256, 3, 1, 1)] * 2
    spec += [(256, 14, 512, 3, 2, 1), (512, 7, 512, 3, 1, 1), (256, 14, 512, 1, 2, 0)]
    spec += [(512, 7, 512, 3, 1, 1)] * 2
    out = []
    for i, (cin, hw, cout, ks, st, pd) in enumerate(spec):
        out.append(ConvCase(f"cfg3_L{i:02d}_{ks}x{ks}_{cin}to{cout}_{hw}s{st}", batch, cin, hw, hw, cout,
                            ks, ks, st, pd, RELU, a_probs=a, config=3, sub=i))
    return out


def cfg4(size: int = 8192) -> GemmCase:
    """Large square GEMM: the VALU roofline point."""
    return GemmCase(f"cfg4_gemm_{size}", size, size, size, SYM, w_probs=(0.335, 0.33, 0.335), config=4)


def cfg5_ragged() -> GemmCase:
    return GemmCase("cfg5a_gemm_512x3136x4609", 512, 3136, 4609, SYM, config=5, sub=0)


def cfg5_gemv() -> GemmCase:
    return GemmCase("cfg5b_gemv_4096x1x4608", 4096, 1, 4608, SYM, config=5, sub=1)


def cfg5_bottleneck(batch: int = 128) -> List[ConvCase]:
    return [
        ConvCase("cfg5c_1x1_256to64_56", batch, 256, 56, 56, 64, 1, 1, 1, 0, RELU, config=5, sub=2),
        ConvCase("cfg5c_1x1_64to256_56", batch, 64, 56, 56, 256, 1, 1, 1, 0, RELU, config=5, sub=3),
    ]


def paper_six(batch: int = 1) -> List[ConvCase]:
    """The six layer shapes of the paper's layer-wise timing (Section 5.1.1): 3x3, stride 1, pad 1, equal
    input and output channels; 64 channels at 28, 56, 112, 224 pixels, then 128 and 256 channels at 56."""
    spec = ((64, 28), (64, 56), (64, 112), (64, 224), (128, 56), (256, 56))
    return [ConvCase(f"case{i + 1}_3x3_{c}_{r}", batch, c, r, r, c, 3, 3, 1, 1, RELU, config=6, sub=i)
            for i, (c, r) in enumerate(spec)]


def trunk_blocks(depth: int = 18):
    """(Cin, Cout, stride) of the basic blocks after the stem for ResNet-18 or ResNet-34."""
    counts = {18: (2, 2, 2, 2), 34: (3, 4, 6, 3)}[depth]
    out = []
    cin = 64
    for stage, n in enumerate(counts):
        cout = 64 << stage
        for i in range(n):
            out.append((cin, cout, 2 if (i == 0 and stage > 0) else 1))
            cin = cout
    return tuple(out)


def trunk_params(depth: int = 18):
    """Synthetic parameters of the ResNet-18- (or ResNet-34-) shaped trunk, as plain numpy arrays.

    Returns a list of blocks; each block is a dict with conv1, conv2 and (for down-sampling blocks)
    shortcut, each a dict: levels OHWI int8, scale, bias fp32, alpha (a1, a2), stride.  For depth 18 the
    layer shapes and weight seeds are those of cfg3's layer list; deeper trunks continue the numbering.
    """
    out = []
    li = 0
    hw = 56

    def conv(cin: int, cout: int, ks: int, stride: int, idx: int):
        k = ks * ks * cin
        lw = levels(rng_for(3, TENSOR_W, idx), (cout, ks, ks, cin))
        r = rng_for(3, TENSOR_SCALE, idx)
        scale = (r.uniform(0.5, 1.5, size=cout) / np.sqrt(k)).astype(np.float32)
        bias = (rng_for(3, TENSOR_BIAS, idx).standard_normal(cout) * 0.3).astype(np.float32)
        a = 0.01 * (idx % 19)
        alpha = (float(np.float32(0.7 + a)), float(np.float32(0.9 - a)))
        return {"levels": lw, "scale": scale, "bias": bias, "alpha": alpha, "stride": stride}

    for cin, cout, stride in trunk_blocks(depth):
        blk = {"conv1": conv(cin, cout, 3, stride, li), "conv2": conv(cout, cout, 3, 1, li + 1), "shortcut": None}
        li += 2
        if stride != 1 or cin != cout:
            blk["shortcut"] = conv(cin, cout, 1, stride, li)
            li += 1
        out.append(blk)
        hw //= stride
    if depth == 18:
        layers = cfg3(batch=1)
        assert li == len(layers)
        flat = [c for b in out for c in ([b["conv1"], b["conv2"]] + ([b["shortcut"]] if b["shortcut"] else []))]
        for c, case in zip(flat, layers):
            assert c["levels"].shape == (case.Cout, case.R, case.S, case.Cin) and c["stride"] == case.stride
    return out


def trunk_input(batch: int, size: int = 56, channels: int = 64) -> np.ndarray:
    """Non-negative fp32 NHWC input of the trunk (what a ReLU after the stem would produce)."""
    r = rng_for(3, TENSOR_A, 999)
    return np.abs(r.standard_normal((batch, size, size, channels))).astype(np.float32)

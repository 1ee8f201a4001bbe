"""Seeded synthetic convolution layers: shapes and input generators only.

This module holds none of the method's arithmetic.  It names the layer shapes the
benchmarks and parity tests run on (AlexNet- and VGG-shaped layers standing in for
the networks the paper measured in Section 5, plus a pointwise / strided mix) and
draws their fp32 inputs from a seeded CPU generator, so that the GPU path and the
CPU oracle can be handed identical host arrays.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    seed: int
    in_dist: str = "u11"      # "u11" = U[-1,1], "u01" = U[0,1]
    w_dist: str = "normal"    # "normal" = N(0, 1/(C*R*S)), "u11" = U[-1,1]

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def crs(self) -> int:
        return self.C * self.R * self.S

    @property
    def flops(self) -> int:
        """2*N*K*C*R*S*P*Q: padded (zero) taps are counted."""
        return 2 * self.N * self.K * self.crs * self.P * self.Q

    @property
    def algorithmic_bytes(self) -> int:
        """Read in and w once, write out once (fp32)."""
        return 4 * (self.N * self.C * self.H * self.W + self.K * self.crs
                    + self.N * self.K * self.P * self.Q)

    def dims(self):
        return (self.N, self.C, self.H, self.W, self.K, self.R, self.S, self.stride, self.pad)

    def with_batch(self, N: int) -> "Layer":
        return Layer(f"{self.name.rsplit('_n', 1)[0]}_n{N}", N, self.C, self.H, self.W, self.K,
                     self.R, self.S, self.stride, self.pad, self.seed, self.in_dist, self.w_dist)


def _mk(group, index, name, N, C, HW, K, RS, stride, pad, **kw):
    seed = kw.pop("seed", 1000 * group + index)
    return Layer(name, N, C, HW, HW, K, RS, RS, stride, pad, seed, **kw)


# Group 1: the small case the oracle finishes instantly (seed 0, U[-1,1] weights).
TOY = _mk(1, 0, "toy_c3_k16_3x3", 1, 3, 32, 16, 3, 1, 1, seed=0, w_dist="u11")

# Group 2: AlexNet-shaped first layer, inputs U[0,1].
ALEX_CONV1 = [
    _mk(2, 0, "alex_conv1_n1", 1, 3, 227, 96, 11, 4, 0, in_dist="u01"),
    _mk(2, 0, "alex_conv1_n64", 64, 3, 227, 96, 11, 4, 0, in_dist="u01"),
]

# Group 3: AlexNet-shaped conv2..conv5, ungrouped.
_ALEX_REST = [
    ("alex_conv2", 96, 27, 256, 5, 1, 2),
    ("alex_conv3", 256, 13, 384, 3, 1, 1),
    ("alex_conv4", 384, 13, 384, 3, 1, 1),
    ("alex_conv5", 384, 13, 256, 3, 1, 1),
]
ALEX_REST = [
    _mk(3, i, f"{nm}_n{N}", N, C, HW, K, RS, st, pd)
    for i, (nm, C, HW, K, RS, st, pd) in enumerate(_ALEX_REST) for N in (1, 64)
]

# Group 4: VGG-16-shaped 3x3 stride-1 pad-1 layers at batch 32.
_VGG = [(64, 224, 64), (128, 112, 128), (256, 56, 256), (512, 28, 512), (512, 14, 512)]
VGG = [
    _mk(4, i, f"vgg_c{C}_{HW}_k{K}_n32", 32, C, HW, K, 3, 1, 1)
    for i, (C, HW, K) in enumerate(_VGG)
]

# Group 5: pointwise / strided mix at batch 64.
MIX = [
    _mk(5, 0, "pw_c256_56_k64_n64", 64, 256, 56, 64, 1, 1, 0),
    _mk(5, 1, "pw_c64_56_k256_n64", 64, 64, 56, 256, 1, 1, 0),
    _mk(5, 2, "s2_c128_56_k256_3x3_n64", 64, 128, 56, 256, 3, 2, 1),
    _mk(5, 3, "s2_c3_224_k64_7x7_n64", 64, 3, 224, 64, 7, 2, 3),
]

# Group 6: GoogLeNet-shaped layers (the paper's third network; its layer list is not in the
# paper's text): the three branch kinds of an inception module -- 1x1 reductions, 3x3 and
# 5x5 convolutions behind them -- at the three spatial sizes such modules run at, with
# channel counts of that kind (many of them not multiples of 32 or 128), and the 3x3 layer
# of the stem.  A suite of its own: not part of the headline metric.
_INCEPTION = [
    ("inc_56_3x3_c64_k192", 64, 56, 192, 3, 1),
    ("inc_28_1x1_c192_k64", 192, 28, 64, 1, 0),
    ("inc_28_3x3_c96_k128", 96, 28, 128, 3, 1),
    ("inc_28_5x5_c16_k32", 16, 28, 32, 5, 2),
    ("inc_14_1x1_c480_k192", 480, 14, 192, 1, 0),
    ("inc_14_3x3_c112_k224", 112, 14, 224, 3, 1),
    ("inc_14_5x5_c24_k64", 24, 14, 64, 5, 2),
    ("inc_7_1x1_c832_k256", 832, 7, 256, 1, 0),
    ("inc_7_3x3_c160_k320", 160, 7, 320, 3, 1),
    ("inc_7_5x5_c32_k128", 32, 7, 128, 5, 2),
]
INCEPTION = [_mk(6, i, f"{nm}_n64", 64, C, HW, K, RS, 1, pd) for i, (nm, C, HW, K, RS, pd) in enumerate(_INCEPTION)]

ALL_LAYERS = [TOY] + ALEX_CONV1 + ALEX_REST + VGG + MIX
BY_NAME = {l.name: l for l in ALL_LAYERS + INCEPTION}

# The layer the headline number is quoted on (largest flop count among the batched
# layers whose shape the main 3x3 kernel serves).
HEADLINE = "vgg_c256_56_k256_n32"


def make_inputs(layer: Layer, N: int | None = None):
    """Host fp32 arrays (in [N,C,H,W], w [K,C,R,S]) drawn from the layer's seed.

    N, if given, truncates the batch: image n is the same whatever N is asked for,
    because images are drawn one after another from the same stream.
    """
    g = torch.Generator(device="cpu")
    g.manual_seed(layer.seed)
    K, C, R, S = layer.K, layer.C, layer.R, layer.S
    if layer.w_dist == "normal":
        w = torch.randn((K, C, R, S), generator=g, dtype=torch.float32) / float(np.sqrt(C * R * S))
    elif layer.w_dist == "u11":
        w = torch.rand((K, C, R, S), generator=g, dtype=torch.float32) * 2.0 - 1.0
    else:
        raise ValueError(layer.w_dist)
    n = layer.N if N is None else min(N, layer.N)
    x = torch.rand((n, C, layer.H, layer.W), generator=g, dtype=torch.float32)
    if layer.in_dist == "u11":
        x = x * 2.0 - 1.0
    elif layer.in_dist != "u01":
        raise ValueError(layer.in_dist)
    return x.numpy(), w.numpy()


def make_integer_inputs(layer: Layer, N: int | None = None, amp: int = 4):
    """Small-integer fp32 inputs (|v| <= amp): every partial sum is exact in fp32
    as long as C*R*S*amp*amp < 2**24, so any summation order gives the same bits."""
    rng = np.random.default_rng(layer.seed + 7)
    n = layer.N if N is None else min(N, layer.N)
    x = rng.integers(-amp, amp + 1, size=(n, layer.C, layer.H, layer.W)).astype(np.float32)
    w = rng.integers(-amp, amp + 1, size=(layer.K, layer.C, layer.R, layer.S)).astype(np.float32)
    return x, w


def sample_points(layer: Layer, npts: int, N: int | None = None, seed: int = 12345) -> np.ndarray:
    """Seeded (n,k,p,q) sample, int32 [npts,4], always including the four corners
    and the last element of the output."""
    n = layer.N if N is None else min(N, layer.N)
    rng = np.random.default_rng(seed + layer.seed)
    pts = np.stack([rng.integers(0, n, npts), rng.integers(0, layer.K, npts),
                    rng.integers(0, layer.P, npts), rng.integers(0, layer.Q, npts)], axis=1)
    fixed = [(0, 0, 0, 0), (n - 1, layer.K - 1, layer.P - 1, layer.Q - 1),
             (0, 0, 0, layer.Q - 1), (0, 0, layer.P - 1, 0), (n - 1, 0, layer.P - 1, layer.Q - 1)]
    pts[: len(fixed)] = np.array(fixed)
    return pts.astype(np.int32)

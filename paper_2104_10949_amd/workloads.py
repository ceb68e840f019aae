"""Seeded synthetic workloads: layer shapes of the five benchmark configurations
and the random draws that fill them.

This module holds shapes and random numbers only.  It does none of the
method's arithmetic (no encoding, no sharing, no ring products), so both the
GPU tests and the CPU oracle can take their inputs from it without sharing any
computation.  Share tensors are uniform on Z_{2^64} whatever the plaintext
(paper Sec. III-B, "Secret sharing": two of the three shares are sampled
uniformly), so a party's operands for timing and bit-exactness checks are drawn
directly as uniform 64-bit words.

The datasets the paper trains on (MNIST, CIFAR-10, Tiny ImageNet, ImageNet;
Sec. V "Deep learning datasets") are not used: tensors of the same shapes stand
in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

BASE_SEED = 20210422
FRAC_BITS = 16  # fixed-point fractional bits of the benchmark configurations


@dataclass(frozen=True)
class Layer:
    """One linear layer as the library sees it.

    kind == "matmul": X [M,K] times Y [N,K]^T.
    kind == "conv":   X NHWC [B,H,W,Cin], weights [Cout,kh,kw,Cin], stride, pad.
    """
    name: str
    kind: str
    M: int = 0
    N: int = 0
    K: int = 0
    B: int = 0
    H: int = 0
    W: int = 0
    Cin: int = 0
    Cout: int = 0
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: int = 0
    x_dist: Tuple[str, float, float] = ("uniform", 0.0, 1.0)
    w_dist: Tuple[str, float, float] = ("normal", 0.0, 0.05)
    repeat: int = 1  # how many layers of exactly this shape the network has

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def gemm(self) -> Tuple[int, int, int]:
        """(M, N, K) of the layer seen as one matrix product."""
        if self.kind == "matmul":
            return self.M, self.N, self.K
        return self.B * self.Ho * self.Wo, self.Cout, self.kh * self.kw * self.Cin

    @property
    def mnk(self) -> int:
        m, n, k = self.gemm
        return m * n * k

    @property
    def x_shape(self) -> Tuple[int, ...]:
        return (self.M, self.K) if self.kind == "matmul" else (self.B, self.H, self.W, self.Cin)

    @property
    def w_shape(self) -> Tuple[int, ...]:
        return (self.N, self.K) if self.kind == "matmul" else (self.Cout, self.kh, self.kw, self.Cin)

    @property
    def z_shape(self) -> Tuple[int, ...]:
        return (self.M, self.N) if self.kind == "matmul" else (self.B, self.Ho, self.Wo, self.Cout)

    @property
    def algorithmic_bytes(self) -> int:
        """Bytes one party's local product must move: both share tensors of each
        operand read once, the output written once, 8 bytes per ring element."""
        nx = int(np.prod(self.x_shape))
        nw = int(np.prod(self.w_shape))
        nz = int(np.prod(self.z_shape))
        return 8 * (2 * nx + 2 * nw + nz)


def _fc(name, M, N, K, **kw) -> Layer:
    return Layer(name=name, kind="matmul", M=M, N=N, K=K, **kw)


def _conv(name, B, HW, Cin, Cout, k, stride=1, pad=0, **kw) -> Layer:
    return Layer(name=name, kind="conv", B=B, H=HW, W=HW, Cin=Cin, Cout=Cout, kh=k, kw=k,
                 stride=stride, pad=pad, **kw)


def config1() -> List[Layer]:
    n01 = ("normal", 0.0, 1.0)
    return [_fc("matmul256", 256, 256, 256, x_dist=n01, w_dist=n01)]


def config2() -> List[Layer]:
    return [_fc("fc1", 128, 128, 784), _fc("fc2", 128, 128, 128), _fc("fc3", 128, 10, 128)]


def config3(alt: bool = False) -> List[Layer]:
    """Small CNN, batch 128.  The default reading runs the second 5x5 conv at
    32x32; alt=True runs it after a 2x2 pooling, at 16x16."""
    hw2 = 16 if alt else 32
    return [_conv("conv1_5x5_3_64", 128, 32, 3, 64, 5, pad=2),
            _conv("conv2_5x5_64_64", 128, hw2, 64, 64, 5, pad=2),
            _conv("conv3_3x3_64_128", 128, 16, 64, 128, 3, pad=1)]


def config4() -> List[Layer]:
    w = ("normal", 0.0, 0.02)
    B = 32
    plan = [(64, [(3, 64), (64, 64)]), (32, [(64, 128), (128, 128)]),
            (16, [(128, 256), (256, 256), (256, 256)]),
            (8, [(256, 512), (512, 512), (512, 512)]),
            (4, [(512, 512), (512, 512), (512, 512)])]
    out: List[Layer] = []
    for bi, (hw, convs) in enumerate(plan, 1):
        for ci, (cin, cout) in enumerate(convs, 1):
            out.append(_conv(f"b{bi}c{ci}_{hw}_{cin}_{cout}", B, hw, cin, cout, 3, pad=1, w_dist=w))
    out += [_fc("fc1", B, 512, 8192, w_dist=w), _fc("fc2", B, 512, 512, w_dist=w),
            _fc("fc3", B, 200, 512, w_dist=w)]
    return out


def config5() -> List[Layer]:
    """ResNet-50-shaped layer set, batch 8, 224x224x3: 53 convolutions + 1 FC.
    Stride 2 sits on the 3x3 conv of the first block of stages 2-4; every stage's
    first block has a 1x1 projection shortcut with the stage's stride.  Layers of
    identical shape are listed once with a repeat count."""
    w = ("normal", 0.0, 0.02)
    B = 8
    out: List[Layer] = [_conv("stem_7x7s2_3_64", B, 224, 3, 64, 7, stride=2, pad=3, w_dist=w)]
    hw, cin = 56, 64
    for stage, (width, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], 1):
        s = 1 if stage == 1 else 2
        cout = 4 * width
        hwo = hw // s
        p = f"s{stage}"
        out.append(_conv(f"{p}b1_1x1a_{cin}_{width}", B, hw, cin, width, 1, w_dist=w))
        out.append(_conv(f"{p}b1_3x3s{s}_{width}", B, hw, width, width, 3, stride=s, pad=1, w_dist=w))
        out.append(_conv(f"{p}b1_1x1b_{width}_{cout}", B, hwo, width, cout, 1, w_dist=w))
        out.append(_conv(f"{p}b1_proj_s{s}_{cin}_{cout}", B, hw, cin, cout, 1, stride=s, w_dist=w))
        r = blocks - 1
        out.append(_conv(f"{p}bx_1x1a_{cout}_{width}", B, hwo, cout, width, 1, w_dist=w, repeat=r))
        out.append(_conv(f"{p}bx_3x3_{width}", B, hwo, width, width, 3, pad=1, w_dist=w, repeat=r))
        out.append(_conv(f"{p}bx_1x1b_{width}_{cout}", B, hwo, width, cout, 1, w_dist=w, repeat=r))
        hw, cin = hwo, cout
    out.append(_fc("fc", B, 1000, 2048, w_dist=w))
    return out


def config_layers(index: int) -> List[Layer]:
    """Layers of benchmark configuration `index` (1-based, in the order of the benchmark definition)."""
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[index]()


def layer_seed(config: int, layer_index: int) -> int:
    return BASE_SEED + 1000 * config + layer_index


def draw_ring(shape, seed: int) -> np.ndarray:
    """Uniform words of Z_{2^64}."""
    rng = np.random.default_rng(seed)
    return rng.integers(0, 1 << 64, size=shape, dtype=np.uint64, endpoint=False)


def draw_reals(shape, dist: Tuple[str, float, float], seed: int) -> np.ndarray:
    """fp64 reals: ("normal", mean, std) or ("uniform", lo, hi)."""
    rng = np.random.default_rng(seed)
    kind, a, b = dist
    if kind == "normal":
        return rng.normal(a, b, size=shape)
    if kind == "uniform":
        return rng.uniform(a, b, size=shape)
    raise ValueError(kind)


def party_operands(layer: Layer, seed: int):
    """The four share tensors one party holds for a layer, (x_i, x_{i+1}, w_i, w_{i+1}),
    each uniform on the ring."""
    return (draw_ring(layer.x_shape, seed), draw_ring(layer.x_shape, seed + 101),
            draw_ring(layer.w_shape, seed + 202), draw_ring(layer.w_shape, seed + 303))


# Byte patterns that stress signed-limb carries and accumulator bounds.
ADVERSARIAL_WORDS = (0x8080808080808080, 0xFFFFFFFFFFFFFFFF, 0x7F7F7F7F7F7F7F7F,
                     0x0000000000000000, 0x0000000000000001, 0x8000000000000000,
                     0x00000000FFFFFFFF, 0x0100000000000000, 0x80FF7F0080FF7F00)

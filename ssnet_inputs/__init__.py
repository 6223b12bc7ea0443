"""Seeded synthetic inputs and workload shapes.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmarks.  It holds no field arithmetic, no sharing, no fixed-point
encoding: only random draws of plain floats / plain integers below a bound,
and the table of layer shapes that defines the ResNet-shaped workloads.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import numpy as np

P61 = (1 << 61) - 1


def gaussian(shape, seed: int) -> np.ndarray:
    """float64 N(0,1) samples of the given shape."""
    return np.random.default_rng(seed).standard_normal(size=shape)


def he_normal(shape, fan_in: int, seed: int) -> np.ndarray:
    """float64 N(0, 2/fan_in) samples (He-normal initialisation)."""
    return np.random.default_rng(seed).standard_normal(size=shape) * np.sqrt(2.0 / fan_in)


def uniform_below(count: int, bound: int, seed: int) -> np.ndarray:
    """uint64 samples, uniform on [0, bound)."""
    return np.random.default_rng(seed).integers(0, bound, size=count, dtype=np.uint64)


@dataclass(frozen=True)
class Layer:
    """One linear layer of a sequential chain (all convs are square, NCHW)."""
    kind: str            # "conv" or "fc"
    cin: int
    cout: int
    ksize: int
    stride: int
    pad: int
    hin: int             # input spatial size (square); 1 for fc
    hout: int
    post: Optional[str]  # plaintext step applied by the harness after this layer:
    #                      "relu", "relu+gap" (global average), "relu+maxpool{k}s{s}[p{pad}]",
    #                      "relu+avgpool{k}s{s}", or None (last layer); see pooling_of

    @property
    def M(self) -> int:
        return self.hout * self.hout

    @property
    def K(self) -> int:
        return self.cin * self.ksize * self.ksize

    @property
    def N(self) -> int:
        return self.cout

    @property
    def macs(self) -> int:
        return self.M * self.K * self.N


def pooling_of(L: Layer):
    """The pooling that follows layer L's ReLU: None, or (kind, kernel, stride, pad) with kind "max" or "avg"
    (square kernels; "relu+maxpool3s2" is the ResNet stem's 3x3 / 2 with padding 1)."""
    post = L.post
    if post in (None, "relu"):
        return None
    if post == "relu+gap":
        return ("avg", L.hout, L.hout, 0)
    if post == "relu+maxpool3s2":
        return ("max", 3, 2, 1)
    import re
    m = re.fullmatch(r"relu\+(max|avg)pool(\d+)s(\d+)(?:p(\d+))?", post)
    if not m:
        raise ValueError(post)
    return (m.group(1), int(m.group(2)), int(m.group(3)), int(m.group(4) or 0))


def resnet_chain(depth: int, image: int = 224, classes: int = 1000) -> List[Layer]:
    """Main-path layers of a bottleneck ResNet as one sequential chain.

    conv1 7x7/2 (3->64), 3x3/2 max-pool, four stages of bottleneck blocks
    (1x1 -> 3x3 -> 1x1 x4; stride 2 sits on the 3x3 of the first block of
    stages 2-4), global average pool, fully connected layer.  Projection
    shortcuts and residual additions are left out: the chain is the sequence
    of conv/FC layers only (50 layers for depth 50, 152 for depth 152).
    """
    blocks = {50: (3, 4, 6, 3), 101: (3, 4, 23, 3), 152: (3, 8, 36, 3)}[depth]
    layers: List[Layer] = []
    h = image
    hout = (h + 2 * 3 - 7) // 2 + 1
    layers.append(Layer("conv", 3, 64, 7, 2, 3, h, hout, "relu+maxpool3s2"))
    h = (hout + 2 * 1 - 3) // 2 + 1
    cin = 64
    for stage, (nblocks, width) in enumerate(zip(blocks, (64, 128, 256, 512))):
        for b in range(nblocks):
            stride = 2 if (stage > 0 and b == 0) else 1
            layers.append(Layer("conv", cin, width, 1, 1, 0, h, h, "relu"))
            h2 = (h + 2 - 3) // stride + 1
            layers.append(Layer("conv", width, width, 3, stride, 1, h, h2, "relu"))
            h = h2
            last = stage == 3 and b == nblocks - 1
            layers.append(Layer("conv", width, 4 * width, 1, 1, 0, h, h,
                                "relu+gap" if last else "relu"))
            cin = 4 * width
    layers.append(Layer("fc", cin, classes, 1, 1, 0, 1, 1, None))
    return layers


def vgg16_chain(image: int = 32, classes: int = 10, hidden: int = 4096) -> List[Layer]:
    """Layers of a VGG16-shaped network for small images (the paper evaluates VGG16 on 32x32 and 64x64
    inputs): thirteen 3x3 convolutions of widths 64,64 | 128,128 | 256x3 | 512x3 | 512x3, a 2x2 / 2 max-pool
    after each group, then three dense layers.  No bias, no BatchNorm; 16 layers."""
    layers: List[Layer] = []
    h, cin = image, 3
    for width, reps in ((64, 2), (128, 2), (256, 3), (512, 3), (512, 3)):
        for r in range(reps):
            layers.append(Layer("conv", cin, width, 3, 1, 1, h, h, "relu+maxpool2s2" if r == reps - 1 else "relu"))
            cin = width
        h //= 2
    feat = cin * h * h
    layers.append(Layer("fc", feat, hidden, 1, 1, 0, 1, 1, "relu"))
    layers.append(Layer("fc", hidden, hidden, 1, 1, 0, 1, 1, "relu"))
    layers.append(Layer("fc", hidden, classes, 1, 1, 0, 1, 1, None))
    return layers


def resnet_basic_chain(depth: int = 18, image: int = 224, classes: int = 1000) -> List[Layer]:
    """Main-path layers of a basic-block ResNet (18 or 34) as one sequential chain: conv1 7x7/2, 3x3/2
    max-pool, stages of two 3x3 convolutions per block (stride 2 on the first convolution of stages 2-4),
    global average, dense layer.  No shortcuts, as in resnet_chain."""
    blocks = {18: (2, 2, 2, 2), 34: (3, 4, 6, 3)}[depth]
    layers: List[Layer] = []
    hout = (image + 2 * 3 - 7) // 2 + 1
    layers.append(Layer("conv", 3, 64, 7, 2, 3, image, hout, "relu+maxpool3s2"))
    h, cin = (hout + 2 - 3) // 2 + 1, 64
    for stage, (nblocks, width) in enumerate(zip(blocks, (64, 128, 256, 512))):
        for b in range(nblocks):
            stride = 2 if (stage > 0 and b == 0) else 1
            h2 = (h + 2 - 3) // stride + 1
            layers.append(Layer("conv", cin, width, 3, stride, 1, h, h2, "relu"))
            last = stage == 3 and b == nblocks - 1
            layers.append(Layer("conv", width, width, 3, 1, 1, h2, h2, "relu+gap" if last else "relu"))
            h, cin = h2, width
    layers.append(Layer("fc", cin, classes, 1, 1, 0, 1, 1, None))
    return layers


def lenet_chain(image: int = 28, classes: int = 10) -> List[Layer]:
    """LeNet-5-shaped stack for 28x28 one-channel images: 5x5 convolutions (1 -> 6, padding 2; 6 -> 16), each
    followed by ReLU and a 2x2 / 2 average pool, then dense layers 120, 84, classes."""
    h1 = image                      # 5x5, padding 2
    h2 = h1 // 2 - 4                # after the pool, then 5x5 without padding
    feat = 16 * (h2 // 2) * (h2 // 2)
    return [Layer("conv", 1, 6, 5, 1, 2, image, h1, "relu+avgpool2s2"),
            Layer("conv", 6, 16, 5, 1, 0, h1 // 2, h2, "relu+avgpool2s2"),
            Layer("fc", feat, 120, 1, 1, 0, 1, 1, "relu"),
            Layer("fc", 120, 84, 1, 1, 0, 1, 1, "relu"),
            Layer("fc", 84, classes, 1, 1, 0, 1, 1, None)]


def alexnet_chain(image: int = 227, classes: int = 1000, hidden: int = 4096) -> List[Layer]:
    """AlexNet-shaped stack: 11x11 / 4 convolution (3 -> 96), 5x5 (96 -> 256, padding 2), 3x3 convolutions
    384, 384, 256, overlapping 3x3 / 2 max-pools without padding after the first, second and fifth
    convolution, then three dense layers."""
    def pooled(h):
        return (h - 3) // 2 + 1
    h1 = (image - 11) // 4 + 1
    p1 = pooled(h1)
    p2 = pooled(p1)
    p3 = pooled(p2)
    return [Layer("conv", 3, 96, 11, 4, 0, image, h1, "relu+maxpool3s2p0"),
            Layer("conv", 96, 256, 5, 1, 2, p1, p1, "relu+maxpool3s2p0"),
            Layer("conv", 256, 384, 3, 1, 1, p2, p2, "relu"),
            Layer("conv", 384, 384, 3, 1, 1, p2, p2, "relu"),
            Layer("conv", 384, 256, 3, 1, 1, p2, p2, "relu+maxpool3s2p0"),
            Layer("fc", 256 * p3 * p3, hidden, 1, 1, 0, 1, 1, "relu"),
            Layer("fc", hidden, hidden, 1, 1, 0, 1, 1, "relu"),
            Layer("fc", hidden, classes, 1, 1, 0, 1, 1, None)]

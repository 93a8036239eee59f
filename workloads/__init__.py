"""Seeded synthetic workloads: layer shapes and input tensors.

This module holds the layer-shape tables of the benchmark configurations and a
counter-based random generator for their tensors.  It contains none of the
convolution's arithmetic: both the CPU oracle's tests and the HIP path's tests
draw their inputs from here, and nothing else is shared between the two.

The paper measured whole CNNs (LeNet, AlexNet, ResNet, a style-transfer net;
Section 4, Tables 2 and 3) on datasets and trained weights that are not
available; the tensors generated here stand in for them.  They follow the
recipe of the build's configurations: x ~ U[-1, 1], w ~ N(0, std^2) with
std = sqrt(2 / fan_in), fan_in = (C/group) * kernel^2 ("He-normal"),
b ~ U[-0.1, 0.1], every value then rounded to FP16 (round to nearest even).
Tensors are returned as numpy float16 arrays; their bit patterns are what both
sides consume.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np

__all__ = [
    "ConvLayer", "uniform01", "normal01", "make_tensors", "make_integer_tensors",
    "config1", "alexnet", "vgg16", "resnet50", "mobilenet_v1", "CONFIGS",
]


@dataclass(frozen=True)
class ConvLayer:
    """One convolution layer: x[N][C][H][W], w[M][C/G][k][k], b[M] -> y[N][M][Ho][Wo]."""
    name: str
    N: int
    C: int
    H: int
    W: int
    M: int          # num_output
    k: int          # kernel (square)
    s: int = 1      # stride
    p: int = 0      # pad (symmetric, zeros)
    G: int = 1      # group
    bias: int = 1
    relu: int = 1

    @property
    def Ho(self) -> int:
        return (self.H + 2 * self.p - self.k) // self.s + 1

    @property
    def Wo(self) -> int:
        return (self.W + 2 * self.p - self.k) // self.s + 1

    @property
    def Cg(self) -> int:
        return self.C // self.G

    @property
    def Mg(self) -> int:
        return self.M // self.G

    @property
    def Kg(self) -> int:
        return self.Cg * self.k * self.k

    @property
    def P(self) -> int:
        return self.N * self.Ho * self.Wo

    @property
    def x_shape(self) -> Tuple[int, int, int, int]:
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self) -> Tuple[int, int, int, int]:
        return (self.M, self.Cg, self.k, self.k)

    @property
    def y_shape(self) -> Tuple[int, int, int, int]:
        return (self.N, self.M, self.Ho, self.Wo)

    @property
    def flops(self) -> int:
        """2 * MACs, padding taps counted, bias and ReLU not."""
        return 2 * self.N * self.M * self.Cg * self.k * self.k * self.Ho * self.Wo

    @property
    def bytes(self) -> int:
        """Algorithmic bytes: each FP16 tensor touched exactly once."""
        nx = self.N * self.C * self.H * self.W
        nw = self.M * self.Cg * self.k * self.k
        ny = self.N * self.M * self.Ho * self.Wo
        return 2 * (nx + nw + ny + (self.M if self.bias else 0))

    def desc(self) -> Tuple[int, ...]:
        """The eleven int32 fields of the C descriptor, in declaration order."""
        return (self.N, self.C, self.H, self.W, self.M, self.k, self.s, self.p,
                self.G, self.bias, self.relu)

    def with_batch(self, N: int) -> "ConvLayer":
        return replace(self, N=N)


# ---------------------------------------------------------------------------
# Counter-based generator: value i of stream `seed` depends on (seed, i) only,
# so any slice of a tensor can be regenerated anywhere, bit for bit.
# ---------------------------------------------------------------------------
_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)


def _splitmix64(z: np.ndarray) -> np.ndarray:
    """The splitmix64 output function applied to an array of uint64 states."""
    with np.errstate(over="ignore"):
        z = z + np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


def _bits(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    with np.errstate(over="ignore"):
        key = _splitmix64(np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)]))
        key = _splitmix64(key ^ np.uint64(stream))
        ctr = np.arange(offset, offset + count, dtype=np.uint64)
        return _splitmix64(ctr * np.uint64(0xD1342543DE82EF95) + key[0])


def uniform01(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    """`count` float64 values uniform in [0, 1), 53 random bits each."""
    return (_bits(seed, stream, count, offset) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal01(seed: int, stream: int, count: int, offset: int = 0) -> np.ndarray:
    """`count` standard normal float64 values (Box-Muller on two uniform streams)."""
    u1 = uniform01(seed, 2 * stream + 0x100, count, offset)
    u2 = uniform01(seed, 2 * stream + 0x101, count, offset)
    r = np.sqrt(-2.0 * np.log(1.0 - u1))          # 1-u1 in (0, 1]
    return r * np.cos(2.0 * np.pi * u2)


_STREAM_X, _STREAM_W, _STREAM_B = 1, 2, 3


def make_tensors(layer: ConvLayer, seed: int = 0):
    """FP16 (x, w, b) for `layer`; b is None when the layer has no bias."""
    nx = int(np.prod(layer.x_shape))
    nw = int(np.prod(layer.w_shape))
    x = (2.0 * uniform01(seed, _STREAM_X, nx) - 1.0).astype(np.float16).reshape(layer.x_shape)
    std = np.sqrt(2.0 / (layer.Cg * layer.k * layer.k))
    w = (std * normal01(seed, _STREAM_W, nw)).astype(np.float16).reshape(layer.w_shape)
    b = None
    if layer.bias:
        b = (0.2 * uniform01(seed, _STREAM_B, layer.M) - 0.1).astype(np.float16)
    return x, w, b


def make_integer_tensors(layer: ConvLayer, seed: int = 0, xmax: int = 4, wmax: int = 2):
    """Small-integer FP16 tensors: x in [-xmax, xmax], w in [-wmax, wmax], b in [-8, 8].

    With Kg * xmax * wmax + 8 <= 2048 every partial sum is an integer that FP16
    and FP32 hold exactly, so any correct implementation returns the exact result.
    """
    nx = int(np.prod(layer.x_shape))
    nw = int(np.prod(layer.w_shape))
    x = np.floor(uniform01(seed, _STREAM_X, nx) * (2 * xmax + 1)) - xmax
    w = np.floor(uniform01(seed, _STREAM_W, nw) * (2 * wmax + 1)) - wmax
    b = None
    if layer.bias:
        b = (np.floor(uniform01(seed, _STREAM_B, layer.M) * 17) - 8).astype(np.float16)
    return (x.astype(np.float16).reshape(layer.x_shape),
            w.astype(np.float16).reshape(layer.w_shape), b)


# ---------------------------------------------------------------------------
# Layer tables.  Each layer of a "stack" is an independent problem with its own
# seeded input of the stated shape (pooling layers between stages are not part
# of the path; they only explain the spatial sizes).
# ---------------------------------------------------------------------------
def config1() -> List[ConvLayer]:
    return [ConvLayer("cfg1.conv", 1, 3, 32, 32, 16, 3, 1, 1, 1, 1, 1)]


def alexnet(N: int = 1) -> List[ConvLayer]:
    return [
        ConvLayer("alex.conv1", N, 3, 227, 227, 96, 11, 4, 0, 1),
        ConvLayer("alex.conv2", N, 96, 27, 27, 256, 5, 1, 2, 2),
        ConvLayer("alex.conv3", N, 256, 13, 13, 384, 3, 1, 1, 1),
        ConvLayer("alex.conv4", N, 384, 13, 13, 384, 3, 1, 1, 2),
        ConvLayer("alex.conv5", N, 384, 13, 13, 256, 3, 1, 1, 2),
    ]


def vgg16(N: int = 1) -> List[ConvLayer]:
    plan = [(3, 64, 224), (64, 64, 224),
            (64, 128, 112), (128, 128, 112),
            (128, 256, 56), (256, 256, 56), (256, 256, 56),
            (256, 512, 28), (512, 512, 28), (512, 512, 28),
            (512, 512, 14), (512, 512, 14), (512, 512, 14)]
    return [ConvLayer(f"vgg.conv{i + 1}", N, c, hw, hw, m, 3, 1, 1, 1)
            for i, (c, m, hw) in enumerate(plan)]


def resnet50(N: int = 1) -> List[ConvLayer]:
    """The twenty distinct conv shapes of the bottleneck trunk (each once).

    Suffix a = first 1x1, b = 3x3, c = last 1x1 (no ReLU); a0/b0 = first block of
    a stage (its 3x3 carries the stride 2), a' = later blocks of stage 1.
    """
    L = [ConvLayer("res.stem", N, 3, 224, 224, 64, 7, 2, 3, 1)]
    stages = [(1, 64, 56), (2, 128, 28), (3, 256, 14), (4, 512, 7)]
    for s, width, hw in stages:
        cin_first = 64 if s == 1 else 2 * width         # previous stage's output channels
        hw_in = hw if s == 1 else 2 * hw
        if s == 1:
            L.append(ConvLayer("res.s1.a", N, 64, 56, 56, 64, 1))
            L.append(ConvLayer("res.s1.a'", N, 256, 56, 56, 64, 1))
        else:
            L.append(ConvLayer(f"res.s{s}.a0", N, cin_first, hw_in, hw_in, width, 1))
            L.append(ConvLayer(f"res.s{s}.b0", N, width, hw_in, hw_in, width, 3, 2, 1))
            L.append(ConvLayer(f"res.s{s}.a", N, 4 * width, hw, hw, width, 1))
        L.append(ConvLayer(f"res.s{s}.b", N, width, hw, hw, width, 3, 1, 1))
        L.append(ConvLayer(f"res.s{s}.c", N, width, hw, hw, 4 * width, 1, relu=0))
    return L


def mobilenet_v1(N: int = 1) -> List[ConvLayer]:
    L = [ConvLayer("mb.conv1", N, 3, 224, 224, 32, 3, 2, 1, 1)]
    # (input channels, pointwise outputs, depthwise stride, input spatial size)
    plan = [(32, 64, 1, 112), (64, 128, 2, 112), (128, 128, 1, 56), (128, 256, 2, 56),
            (256, 256, 1, 28), (256, 512, 2, 28)] + [(512, 512, 1, 14)] * 5 + \
           [(512, 1024, 2, 14), (1024, 1024, 1, 7)]
    for i, (c, m, s, hw) in enumerate(plan, start=1):
        ho = (hw + 2 - 3) // s + 1
        L.append(ConvLayer(f"mb.dw{i}", N, c, hw, hw, c, 3, s, 1, c))
        L.append(ConvLayer(f"mb.pw{i}", N, c, ho, ho, m, 1))
    return L


CONFIGS: Dict[str, callable] = {
    "cfg1": lambda N=1: config1(),
    "alexnet": alexnet,
    "vgg16": vgg16,
    "resnet50": resnet50,
    "mobilenet_v1": mobilenet_v1,
}


def layer_seed(config: str, index: int) -> int:
    """Seed of layer `index` of a configuration (config 1 uses seed 0)."""
    if config == "cfg1":
        return 0
    base = {"alexnet": 2, "vgg16": 3, "resnet50": 4, "mobilenet_v1": 5}[config]
    return base * 1000 + index

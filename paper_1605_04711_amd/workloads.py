"""Seeded synthetic inputs and layer-shape tables for the paper's workloads.

This module holds NO arithmetic of the method: it only draws random tensors
(numpy PCG64, seed = 160504711 + 1000*config + tensor_index), rounds
activations to bf16 where a workload is bf16, and lists the convolution /
fully-connected shapes of the networks named in Sec. 3.1 (LeNet-5-style, VGG-7,
ResNet-18) plus the stand-alone GEMM and the VGG-16-style detection backbone
that stand in for the paper's MNIST / CIFAR-10 / ImageNet / PASCAL VOC runs.
Weights follow the paper's own modelling assumption (normally distributed,
Sec. 2.3): Kaiming normal N(0, 2/fan_in).  It serves both the GPU tests /
benchmark and the CPU oracle's callers; neither side's code lives here.
"""

from dataclasses import dataclass

import numpy as np

BASE_SEED = 160504711
IDX_INPUT = 900
IDX_DY = 901


def rng(config, tensor_index):
    return np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * int(config) + int(tensor_index)))


def f32_to_bf16_bits(a):
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16). Finite inputs."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(a):
    """float32 array whose values are exactly representable in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(a))


def normal(config, tensor_index, shape, std=1.0, chunk=1 << 24):
    g = rng(config, tensor_index)
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        out[lo:hi] = g.standard_normal(hi - lo, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out.reshape(shape)


def uniform01(config, tensor_index, shape):
    return rng(config, tensor_index).random(size=shape, dtype=np.float32)


@dataclass(frozen=True)
class Layer:
    """One ternarized conv / FC layer.  Activations NHWC, filters [O][C][R][S]."""
    name: str
    N: int
    H: int
    W: int
    C: int
    O: int
    R: int = 1
    S: int = 1
    stride: int = 1
    pad: int = 0
    dil: int = 1

    @property
    def P(self):
        return (self.H + 2 * self.pad - self.dil * (self.R - 1) - 1) // self.stride + 1

    @property
    def Q(self):
        return (self.W + 2 * self.pad - self.dil * (self.S - 1) - 1) // self.stride + 1

    @property
    def gemm_mnk(self):
        return (self.N * self.P * self.Q, self.O, self.R * self.S * self.C)

    @property
    def flops(self):
        m, n, k = self.gemm_mnk
        return 2 * m * n * k

    @property
    def n_weights(self):
        return self.O * self.C * self.R * self.S

    @property
    def w_shape(self):
        return (self.O, self.C, self.R, self.S)

    @property
    def x_shape(self):
        return (self.N, self.H, self.W, self.C)

    @property
    def y_shape(self):
        return (self.N, self.P, self.Q, self.O)

    def with_batch(self, n):
        return Layer(self.name, n, self.H, self.W, self.C, self.O, self.R, self.S,
                     self.stride, self.pad, self.dil)


def kaiming_weights(config, layer_index, layer):
    fan_in = layer.C * layer.R * layer.S
    return normal(config, layer_index, layer.w_shape, std=float(np.sqrt(2.0 / fan_in)))


def lenet5(batch=64):
    """32-C5 + MP2 + 64-C5 + MP2 + 512 FC + 10 (Sec. 3.1, MNIST); 5x5, stride 1, no padding."""
    return [
        Layer("conv1", batch, 28, 28, 1, 32, 5, 5),
        Layer("conv2", batch, 12, 12, 32, 64, 5, 5),
        Layer("fc1", batch, 1, 1, 1024, 512),
        Layer("fc2", batch, 1, 1, 512, 10),
    ]


def vgg7(batch=128):
    """2x(128-C3) + MP2 + 2x(256-C3) + MP2 + 2x(512-C3) + MP2 + 1024-FC + 10 (Sec. 3.1, CIFAR-10)."""
    return [
        Layer("c1", batch, 32, 32, 3, 128, 3, 3, 1, 1),
        Layer("c2", batch, 32, 32, 128, 128, 3, 3, 1, 1),
        Layer("c3", batch, 16, 16, 128, 256, 3, 3, 1, 1),
        Layer("c4", batch, 16, 16, 256, 256, 3, 3, 1, 1),
        Layer("c5", batch, 8, 8, 256, 512, 3, 3, 1, 1),
        Layer("c6", batch, 8, 8, 512, 512, 3, 3, 1, 1),
        Layer("fc1", batch, 1, 1, 8192, 1024),
        Layer("fc2", batch, 1, 1, 1024, 10),
    ]


def resnet18(batch=64, width_mult=1.0):
    """ResNet-18 basic blocks (Sec. 3.1, ImageNet); width_mult=1.5 gives ResNet-18B."""
    w = [int(round(c * width_mult)) for c in (64, 128, 256, 512)]
    layers = [Layer("stem", batch, 224, 224, 3, w[0], 7, 7, 2, 3)]
    hw, cin = 56, w[0]
    for si, cout in enumerate(w):
        for bi in range(2):
            stride = 2 if (si > 0 and bi == 0) else 1
            layers.append(Layer(f"l{si+1}.{bi}.conv1", batch, hw, hw, cin, cout, 3, 3, stride, 1))
            if stride == 2 or cin != cout:
                layers.append(Layer(f"l{si+1}.{bi}.down", batch, hw, hw, cin, cout, 1, 1, stride, 0))
            hw = hw // stride
            layers.append(Layer(f"l{si+1}.{bi}.conv2", batch, hw, hw, cout, cout, 3, 3, 1, 1))
            cin = cout
    layers.append(Layer("fc", batch, 1, 1, cin, 1000))
    return layers


def gemm_config():
    """Stand-alone ternary GEMM: X [8192 x 4096] bf16, W [4096 x 4096]."""
    return Layer("gemm", 8192, 1, 1, 4096, 4096)


def vgg16_ssd(batch=32):
    """VGG-16-style detection backbone (300x300), the stand-in for the detection workload."""
    cfg = [(300, 3, 64), (300, 64, 64), (150, 64, 128), (150, 128, 128),
           (75, 128, 256), (75, 256, 256), (75, 256, 256),
           (38, 256, 512), (38, 512, 512), (38, 512, 512),
           (19, 512, 512), (19, 512, 512), (19, 512, 512)]
    layers = [Layer(f"conv{i+1}", batch, hw, hw, ci, co, 3, 3, 1, 1) for i, (hw, ci, co) in enumerate(cfg)]
    layers.append(Layer("fc6", batch, 19, 19, 512, 1024, 3, 3, 1, 6, 6))
    layers.append(Layer("fc7", batch, 19, 19, 1024, 1024, 1, 1))
    return layers


CONFIGS = {0: lenet5, 1: vgg7, 2: resnet18, 4: vgg16_ssd}

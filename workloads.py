"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws numbers.  It holds none of the method's arithmetic
(no quantizer, no contraction, no histogram): the CPU oracle and the HIP path
each receive the same arrays from here and do everything else on their own.

The tensors stand in for CIFAR-10/100 batches and trained AlexNet / ResNet
weights (Sec. 4.1 of the paper), which are not available: only shapes and value
distributions are reproduced.  Layouts: activations NHWC, weights KRSC
(Cout, R, S, Cin), both row-major; GEMM operands row-major.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def _rng(seed: int, tensor_id: int) -> np.random.Generator:
    # one independent stream per (config seed, tensor id)
    return np.random.Generator(np.random.PCG64([int(seed), int(tensor_id)]))


def normal(shape, std: float, seed: int, tensor_id: int = 0) -> np.ndarray:
    return (_rng(seed, tensor_id).standard_normal(shape) * std).astype(np.float32)


def relu_normal(shape, seed: int, tensor_id: int = 0) -> np.ndarray:
    """Post-ReLU activations: max(N(0,1), 0)."""
    x = _rng(seed, tensor_id).standard_normal(shape).astype(np.float32)
    return np.maximum(x, np.float32(0))


def he_normal_weights(k: int, r: int, s: int, c: int, seed: int, tensor_id: int = 0,
                      zero_frac: float = 0.0) -> np.ndarray:
    """KRSC weights ~ N(0, 2/fan_in) with an independent Bernoulli(zero_frac) mask of exact zeros."""
    g = _rng(seed, tensor_id)
    w = (g.standard_normal((k, r, s, c)) * np.sqrt(2.0 / (r * s * c))).astype(np.float32)
    if zero_frac > 0.0:
        w[g.random((k, r, s, c)) < zero_frac] = np.float32(0)
    return w


@dataclass
class ConvShape:
    n: int
    h: int
    w: int
    c: int
    k: int
    r: int = 3
    s: int = 3
    stride: int = 1
    pad: int = 1

    @property
    def p(self) -> int:
        return (self.h + 2 * self.pad - self.r) // self.stride + 1

    @property
    def q(self) -> int:
        return (self.w + 2 * self.pad - self.s) // self.stride + 1

    @property
    def macs(self) -> int:
        return self.n * self.p * self.q * self.k * self.r * self.s * self.c


@dataclass
class ConvLayerInputs:
    shape: ConvShape
    x: np.ndarray      # fp32 NHWC
    w: np.ndarray      # fp32 KRSC
    dy: np.ndarray     # fp32 N,P,Q,K
    wl: int
    fl: int
    name: str = ""


def conv_layer(shape: ConvShape, wl: int, fl: int, seed: int, zero_frac: float = 0.0,
               name: str = "") -> ConvLayerInputs:
    """X = ReLU(N(0,1)), W ~ He-normal (optionally with exact zeros), dY ~ N(0, 0.25^2)."""
    x = relu_normal((shape.n, shape.h, shape.w, shape.c), seed, 1)
    w = he_normal_weights(shape.k, shape.r, shape.s, shape.c, seed, 2, zero_frac)
    dy = normal((shape.n, shape.p, shape.q, shape.k), 0.25, seed, 3)
    return ConvLayerInputs(shape, x, w, dy, wl, fl, name)


# ---- the five benchmark configurations ------------------------------------------------------

def config1_gemm(seed: int = 0):
    """A, B fp32[256,256] ~ N(0, 0.05^2); quantized to <8,6>."""
    return normal((256, 256), 0.05, seed, 1), normal((256, 256), 0.05, seed, 2)


def config1_kld_tensor(seed: int = 0, n: int = 65536) -> np.ndarray:
    """Weight tensor of 65,536 values ~ N(0, 0.05^2); searched over WL 2..16, il=2, 2048 bins."""
    return normal((n,), 0.05, seed, 3)


def config2(batch: int = 128, seed: int = 2) -> ConvLayerInputs:
    """AlexNet-CIFAR-style conv: 64ch 16x16 -> 192ch 3x3 s1 p1, all tensors <8,5>."""
    return conv_layer(ConvShape(batch, 16, 16, 64, 192), 8, 5, seed, name="alexnet_conv2")


def config3(batch: int = 256, seed: int = 3) -> ConvLayerInputs:
    """ResNet-18-CIFAR-style block conv: 128->128 3x3 at 16x16, 50% zero weights, <12,9>."""
    return conv_layer(ConvShape(batch, 16, 16, 128, 128), 12, 9, seed, zero_frac=0.5,
                      name="resnet_block_conv")


@dataclass
class LayerSpec:
    name: str
    shape: ConvShape          # FC layers are 1x1 convs on a 1x1 map
    wl: int
    fl: int
    zero_frac: float = 0.0


def alexnet_cifar_layers(batch: int = 128, seed: int = 4) -> list[LayerSpec]:
    """5 conv + 3 FC layers of an AlexNet-for-CIFAR10 shape; WL per layer drawn from {4,6,8,12,16}."""
    g = _rng(seed, 0)
    shapes = [
        ("conv1", ConvShape(batch, 32, 32, 3, 64)),
        ("conv2", ConvShape(batch, 16, 16, 64, 192)),
        ("conv3", ConvShape(batch, 8, 8, 192, 384)),
        ("conv4", ConvShape(batch, 8, 8, 384, 256)),
        ("conv5", ConvShape(batch, 8, 8, 256, 256)),
        ("fc6", ConvShape(batch, 1, 1, 4096, 4096, 1, 1, 1, 0)),
        ("fc7", ConvShape(batch, 1, 1, 4096, 4096, 1, 1, 1, 0)),
        ("fc8", ConvShape(batch, 1, 1, 4096, 10, 1, 1, 1, 0)),
    ]
    out = []
    for name, shp in shapes:
        wl = int(g.choice([4, 6, 8, 12, 16]))
        out.append(LayerSpec(name, shp, wl, wl - 3))
    return out


def alexnet_cifar_chain(batch: int = 128, seed: int = 4):
    """The same eight layers as a feed-forward chain: (spec, relu, pool) per layer; 2x2/2 max-pooling after
    conv1, conv2 and conv5 takes 32x32 down to the 4x4x256 = 4096 inputs of fc6; no ReLU on the logits."""
    pooled = {"conv1", "conv2", "conv5"}
    return [(sp, sp.name != "fc8", sp.name in pooled) for sp in alexnet_cifar_layers(batch, seed)]


def resnet18_cifar_layers(batch: int = 256, seed: int = 5) -> list[LayerSpec]:
    """ResNet-18 at CIFAR resolution (about 11.2 M weights), 30% zero weights, WL uniform in 4..16."""
    g = _rng(seed, 0)
    shapes = [("stem", ConvShape(batch, 32, 32, 3, 64))]
    cin, res = 64, 32
    for stage, cout in enumerate([64, 128, 256, 512]):
        for block in range(2):
            stride = 2 if (stage > 0 and block == 0) else 1
            shapes.append((f"s{stage}b{block}c1", ConvShape(batch, res, res, cin, cout, 3, 3, stride, 1)))
            if stride == 2:
                shapes.append((f"s{stage}b{block}proj", ConvShape(batch, res, res, cin, cout, 1, 1, 2, 0)))
                res //= 2
            shapes.append((f"s{stage}b{block}c2", ConvShape(batch, res, res, cout, cout, 3, 3, 1, 1)))
            cin = cout
    shapes.append(("fc", ConvShape(batch, 1, 1, 512, 100, 1, 1, 1, 0)))
    out = []
    for name, shp in shapes:
        wl = int(g.integers(4, 17))
        out.append(LayerSpec(name, shp, wl, wl - 3, 0.3))
    return out


def resnet18_cifar_graph(batch: int = 256, seed: int = 5):
    """The same 21 layers as the graph of a residual network: per layer (spec, relu, bn, src, res, gap), src / res the
    indices of the layer that feeds the convolution and of the shortcut that joins after its batch norm (-1: the layer
    before / none).  Basic blocks conv-bn-relu-conv-bn(+shortcut)-relu; the first block of stages 1-3 halves the map
    with stride 2 and a 1x1 projection on the shortcut; global average pooling before the fully connected layer."""
    specs = {sp.name: (i, sp) for i, sp in enumerate(resnet18_cifar_layers(batch, seed))}
    out = [None] * len(specs)
    out[0] = (specs["stem"][1], True, True, -1, -1, False)
    last = 0
    for stage in range(4):
        for block in range(2):
            i1, s1 = specs[f"s{stage}b{block}c1"]
            i2, s2 = specs[f"s{stage}b{block}c2"]
            out[i1] = (s1, True, True, last, -1, False)
            short = last
            if f"s{stage}b{block}proj" in specs:
                ip, sp = specs[f"s{stage}b{block}proj"]
                out[ip] = (sp, False, True, last, -1, False)
                short = ip
            out[i2] = (s2, True, True, i1, short, stage == 3 and block == 1)
            last = i2
    ifc, sfc = specs["fc"]
    out[ifc] = (sfc, False, False, last, -1, False)
    return out


def layer_inputs(spec: LayerSpec, seed: int) -> ConvLayerInputs:
    return conv_layer(spec.shape, spec.wl, spec.fl, seed, spec.zero_frac, spec.name)

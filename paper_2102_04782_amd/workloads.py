"""Seeded synthetic workloads: layer shapes and input tensors.

This module holds NONE of the method's arithmetic (no quantizer, no statistics,
no convolution).  It only says which layers are measured and draws their fp32
inputs, so that the HIP path and the CPU oracle can be fed the same tensors.

The inputs stand in for the ImageNet ResNet-50 / MobileNetV2 gradients the
paper measures on (its per-channel gradient histograms show two shapes, a bell
and a sharp peak with a long tail; its speed figures use ResNet-50 conv layers
at batch 64).  Recipe:

* dY: even channels N(0, sigma_c); odd channels Laplace(0, b_c) with an
  independent 1 % of entries multiplied by 50 (the long tail);
  sigma_c, b_c = 10 ** U[-4, -1].
* clip state from "the previous iteration": rho_c * max|dY_c|, rho_c ~ U[0.5, 1].
* X: N(0,1) for the small case, |N(0,1)| (post-ReLU) otherwise.
* W: N(0, 0.1) for the small case, Kaiming-normal std = sqrt(2 / (Cout*kH*kW)) otherwise.
* seed = 20210204 * 1000 + 100 * config + layer index.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List

import numpy as np


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    Cin: int
    Hin: int
    Win: int
    Cout: int
    kH: int
    kW: int
    stride: int = 1
    pad: int = 0
    dil: int = 1
    groups: int = 1

    @property
    def Ho(self) -> int:
        return (self.Hin + 2 * self.pad - self.dil * (self.kH - 1) - 1) // self.stride + 1

    @property
    def Wo(self) -> int:
        return (self.Win + 2 * self.pad - self.dil * (self.kW - 1) - 1) // self.stride + 1

    @property
    def x_shape(self):
        return (self.N, self.Cin, self.Hin, self.Win)

    @property
    def w_shape(self):
        return (self.Cout, self.Cin // self.groups, self.kH, self.kW)

    @property
    def y_shape(self):
        return (self.N, self.Cout, self.Ho, self.Wo)

    @property
    def macs(self) -> int:
        """True multiply-accumulates of one of the three convolutions (padding taps counted)."""
        return self.N * self.Ho * self.Wo * self.Cout * (self.Cin // self.groups) * self.kH * self.kW

    def desc_fields(self):
        """The 14 integers of a convolution descriptor, in declaration order."""
        return (self.N, self.Cin, self.Hin, self.Win, self.Cout, self.kH, self.kW, self.stride, self.stride, self.pad,
                self.pad, self.dil, self.dil, self.groups)


def seed_for(config: int, layer_index: int = 0) -> int:
    return 20210204 * 1000 + 100 * config + layer_index


# --------------------------------------------------------------------------- layer tables

def config1() -> List[Layer]:
    return [Layer("tiny3x3", 4, 16, 16, 16, 16, 3, 3, 1, 1)]


def config2() -> List[Layer]:
    return [Layer("res2_3x3", 32, 64, 56, 56, 64, 3, 3, 1, 1)]


def config3() -> List[Layer]:
    return [
        Layer("res5_3x3", 128, 512, 7, 7, 512, 3, 3, 1, 1),
        Layer("res5_1x1_2048_512", 128, 2048, 7, 7, 512, 1, 1, 1, 0),
        Layer("res5_1x1_512_2048", 128, 512, 7, 7, 2048, 1, 1, 1, 0),
    ]


def resnet50(N: int = 64) -> List[Layer]:
    """ResNet-50, bottleneck [3,4,6,3], 224x224 input; stride 2 sits on the 3x3 of the first block of
    stages 2-4 and on the 1x1 shortcut projection.  1 + 16*3 + 4 = 53 convolutions."""
    layers = [Layer("stem7x7", N, 3, 224, 224, 64, 7, 7, 2, 3)]
    cin, hw = 64, 56
    for stage, (mid, blocks) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], start=2):
        cout = mid * 4
        for b in range(blocks):
            s = 2 if (b == 0 and stage > 2) else 1
            tag = f"res{stage}{chr(ord('a') + b)}"
            layers.append(Layer(f"{tag}_1x1a", N, cin, hw, hw, mid, 1, 1, 1, 0))
            layers.append(Layer(f"{tag}_3x3", N, mid, hw, hw, mid, 3, 3, s, 1))
            hw2 = hw // s
            layers.append(Layer(f"{tag}_1x1b", N, mid, hw2, hw2, cout, 1, 1, 1, 0))
            if b == 0:
                layers.append(Layer(f"{tag}_proj", N, cin, hw, hw, cout, 1, 1, s, 0))
            cin, hw = cout, hw2
    assert len(layers) == 53
    return layers


def config4() -> List[Layer]:
    return resnet50(64)


def mobilenetv2(N: int = 128) -> List[Layer]:
    """MobileNetV2 width 1.0, 224x224: the 17 inverted-residual blocks (t, c, n, s)."""
    cfg = [(1, 16, 1, 1), (6, 24, 2, 2), (6, 32, 3, 2), (6, 64, 4, 2), (6, 96, 3, 1), (6, 160, 3, 2), (6, 320, 1, 1)]
    layers: List[Layer] = []
    cin, hw, blk = 32, 112, 0
    for t, c, n, s in cfg:
        for i in range(n):
            stride = s if i == 0 else 1
            hid = cin * t
            blk += 1
            if t != 1:
                layers.append(Layer(f"b{blk}_expand", N, cin, hw, hw, hid, 1, 1, 1, 0))
            layers.append(Layer(f"b{blk}_dw", N, hid, hw, hw, hid, 3, 3, stride, 1, 1, hid))
            hw2 = (hw + 2 - 3) // stride + 1
            layers.append(Layer(f"b{blk}_project", N, hid, hw2, hw2, c, 1, 1, 1, 0))
            cin, hw = c, hw2
    assert blk == 17 and len(layers) == 50
    return layers


def config5() -> List[Layer]:
    return mobilenetv2(128)


def config_layers(config: int) -> List[Layer]:
    return {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}[config]()


def shrink(layer: Layer, N: int) -> Layer:
    """Same layer at a smaller batch (for oracle-sized parity runs of the big configs)."""
    return replace(layer, N=N)


# --------------------------------------------------------------------------- tensors

def make_dY(layer: Layer, seed: int) -> np.ndarray:
    """Mixed bell-shaped / long-tailed output gradient, fp32 NCHW."""
    rng = np.random.default_rng(seed)
    N, C, H, W = layer.y_shape
    scale = (10.0 ** rng.uniform(-4.0, -1.0, size=C)).astype(np.float64)
    out = np.empty((N, C, H, W), dtype=np.float32)
    for c in range(C):
        if c % 2 == 0:
            v = rng.normal(0.0, scale[c], size=(N, H, W))
        else:
            v = rng.laplace(0.0, scale[c], size=(N, H, W))
            tail = rng.random(size=(N, H, W)) < 0.01
            v = np.where(tail, v * 50.0, v)
        out[:, c] = v.astype(np.float32)
    return out


def make_state(dY: np.ndarray, seed: int) -> np.ndarray:
    """Clip values left by a plausible previous iteration: rho_c * max|dY_c|, rho_c ~ U[0.5, 1]."""
    rng = np.random.default_rng(seed + 7)
    C = dY.shape[1]
    rho = rng.uniform(0.5, 1.0, size=C)
    gmax = np.abs(dY).max(axis=(0, 2, 3)).astype(np.float64)
    return (rho * gmax).astype(np.float32)


def make_X(layer: Layer, seed: int, post_relu: bool = True) -> np.ndarray:
    rng = np.random.default_rng(seed + 1)
    x = rng.standard_normal(size=layer.x_shape, dtype=np.float32)
    return np.abs(x) if post_relu else x


def make_W(layer: Layer, seed: int, kaiming: bool = True) -> np.ndarray:
    rng = np.random.default_rng(seed + 2)
    std = float(np.sqrt(2.0 / (layer.Cout * layer.kH * layer.kW))) if kaiming else 0.1
    return (rng.standard_normal(size=layer.w_shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def make_inputs(config: int, layer_index: int = 0, layer: Layer | None = None):
    """(layer, X, W, dY, s_state) for one layer of a config, host fp32 arrays."""
    if layer is None:
        layer = config_layers(config)[layer_index]
    seed = seed_for(config, layer_index)
    small = config == 1
    X = make_X(layer, seed, post_relu=not small)
    W = make_W(layer, seed, kaiming=not small)
    dY = make_dY(layer, seed)
    st = make_state(dY, seed)
    return layer, X, W, dY, st


def make_dY_device(layer: Layer, seed: int, device="cuda"):
    """Same recipe drawn with torch on the device, for shapes too large to ship from the host.
    Values differ from make_dY (another generator); the distribution does not."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    N, C, H, W = layer.y_shape
    scale = 10.0 ** (torch.rand(C, generator=gen, device=device) * 3.0 - 4.0)
    z = torch.randn((N, C, H, W), generator=gen, device=device)
    # Laplace(0,1) by inverse CDF on odd channels
    u = torch.rand((N, (C + 1) // 2, H, W), generator=gen, device=device) - 0.5
    odd = z[:, 1::2]
    no = odd.shape[1]
    lap = -torch.sign(u[:, :no]) * torch.log1p(-2.0 * u[:, :no].abs().clamp(max=0.4999999))
    tail = torch.rand(lap.shape, generator=gen, device=device) < 0.01
    z[:, 1::2] = torch.where(tail, lap * 50.0, lap)
    z *= scale.view(1, C, 1, 1)
    return z.contiguous()

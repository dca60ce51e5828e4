"""Seeded synthetic inputs for the low-bit convolution path.

This module only draws random tensors and picks clip bounds from their
statistics.  It holds none of the quantizer's or the convolution's arithmetic,
which is why both the GPU tests and the CPU oracle tests may use it.

The tensors stand in for the ImageNet activations and trained weights the
paper ran on (Sec. 4.1, 4.5): only layer shapes and value distributions are
taken -- ResNet-18 and MobileNetV2 from the paper's network list (Sec. 4.1),
with the first convolution (and the final classifier) left in floating
point, as in the paper's experimental setup.

Everything is generated on the CPU with a counter-seeded torch generator, in
NCHW / OIHW float32, so that a CPU checker and the GPU see identical bits.
"""
from dataclasses import dataclass, replace
from typing import List, Tuple

import numpy as np
import torch

BASE_SEED = 190805033


@dataclass(frozen=True)
class ConvLayer:
    """Geometry of one quantized convolution layer."""
    name: str
    N: int
    C_in: int
    H: int
    W: int
    C_out: int
    R: int
    S: int
    stride: int
    pad: int
    bits: int
    count: int = 1          # how many times the network repeats this shape

    @property
    def Ho(self):
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Wo(self):
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def macs(self):
        """Dense multiply-accumulates (padding taps included)."""
        return self.N * self.Ho * self.Wo * self.C_out * self.C_in * self.R * self.S

    def with_(self, **kw):
        return replace(self, **kw)


def _c3(name, N, ci, hw, co, stride=1, bits=4, count=1):
    return ConvLayer(name, N, ci, hw, hw, co, 3, 3, stride, 1, bits, count)


def _c1(name, N, ci, hw, co, stride=1, bits=4, count=1):
    return ConvLayer(name, N, ci, hw, hw, co, 1, 1, stride, 0, bits, count)


def resnet18_layers(N=64, bits=4) -> List[ConvLayer]:
    """The 19 convolutions of ResNet-18 that follow conv1 (224x224 input)."""
    return [
        _c3("r18.s1.3x3.64-64@56", N, 64, 56, 64, 1, bits, 4),
        _c3("r18.s2.3x3s2.64-128@56", N, 64, 56, 128, 2, bits, 1),
        _c3("r18.s2.3x3.128-128@28", N, 128, 28, 128, 1, bits, 3),
        _c1("r18.s2.1x1s2.64-128@56", N, 64, 56, 128, 2, bits, 1),
        _c3("r18.s3.3x3s2.128-256@28", N, 128, 28, 256, 2, bits, 1),
        _c3("r18.s3.3x3.256-256@14", N, 256, 14, 256, 1, bits, 3),
        _c1("r18.s3.1x1s2.128-256@28", N, 128, 28, 256, 2, bits, 1),
        _c3("r18.s4.3x3s2.256-512@14", N, 256, 14, 512, 2, bits, 1),
        _c3("r18.s4.3x3.512-512@7", N, 512, 7, 512, 1, bits, 3),
        _c1("r18.s4.1x1s2.256-512@14", N, 256, 14, 512, 2, bits, 1),
    ]


def mobilenetv2_pointwise_layers(N=64, bits=4) -> List[ConvLayer]:
    """Expansion-6 pointwise pairs of MobileNetV2 at their stage resolutions."""
    return [
        _c1("mbv2.1x1.24-144@56", N, 24, 56, 144, 1, bits),
        _c1("mbv2.1x1.144-24@56", N, 144, 56, 24, 1, bits),
        _c1("mbv2.1x1.96-576@14", N, 96, 14, 576, 1, bits),
        _c1("mbv2.1x1.576-96@14", N, 576, 14, 96, 1, bits),
        _c1("mbv2.1x1.320-1280@7", N, 320, 7, 1280, 1, bits),
    ]


def vgg16_layers(N=32, bits=2) -> List[ConvLayer]:
    """The 12 3x3 convolutions of VGG-16 with C_in >= 64 (224x224 input)."""
    return [
        _c3("vgg.64-64@224", N, 64, 224, 64, 1, bits, 1),
        _c3("vgg.64-128@112", N, 64, 112, 128, 1, bits, 1),
        _c3("vgg.128-128@112", N, 128, 112, 128, 1, bits, 1),
        _c3("vgg.128-256@56", N, 128, 56, 256, 1, bits, 1),
        _c3("vgg.256-256@56", N, 256, 56, 256, 1, bits, 2),
        _c3("vgg.256-512@28", N, 256, 28, 512, 1, bits, 1),
        _c3("vgg.512-512@28", N, 512, 28, 512, 1, bits, 2),
        _c3("vgg.512-512@14", N, 512, 14, 512, 1, bits, 3),
    ]


@dataclass(frozen=True)
class Recipe:
    """How a config draws its tensors and picks its clip bounds."""
    act: str            # "relu_normal" | "half_normal"
    act_bounds: str     # "fixed" | "percentile"
    act_arg: Tuple[float, float]   # (l, u) if fixed; (0, q) if percentile
    w_std: str          # "fixed" | "he"
    w_std_arg: float
    w_bounds: str       # "3sigma" | "abs_percentile" | "minmax"
    w_arg: float = 0.0


CFG1_LAYER = _c3("cfg1.3x3.64-64@32", 1, 64, 32, 64, 1, 4)
CFG2_LAYER = _c3("cfg2.3x3.256-256@14", 32, 256, 14, 256, 1, 4)

RECIPES = {
    1: Recipe("relu_normal", "fixed", (0.0, 3.0), "fixed", 0.05, "3sigma"),
    2: Recipe("half_normal", "fixed", (0.0, 2.5), "fixed", 0.02, "abs_percentile", 99.9),
    3: Recipe("half_normal", "percentile", (0.0, 99.9), "he", 0.0, "abs_percentile", 99.9),
    4: Recipe("half_normal", "percentile", (0.0, 99.9), "he", 0.0, "abs_percentile", 99.9),
    5: Recipe("half_normal", "percentile", (0.0, 99.5), "he", 0.0, "minmax"),
}


def config_layers(cfg: int, bits=None) -> List[ConvLayer]:
    if cfg == 1:
        return [CFG1_LAYER]
    if cfg == 2:
        return [CFG2_LAYER]
    if cfg == 3:
        return resnet18_layers(64, 4 if bits is None else bits)
    if cfg == 4:
        return mobilenetv2_pointwise_layers(64, 4)
    if cfg == 5:
        return vgg16_layers(32, 2)
    raise ValueError("config 1..5")


def layer_seed(cfg: int, layer_index: int) -> int:
    return BASE_SEED + 1000 * cfg + layer_index


def _percentile(t: torch.Tensor, q: float) -> float:
    """q-th percentile (0..100) of a tensor of any size, nearest-rank."""
    flat = t.reshape(-1)
    k = int(np.ceil(q / 100.0 * flat.numel()))
    k = min(max(k, 1), flat.numel())
    return float(torch.kthvalue(flat, k).values)


def make_layer_inputs(layer: ConvLayer, recipe: Recipe, seed: int):
    """Returns dict with x (NCHW f32), w (OIHW f32), l_a, u_a (python floats
    that are exactly float32), l_w, u_w (float32 arrays [C_out])."""
    g = torch.Generator().manual_seed(seed)
    x = torch.randn((layer.N, layer.C_in, layer.H, layer.W), generator=g, dtype=torch.float32)
    if recipe.act == "relu_normal":
        x.clamp_(min=0.0)
    elif recipe.act == "half_normal":
        x.abs_()
    else:
        raise ValueError(recipe.act)
    fan_in = layer.C_in * layer.R * layer.S
    std = recipe.w_std_arg if recipe.w_std == "fixed" else float(np.sqrt(2.0 / fan_in))
    w = torch.randn((layer.C_out, layer.C_in, layer.R, layer.S), generator=g,
                    dtype=torch.float32) * std

    if recipe.act_bounds == "fixed":
        l_a, u_a = recipe.act_arg
    else:
        l_a, u_a = 0.0, _percentile(x, recipe.act_arg[1])
    l_a = float(np.float32(l_a))
    u_a = float(np.float32(u_a))

    wf = w.reshape(layer.C_out, -1)
    if recipe.w_bounds == "3sigma":
        sig = wf.std(dim=1, unbiased=False)
        u_w = (3.0 * sig).numpy().astype(np.float32)
        l_w = (-u_w).astype(np.float32)
    elif recipe.w_bounds == "abs_percentile":
        k = int(np.ceil(recipe.w_arg / 100.0 * wf.shape[1]))
        k = min(max(k, 1), wf.shape[1])
        u_w = torch.kthvalue(wf.abs(), k, dim=1).values.numpy().astype(np.float32)
        l_w = (-u_w).astype(np.float32)
    elif recipe.w_bounds == "minmax":
        l_w = wf.min(dim=1).values.numpy().astype(np.float32)
        u_w = wf.max(dim=1).values.numpy().astype(np.float32)
    else:
        raise ValueError(recipe.w_bounds)
    return {"x": x, "w": w, "l_a": l_a, "u_a": u_a, "l_w": l_w, "u_w": u_w}


def make_config_layer(cfg: int, layer_index: int = 0, bits=None, batch=None):
    """(layer, inputs) for layer ``layer_index`` of config ``cfg``; ``batch``
    overrides N (used to cut big layers down for element-by-element checks)."""
    layer = config_layers(cfg, bits)[layer_index]
    if batch is not None:
        layer = layer.with_(N=batch)
    return layer, make_layer_inputs(layer, RECIPES[cfg], layer_seed(cfg, layer_index))


def small_random_case(seed, N, C_in, H, W, C_out, R, stride, pad, bits,
                      l_a=0.0, u_a=2.5, asym_w=True):
    """A small layer with generic (non-zero l_a, asymmetric weight bounds)
    settings for edge-case tests."""
    layer = ConvLayer("small", N, C_in, H, W, C_out, R, R, stride, pad, bits)
    g = torch.Generator().manual_seed(BASE_SEED + seed)
    x = torch.randn((N, C_in, H, W), generator=g, dtype=torch.float32) * 1.2 + 0.5 * (l_a + u_a)
    w = torch.randn((C_out, C_in, R, R), generator=g, dtype=torch.float32) * 0.1
    wf = w.reshape(C_out, -1)
    if asym_w:
        l_w = (wf.min(dim=1).values * 0.8).numpy().astype(np.float32)
        u_w = (wf.max(dim=1).values * 0.9).numpy().astype(np.float32)
    else:
        u_w = (wf.abs().max(dim=1).values).numpy().astype(np.float32)
        l_w = (-u_w).astype(np.float32)
    return layer, {"x": x, "w": w, "l_a": float(np.float32(l_a)), "u_a": float(np.float32(u_a)),
                   "l_w": l_w, "u_w": u_w}


def affine_params(seed, C_out, shift_std=0.3):
    """Per-channel scale and shift standing in for a folded batch normalisation
    between two quantized layers: scale in [0.5, 1.5] with a few negative
    entries, shift ~ N(0, shift_std^2).  float32 numpy arrays."""
    g = torch.Generator().manual_seed(BASE_SEED + 77 + seed)
    scale = torch.rand(C_out, generator=g, dtype=torch.float32) + 0.5
    flip = torch.rand(C_out, generator=g) < 0.1
    scale = torch.where(flip, -scale, scale)
    shift = torch.randn(C_out, generator=g, dtype=torch.float32) * shift_std
    return scale.numpy().astype(np.float32), shift.numpy().astype(np.float32)


def soft_quant_case(seed, n, l, u):
    """Inputs of the training-mode kernels: a tensor that covers [l, u] with both
    tails (about a tenth of the values clipped on each side) and an upstream
    gradient ~ N(0, 1).  float32 CPU tensors."""
    g = torch.Generator().manual_seed(BASE_SEED + 500 + seed)
    mid, half = 0.5 * (l + u), 0.5 * (u - l)
    x = torch.randn(n, generator=g, dtype=torch.float32) * (0.78 * half) + mid
    grad_y = torch.randn(n, generator=g, dtype=torch.float32)
    return x, grad_y

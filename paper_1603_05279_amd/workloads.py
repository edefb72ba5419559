"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random tensors of the stated shapes and distributions and
lists the layer geometry.  It contains none of the method's arithmetic (no sign, no
scaling factors, no convolution), so the GPU path and the CPU oracle can both be fed
from it without sharing any code of the method.  The tensors stand in for the
activations and weights of the AlexNet and ResNet-18 layers the paper evaluates on
(sec. 4): only the layer shapes are taken from those networks.

All draws use a torch CPU generator seeded with 1000 + config index (+ layer index
for multi-layer configurations), so every machine regenerates identical arrays.
"""
from dataclasses import dataclass
from typing import List, Optional

import numpy as np
import torch

BN_EPS = 1e-5


@dataclass(frozen=True)
class ConvLayer:
    """Geometry of one binary convolution layer: input n x c x h x w, k_out filters c x kh x kw."""
    name: str
    n: int
    c: int
    h: int
    w: int
    k_out: int
    kh: int
    kw: int
    stride: int
    pad: int
    w_std: float
    batchnorm: bool = False

    @property
    def h_out(self):
        return (self.h + 2 * self.pad - self.kh) // self.stride + 1

    @property
    def w_out(self):
        return (self.w + 2 * self.pad - self.kw) // self.stride + 1

    @property
    def bit_macs(self):
        """One binary operation = one +-1 multiply-accumulate; border taps counted as full
        (op count c*N_W*N_I per filter of the efficiency analysis, sec. 4.1)."""
        return self.n * self.k_out * self.h_out * self.w_out * self.c * self.kh * self.kw

    def with_batch(self, n):
        return ConvLayer(self.name, n, self.c, self.h, self.w, self.k_out, self.kh, self.kw,
                         self.stride, self.pad, self.w_std, self.batchnorm)


@dataclass(frozen=True)
class LinearLayer:
    name: str
    batch: int
    in_features: int
    out_features: int
    w_std: float

    @property
    def bit_macs(self):
        return self.batch * self.in_features * self.out_features


# configs[0] .. configs[4] of the benchmark definition
CONFIGS = {
    "tiny": [ConvLayer("tiny_64x14x14_k3", 1, 64, 14, 14, 64, 3, 3, 1, 1, 1.0)],
    "alexnet_conv2": [ConvLayer("alexnet_conv2", 64, 96, 27, 27, 256, 5, 5, 1, 2, 0.05)],
    "alexnet_conv345": [
        ConvLayer("alexnet_conv3", 128, 256, 13, 13, 384, 3, 3, 1, 1, 0.05, True),
        ConvLayer("alexnet_conv4", 128, 384, 13, 13, 384, 3, 3, 1, 1, 0.05, True),
        ConvLayer("alexnet_conv5", 128, 384, 13, 13, 256, 3, 3, 1, 1, 0.05, True),
    ],
    "resnet18": [
        ConvLayer("resnet18_64x56", 256, 64, 56, 56, 64, 3, 3, 1, 1, 0.02),
        ConvLayer("resnet18_128x28", 256, 128, 28, 28, 128, 3, 3, 1, 1, 0.02),
        ConvLayer("resnet18_256x14", 256, 256, 14, 14, 256, 3, 3, 1, 1, 0.02),
        ConvLayer("resnet18_512x7", 256, 512, 7, 7, 512, 3, 3, 1, 1, 0.02),
    ],
    "fc": [LinearLayer("fc_9216x4096", 256, 9216, 4096, 0.01)],
}
CONFIG_INDEX = {"tiny": 0, "alexnet_conv2": 1, "alexnet_conv345": 2, "resnet18": 3, "fc": 4}


def _gen(seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def conv_inputs(layer: ConvLayer, seed: int, batch: Optional[int] = None):
    """Returns dict(x, w, bn_scale, bn_shift) of float32 numpy arrays (bn_* None without BatchNorm).

    x ~ N(0,1) of shape [n][c][h][w]; w ~ N(0, w_std) of shape [k_out][c][kh][kw].
    BatchNorm parameters: gamma ~ U(0.5,1.5), beta ~ N(0,0.1), running mean 0, variance 1,
    eps 1e-5, handed over in the folded inference form scale = gamma/sqrt(var+eps),
    shift = beta - mean*scale (both float32)."""
    g = _gen(seed)
    n = layer.n if batch is None else batch
    x = torch.randn((n, layer.c, layer.h, layer.w), generator=g, dtype=torch.float32)
    w = torch.randn((layer.k_out, layer.c, layer.kh, layer.kw), generator=g, dtype=torch.float32)
    w = w * layer.w_std
    out = {"x": x.numpy(), "w": w.numpy(), "bn_scale": None, "bn_shift": None}
    if layer.batchnorm:
        gamma = torch.rand(layer.c, generator=g, dtype=torch.float32) + 0.5
        beta = torch.randn(layer.c, generator=g, dtype=torch.float32) * 0.1
        mean = torch.zeros(layer.c, dtype=torch.float32)
        var = torch.ones(layer.c, dtype=torch.float32)
        scale = gamma / torch.sqrt(var + BN_EPS)
        shift = beta - mean * scale
        out["bn_scale"] = scale.numpy()
        out["bn_shift"] = shift.numpy()
    return out


def linear_inputs(layer: LinearLayer, seed: int, batch: Optional[int] = None):
    """x ~ N(0,1) [batch][in_features], w ~ N(0, w_std) [out_features][in_features]."""
    g = _gen(seed)
    b = layer.batch if batch is None else batch
    x = torch.randn((b, layer.in_features), generator=g, dtype=torch.float32)
    w = torch.randn((layer.out_features, layer.in_features), generator=g, dtype=torch.float32)
    w = w * layer.w_std
    return {"x": x.numpy(), "w": w.numpy()}


def config_layers(name: str) -> List:
    return list(CONFIGS[name])


def config_seed(name: str, layer_idx: int = 0) -> int:
    return 1000 + CONFIG_INDEX[name] + 100 * layer_idx


def random_conv_case(seed, n, c, h, w, k_out, kh, kw, with_zeros=False):
    """Small free-form case for tests: N(0,1) input and weights; optionally plants +-0.0
    entries so the sign rule at zero is exercised."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, c, h, w)).astype(np.float32)
    wt = rng.standard_normal((k_out, c, kh, kw)).astype(np.float32)
    if with_zeros:
        flat = x.reshape(-1)
        idx = rng.choice(flat.size, size=max(1, flat.size // 16), replace=False)
        flat[idx[::2]] = 0.0
        flat[idx[1::2]] = -0.0
        wf = wt.reshape(-1)
        idw = rng.choice(wf.size, size=max(1, wf.size // 16), replace=False)
        wf[idw[::2]] = 0.0
        wf[idw[1::2]] = -0.0
    return x, wt

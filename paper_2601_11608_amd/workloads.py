"""Seeded synthetic inputs shaped like the benchmark layers.

This module holds no arithmetic of the method: it only draws tensors.  Both
the GPU tests/benchmark and the CPU oracle's callers take their inputs from
here so that they see the same bits.  Values are drawn with a seeded torch
CPU generator in fp32 and rounded once to the layer's dtype.

The paper's own models are proprietary and it uses no public dataset; its
Table 1 only motivates C_in = 3 first layers.  These layers stand in for
them.
"""
import math

import torch

DTYPES = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


class Layer:
    def __init__(self, name, N, H, W, C_in, C_out, KH, KW, pad, F, dtype, bias, x_dist, relu=False):
        self.name, self.N, self.H, self.W = name, N, H, W
        self.C_in, self.C_out, self.KH, self.KW, self.pad, self.F = C_in, C_out, KH, KW, pad, F
        self.dtype, self.bias, self.x_dist, self.relu = dtype, bias, x_dist, relu

    def plan_args(self):
        return (self.N, self.H, self.W, self.C_in, self.C_out, self.KH, self.KW, self.pad, self.F)

    def with_batch(self, N):
        c = Layer(**{**self.__dict__})
        c.N = N
        return c


def fold_factor_for(C_in, W):
    """Smallest power-of-two F with F*C_in a multiple of 16 and W divisible by F
    (the rule used for the 5-layer stack); 1 when C_in is already a multiple of 32."""
    if C_in % 32 == 0:
        return 1
    F = 1
    while (F * C_in) % 16 != 0 or W % F != 0:
        F *= 2
        if F > W:
            raise ValueError("no fold factor for C_in=%d W=%d" % (C_in, W))
    return F


CONFIGS = {
    # 0: small fp32 case the oracle finishes at once
    "c1": [Layer("c1", 1, 32, 32, 3, 16, 3, 3, 1, 8, "f32", False, "uniform")],
    # 1: VGG-style first layer (headline)
    "c2": [Layer("c2", 64, 224, 224, 3, 64, 3, 3, 1, 16, "f16", True, "normal")],
    # 2: misaligned mid-network layer
    "c3": [Layer("c3", 32, 112, 112, 12, 48, 3, 3, 1, 4, "bf16", False, "relu_normal")],
    # 3: Conv1d, audio-like (H = KH = 1)
    "c4": [Layer("c4", 16, 1, 16000, 1, 64, 1, 9, 4, 32, "f16", False, "normal_0.3")],
}
_C5 = [3, 20, 36, 68, 132, 256]
CONFIGS["c5"] = [
    Layer("c5_L%d" % (i + 1), 32, 112, 112, _C5[i], _C5[i + 1], 3, 3, 1, fold_factor_for(_C5[i], 112), "bf16",
          False, "normal", relu=(i < 4))
    for i in range(5)
]
CONFIG_SEEDS = {"c1": 1000, "c2": 1001, "c3": 1002, "c4": 1003, "c5": 1004}


def draw_input(layer, gen, N=None):
    N = layer.N if N is None else N
    shape = (N, layer.H, layer.W, layer.C_in)
    if layer.x_dist == "uniform":
        x = torch.rand(shape, generator=gen) * 2 - 1
    elif layer.x_dist == "normal":
        x = torch.randn(shape, generator=gen)
    elif layer.x_dist == "relu_normal":
        x = torch.relu(torch.randn(shape, generator=gen))
    elif layer.x_dist == "normal_0.3":
        x = torch.randn(shape, generator=gen) * 0.3
    else:
        raise ValueError(layer.x_dist)
    return x.to(DTYPES[layer.dtype])


def draw_filter(layer, gen):
    shape = (layer.KH, layer.KW, layer.C_in, layer.C_out)
    if layer.x_dist == "uniform":
        w = torch.rand(shape, generator=gen) * 2 - 1
    else:  # Kaiming-normal, fan_in = KH*KW*C_in
        w = torch.randn(shape, generator=gen) * math.sqrt(2.0 / (layer.KH * layer.KW * layer.C_in))
    return w.to(DTYPES[layer.dtype])


def draw_bias(layer, gen):
    if not layer.bias:
        return None
    return (torch.rand((layer.C_out,), generator=gen) * 0.2 - 0.1).to(DTYPES[layer.dtype])


def make_config(name, N=None, seed=None):
    """Returns (layers, x, [w_i], [b_i]) as CPU tensors for config ``name``;
    ``N`` overrides the batch size (images are independent)."""
    layers = CONFIGS[name]
    gen = torch.Generator(device="cpu")
    gen.manual_seed(CONFIG_SEEDS[name] if seed is None else seed)
    x = draw_input(layers[0], gen, N)
    ws = [draw_filter(l, gen) for l in layers]
    bs = [draw_bias(l, gen) for l in layers]
    if N is not None:
        layers = [l.with_batch(N) for l in layers]
    return layers, x, ws, bs


def make_layer(layer, seed):
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    return draw_input(layer, gen), draw_filter(layer, gen), draw_bias(layer, gen)

"""Shared test helpers (no method arithmetic: conversions and the error metric)."""
import numpy as np
import torch

TOL = {"f32": 1e-5, "f16": 2e-3, "bf16": 8e-3}   # max over images of relative L2 error vs the fp64 oracle
TORCH_DT = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def f64(t):
    """torch tensor (any float dtype, any device) -> numpy float64, exactly."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def bits_as_f64(t):
    """Element bit patterns as float64 integers (exact), for bit-exactness checks
    of pure data movement through the value-agnostic oracle routines."""
    t = t.detach().to("cpu").contiguous()
    it = torch.int16 if t.element_size() == 2 else torch.int32
    return t.view(it).to(torch.float64).numpy()


def bits(t):
    t = t.detach().to("cpu").contiguous()
    it = torch.int16 if t.element_size() == 2 else torch.int32
    return t.view(it).numpy()


def rel_l2_per_image(y, ref):
    """max over images n of ||y[n]-ref[n]||_2 / ||ref[n]||_2 (float64 numpy inputs)."""
    y = y.reshape(y.shape[0], -1)
    ref = ref.reshape(ref.shape[0], -1)
    num = np.sqrt(((y - ref) ** 2).sum(axis=1))
    den = np.sqrt((ref ** 2).sum(axis=1))
    den = np.where(den == 0, 1.0, den)
    return float((num / den).max())

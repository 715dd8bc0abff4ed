"""Seeded synthetic inputs for the S-STE sparse-linear hot path.

This module holds NO arithmetic of the method (no projection, no sparsifier, no GEMM, no 8-bit
rescaling): it only draws Gaussian tensors with the shapes and scales of GPT-2 layers and rounds them
to bf16 with PyTorch's CPU cast.  Both the HIP path and the CPU oracle are fed from here so
that they see identical bits.

Shapes: W is (O, I) = (out, in) row-major, X is (T, I), dY is (T, O); T = batch x sequence tokens.
Distributions: W ~ N(0, 0.02^2) (GPT-2 initialisation), X ~ N(0, 1), dY ~ N(0, (1e-3)^2); the
second parameter quoted for each workload is a standard deviation.
"""
from dataclasses import dataclass
from typing import List, Tuple

import numpy as np
import torch

KIND_W, KIND_X, KIND_DY, KIND_UPDATE = 0, 1, 2, 3


@dataclass(frozen=True)
class Layer:
    name: str
    O: int
    I: int


@dataclass(frozen=True)
class Workload:
    cfg: int
    name: str
    T: int
    dtype: str            # "bf16" or "e4m3" (storage type of packed weights, X and dY)
    layers: Tuple[Layer, ...]
    base_seed: int


WORKLOADS = {
    1: Workload(1, "tiny 256x1024, 512 tokens", 512, "bf16", (Layer("fc", 256, 1024),), 0),
    2: Workload(2, "GPT-2-124M FFN fc1 3072x768, 8192 tokens", 8192, "bf16", (Layer("fc1", 3072, 768),), 2000),
    3: Workload(3, "GPT-2-350M FFN pair, 16384 tokens", 16384, "bf16",
                (Layer("fc1", 4096, 1024), Layer("fc2", 1024, 4096)), 3000),
    4: Workload(4, "GPT-2-774M block linears, 16384 tokens", 16384, "bf16",
                (Layer("qkv", 3840, 1280), Layer("proj", 1280, 1280), Layer("fc1", 5120, 1280),
                 Layer("fc2", 1280, 5120)), 4000),
    5: Workload(5, "GPT-2-774M block linears FP8 e4m3, 32768 tokens", 32768, "e4m3",
                (Layer("qkv", 3840, 1280), Layer("proj", 1280, 1280), Layer("fc1", 5120, 1280),
                 Layer("fc2", 1280, 5120)), 5000),
}

W_STD, X_STD, DY_STD, UPDATE_STD = 0.02, 1.0, 1e-3, 1e-4


def _generator(base_seed: int, layer_index: int, kind: int, step: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([base_seed, layer_index, kind, step])))


def gaussian_f32(shape, std, base_seed, layer_index, kind, step=0) -> np.ndarray:
    g = _generator(base_seed, layer_index, kind, step)
    out = g.standard_normal(size=shape, dtype=np.float32)
    out *= np.float32(std)
    return out


def to_bf16_bits(x_f32: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even (PyTorch CPU cast)."""
    t = torch.from_numpy(np.ascontiguousarray(x_f32)).to(torch.bfloat16)
    return t.view(torch.uint16).numpy().copy()


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(bits)).view(torch.bfloat16).to(torch.float32)
    return t.numpy().copy()


def weight_bits(wl: Workload, layer_index: int, O=None, I=None) -> np.ndarray:
    """bf16 master weight (O, I) as uint16 patterns."""
    L = wl.layers[layer_index]
    shape = (O or L.O, I or L.I)
    return to_bf16_bits(gaussian_f32(shape, W_STD, wl.base_seed, layer_index, KIND_W))


def weight_update_bits(w_bits: np.ndarray, wl: Workload, layer_index: int, step: int) -> np.ndarray:
    """Stand-in for an optimizer step on the dense master weight: W <- bf16(W + N(0, 1e-4^2))."""
    w = bf16_bits_to_f32(w_bits)
    w += gaussian_f32(w.shape, UPDATE_STD, wl.base_seed, layer_index, KIND_UPDATE, step)
    return to_bf16_bits(w)


def activations(wl: Workload, layer_index: int, T=None, I=None):
    """X (T, I) as bf16 patterns (uint16), and the scale 1 that goes with unquantised storage.  The
    8-bit workload derives its e4m3 operand from these with the per-tensor rescale + cast of Sec. 5.2,
    which is part of the method: the library's sste_cast_fp8 on one side, the oracle's cast on the other."""
    L = wl.layers[layer_index]
    x = gaussian_f32((T or wl.T, I or L.I), X_STD, wl.base_seed, layer_index, KIND_X)
    return to_bf16_bits(x), np.float32(1.0)


def output_gradient(wl: Workload, layer_index: int, T=None, O=None):
    """dY (T, O) as bf16 patterns (uint16) and the scale 1, like ``activations``."""
    L = wl.layers[layer_index]
    g = gaussian_f32((T or wl.T, O or L.O), DY_STD, wl.base_seed, layer_index, KIND_DY)
    return to_bf16_bits(g), np.float32(1.0)

"""Seeded synthetic inputs for the 3x3 convolution layers (shared by tests, bench, smoke).

Holds none of the method's arithmetic: only shapes and random draws.  The layer
shapes are Stable-Diffusion-shaped 3x3 / stride 1 / pad 1 convolutions (UNet and
VAE decoder), standing in for the real checkpoints the paper measured on
(Section "Evaluation"), plus the five layer shapes of the paper's Table 1.

Recipe: one CPU generator per layer, seed = BASE_SEED + layer index; draw x, then
w, then bias, each as fp32 standard normals scaled by its standard deviation
(x: 1, w: 1/sqrt(9*C), bias: 0.01), then cast once to the storage dtype.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import torch

BASE_SEED = 241205781


@dataclass(frozen=True)
class Layer:
    name: str
    N: int
    C: int
    K: int
    H: int
    W: int
    dtype: str          # "f32" | "f16"
    index: int          # position in ALL_LAYERS; fixes the seed

    @property
    def direct_flops(self) -> int:
        return 2 * self.N * self.K * self.C * self.H * self.W * 9


def _mk(rows):
    return [Layer(name, N, C, K, HW, HW, dt, i) for i, (name, N, C, K, HW, dt) in enumerate(rows)]


# name, N, C, K, H=W, dtype
ALL_LAYERS = _mk([
    ("A_conv_in",      1,    4,  320,   64, "f32"),
    ("B_resblock",     2,  320,  320,   64, "f16"),
    ("C1_unet",        2,  320,  640,   32, "f16"),
    ("C2_unet",        2,  640,  640,   32, "f16"),
    ("C3_unet",        2,  640, 1280,   16, "f16"),
    ("C4_unet",        2, 1280, 1280,   16, "f16"),
    ("C5_unet",        2, 1280, 1280,    8, "f16"),
    ("C6_unet",        2, 2560, 1280,    8, "f16"),
    ("C7_unet",        2, 1920,  640,   32, "f16"),
    ("C8_unet",        2,  960,  320,   64, "f16"),
    ("D1_sdxl",        2,  320,  320,  128, "f16"),
    ("D2_sdxl",        2,  640,  640,   64, "f16"),
    ("D3_sdxl",        2, 1280, 1280,   32, "f16"),
    ("E1_vae",         1,  512,  512,  128, "f16"),
    ("E2_vae",         1,  512,  512,  256, "f16"),
    ("E3_vae",         1,  256,  256,  512, "f16"),
    ("E4_vae",         1,  128,  128, 1024, "f16"),
    ("E5_vae_out",     1,  128,    3, 1024, "f16"),
    # the paper's Table 1 shapes, batch 1
    ("T1_640_640_32",    1,  640,  640, 32, "f16"),
    ("T1_1280_1280_16",  1, 1280, 1280, 16, "f16"),
    ("T1_2560_1280_16",  1, 2560, 1280, 16, "f16"),
    ("T1_320_320_64",    1,  320,  320, 64, "f16"),
    ("T1_640_320_64",    1,  640,  320, 64, "f16"),
    # the same five shapes with fp32 storage (the paper's F32 model type)
    ("T1f32_640_640_32",    1,  640,  640, 32, "f32"),
    ("T1f32_1280_1280_16",  1, 1280, 1280, 16, "f32"),
    ("T1f32_2560_1280_16",  1, 2560, 1280, 16, "f32"),
    ("T1f32_320_320_64",    1,  320,  320, 64, "f32"),
    ("T1f32_640_320_64",    1,  640,  320, 64, "f32"),
])
LAYERS = {l.name: l for l in ALL_LAYERS}

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}


def make_inputs(N: int, C: int, K: int, H: int, W: int, dtype: str = "f32",
                seed: int = BASE_SEED, with_bias: bool = True):
    """(x[N,C,H,W], w[K,C,3,3], bias[K] fp32 or None) as CPU tensors."""
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    x = torch.randn((N, C, H, W), generator=g, dtype=torch.float32)
    w = torch.randn((K, C, 3, 3), generator=g, dtype=torch.float32) * (1.0 / (9.0 * C) ** 0.5)
    b: Optional[torch.Tensor] = torch.randn((K,), generator=g, dtype=torch.float32) * 0.01
    td = TORCH_DTYPE[dtype]
    return x.to(td), w.to(td), (b if with_bias else None)


def make_layer_inputs(layer: Layer, dtype: Optional[str] = None):
    return make_inputs(layer.N, layer.C, layer.K, layer.H, layer.W,
                       dtype or layer.dtype, BASE_SEED + layer.index)

"""Seeded synthetic inputs for the five benchmark configurations.

Only random-number generation and reshaping live here: nothing of the layer's
arithmetic.  Both the GPU path and the CPU oracle are fed from these tensors.
The inputs stand in for the paper's workloads (teacher-MLP regression, the
methane table, CIFAR-10 images): same shapes and value distributions, no item
of those datasets.
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    n_in: int
    n_out: int
    grid: int
    batch: int
    coef_std: float
    seed: int
    x_kind: str = "normal"        # "normal" | "normal_t3" | "correlated" | "pixels"
    storage: tuple = ("f32",)     # coefficient storage variants measured for this config


# benchmark configs; cfg2 is a stack, listed layer by layer.
CFG1 = Workload("cfg1_16x16_G8", 16, 16, 8, 256, 0.1, 1)
CFG2_LAYERS = (
    Workload("cfg2_l0_64x256_G16", 64, 256, 16, 65536, 0.1, 20, x_kind="correlated"),
    Workload("cfg2_l1_256x256_G16", 256, 256, 16, 65536, 0.1, 21),
    Workload("cfg2_l2_256x256_G16", 256, 256, 16, 65536, 0.1, 22),
    Workload("cfg2_l3_256x1_G16", 256, 1, 16, 65536, 0.1, 23),
)
CFG3 = Workload("cfg3_1024x1024_G16", 1024, 1024, 16, 8192, 0.05, 3, storage=("f32", "f16"))
CFG4 = Workload("cfg4_128x128_G12_rows262144", 128, 128, 12, 262144, 0.1, 4, x_kind="pixels")
CFG5 = Workload("cfg5_4096x4096_G32", 4096, 4096, 32, 4096, 0.05, 5, x_kind="normal_t3",
                storage=("bf16",))

BY_NAME = {w.name: w for w in (CFG1, *CFG2_LAYERS, CFG3, CFG4, CFG5)}


@dataclass(frozen=True)
class ConvWorkload:
    """A convolution stage: channels-last images [n][h][w][c_in], kh x kw windows."""
    name: str
    n: int
    h: int
    w: int
    c_in: int
    kh: int
    kw: int
    stride: int
    n_out: int
    grid: int
    coef_std: float
    seed: int
    x_kind: str = "normal"
    storage: tuple = ("f32",)

    @property
    def n_in(self) -> int:
        return self.kh * self.kw * self.c_in

    @property
    def out_hw(self):
        return (self.h - self.kh) // self.stride + 1, (self.w - self.kw) // self.stride + 1

    @property
    def batch(self) -> int:      # rows of the equivalent fully connected layer
        oh, ow = self.out_hw
        return self.n * oh * ow


# Stages shaped like the convolutional backbones of Sec. 5 at width 128: the second 2x2 stride-2
# stage of the 32x32 backbone (16x16 feature maps), the second 3x3 stride-3 stage of the 81x81
# one (27x27 feature maps), and an overlapping 3x3 stride-1 stage for the gradient gathering.
# Feature maps are standardised (batch normalisation without affine parameters precedes every
# lmKAN layer), hence N(0,1) inputs.
CONV_2X2 = ConvWorkload("conv_2x2s2_16x16x128_to_128_G12", 1024, 16, 16, 128, 2, 2, 2, 128, 12, 0.1, 40)
CONV_3X3 = ConvWorkload("conv_3x3s3_27x27x32_to_96_G12", 512, 27, 27, 32, 3, 3, 3, 96, 12, 0.1, 41)
CONV_3X3_S1 = ConvWorkload("conv_3x3s1_16x16x32_to_64_G12", 256, 16, 16, 32, 3, 3, 1, 64, 12, 0.1, 42)
CONV_BY_NAME = {w.name: w for w in (CONV_2X2, CONV_3X3, CONV_3X3_S1)}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def make_image(w: ConvWorkload, device) -> torch.Tensor:
    """Feature maps [n][h][w][c_in] float32 ~ N(0,1)."""
    g = _gen(device, 1000 + w.seed)
    return torch.randn((w.n, w.h, w.w, w.c_in), generator=g, device=device, dtype=torch.float32)


def make_x(w: Workload, device, batch: int | None = None) -> torch.Tensor:
    """Layer inputs [batch][n_in] float32."""
    B = w.batch if batch is None else batch
    g = _gen(device, 1000 + w.seed)
    if w.x_kind == "normal":
        return torch.randn((B, w.n_in), generator=g, device=device, dtype=torch.float32)
    if w.x_kind == "normal_t3":
        # per element, a fair coin picks N(0,1) or Student-t with 3 degrees of freedom
        z = torch.randn((B, w.n_in), generator=g, device=device, dtype=torch.float32)
        chi = torch.randn((3, B, w.n_in), generator=g, device=device, dtype=torch.float32)
        t3 = z / torch.sqrt(chi.square().sum(0) / 3.0)
        coin = torch.rand((B, w.n_in), generator=g, device=device) < 0.5
        z2 = torch.randn((B, w.n_in), generator=g, device=device, dtype=torch.float32)
        return torch.where(coin, z2, t3).contiguous()
    if w.x_kind == "correlated":
        # unit-variance features with a random linear correlation: x = z A, rows of A^T normalised
        z = torch.randn((B, w.n_in), generator=g, device=device, dtype=torch.float32)
        A = torch.randn((w.n_in, w.n_in), generator=g, device=device, dtype=torch.float32)
        A = A / A.norm(dim=0, keepdim=True)
        return (z @ A).contiguous()
    if w.x_kind == "pixels":
        # images U[0,1] of 3 channels, one row per pixel, lifted to n_in channels by a fixed
        # random per-pixel linear map and standardised per channel (a 1x1-convolution stem
        # followed by batch normalisation without affine parameters)
        px = torch.rand((B, 3), generator=g, device=device, dtype=torch.float32)
        Wm = torch.randn((3, w.n_in), generator=g, device=device, dtype=torch.float32)
        bias = torch.randn((w.n_in,), generator=g, device=device, dtype=torch.float32)
        h = px @ Wm + bias
        h = (h - h.mean(0, keepdim=True)) / h.std(0, keepdim=True)
        return h.contiguous()
    raise ValueError(w.x_kind)


def make_coef(w: Workload, device) -> torch.Tensor:
    """float32 master coefficients [G+1][G+1][n_in/2][n_out] ~ N(0, coef_std)."""
    g = _gen(device, 2000 + w.seed)
    shape = (w.grid + 1, w.grid + 1, w.n_in // 2, w.n_out)
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32) * w.coef_std


def make_coef_bf16_chunked(w: Workload, device) -> torch.Tensor:
    """Same distribution generated slab by slab straight into bfloat16 (for tables too large
    to hold a float32 master next to them)."""
    g = _gen(device, 2000 + w.seed)
    W = w.grid + 1
    out = torch.empty((W, W, w.n_in // 2, w.n_out), device=device, dtype=torch.bfloat16)
    for a in range(W):
        out[a] = (torch.randn((W, w.n_in // 2, w.n_out), generator=g, device=device,
                              dtype=torch.float32) * w.coef_std).to(torch.bfloat16)
    return out


def make_grad_y(w: Workload, device, batch: int | None = None) -> torch.Tensor:
    B = w.batch if batch is None else batch
    g = _gen(device, 3000 + w.seed)
    return torch.randn((B, w.n_out), generator=g, device=device, dtype=torch.float32)


def store(coef_f32: torch.Tensor, storage: str) -> torch.Tensor:
    """Round the float32 master once (round-to-nearest-even) to the storage type."""
    return {"f32": coef_f32, "f16": coef_f32.to(torch.float16),
            "bf16": coef_f32.to(torch.bfloat16)}[storage]

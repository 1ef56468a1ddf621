"""Seeded synthetic inputs for the linear-angular attention layer.

This module only draws random tensors of ViT-stage shapes. It holds none of
the layer's arithmetic, so both the CPU oracle's tests and the HIP path's
tests can take their inputs from it without sharing any method code.

The five workloads stand in for the paper's ImageNet / COCO / ADE20K feature
maps (Sec. 4.1): a 14x14 classification stage, a 28x28 early stage, a 64x64
detection-resolution map and a 128x128 dense-prediction map. Values are i.i.d.
Gaussian; the depthwise-conv filters have std 0.1.

Draw order (fp32, CPU generator): Q, K, V, W, then the outlier mask if the
workload has one. Tensors are then cast to the I/O dtype; whoever consumes
them sees exactly the cast values.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16" | "f16"
    B: int
    heads: int
    d: int
    grid_h: int
    grid_w: int
    dw_kernel: int
    outlier_frac: float = 0.0   # fraction of tokens whose q,k,v are scaled
    outlier_scale: float = 1.0
    seed: int = 0

    @property
    def N(self) -> int:
        return self.grid_h * self.grid_w

    @property
    def units(self) -> int:
        return self.B * self.heads

    @property
    def tokens(self) -> int:
        return self.B * self.N

    @property
    def elems(self) -> int:
        return self.B * self.heads * self.N * self.d

    @property
    def itemsize(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def asdict(self) -> dict:
        out = asdict(self)
        out["N"] = self.N
        return out


# The five benchmark workloads, in the order the baseline file lists them.
WORKLOADS = (
    Workload("cfg1_f32_b1_h4_d32_n196_k3", "f32", 1, 4, 32, 14, 14, 3),
    Workload("cfg2_bf16_b64_h8_d64_n196_k3", "bf16", 64, 8, 64, 14, 14, 3),
    Workload("cfg3_bf16_b32_h6_d64_n784_k3_outliers", "bf16", 32, 6, 64, 28, 28, 3,
             outlier_frac=0.05, outlier_scale=8.0),
    Workload("cfg4_bf16_b8_h8_d64_n4096_k5", "bf16", 8, 8, 64, 64, 64, 5),
    Workload("cfg5_bf16_b2_h12_d64_n16384_k9", "bf16", 2, 12, 64, 128, 128, 9),
)


# Further shapes for measurements beyond the five benchmark workloads (bench.py --workload NAME):
# the dtypes and head widths of the wider coverage, at the size of cfg4 / cfg5.
EXTRA_WORKLOADS = (
    Workload("x_f16_b8_h8_d64_n4096_k5", "f16", 8, 8, 64, 64, 64, 5),
    Workload("x_f16_b2_h12_d64_n16384_k9", "f16", 2, 12, 64, 128, 128, 9),
    Workload("x_bf16_b8_h4_d128_n4096_k5", "bf16", 8, 4, 128, 64, 64, 5),
    Workload("x_bf16_b8_h32_d16_n4096_k5", "bf16", 8, 32, 16, 64, 64, 5),
    Workload("x_f16_b64_h8_d64_n196_k3", "f16", 64, 8, 64, 14, 14, 3),
    Workload("x_bf16_b8_h16_d32_n4096_k5", "bf16", 8, 16, 32, 64, 64, 5),
    Workload("x_bf16_b64_h16_d32_n196_k3", "bf16", 64, 16, 32, 14, 14, 3),
    Workload("x_bf16_b32_h1_d96_n3136_k3", "bf16", 32, 1, 96, 56, 56, 3),
    Workload("x_bf16_b32_h4_d96_n196_k3", "bf16", 32, 4, 96, 14, 14, 3),
)


def workload(index_or_name) -> Workload:
    if isinstance(index_or_name, int):
        return WORKLOADS[index_or_name]
    for w in WORKLOADS + EXTRA_WORKLOADS:
        if w.name == index_or_name or w.name.startswith(str(index_or_name) + "_"):
            return w
    raise KeyError(index_or_name)


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[name]


def make_inputs(wl: Workload, seed: int | None = None, with_bias: bool = False) -> dict:
    """CPU tensors q,k,v [B,heads,N,d], w [heads,d,k,k], bias [heads,d] or None."""
    g = torch.Generator(device="cpu")
    g.manual_seed(wl.seed if seed is None else seed)
    shape = (wl.B, wl.heads, wl.N, wl.d)
    q = torch.randn(shape, generator=g, dtype=torch.float32)
    k = torch.randn(shape, generator=g, dtype=torch.float32)
    v = torch.randn(shape, generator=g, dtype=torch.float32)
    w = torch.randn((wl.heads, wl.d, wl.dw_kernel, wl.dw_kernel), generator=g,
                    dtype=torch.float32) * 0.1
    if wl.outlier_frac > 0.0:
        # one Bernoulli draw per (batch, token), shared by all heads and by q, k and v
        u = torch.rand((wl.B, 1, wl.N, 1), generator=g, dtype=torch.float32)
        scale = torch.where(u < wl.outlier_frac,
                            torch.tensor(wl.outlier_scale), torch.tensor(1.0))
        q, k, v = q * scale, k * scale, v * scale
    bias = None
    if with_bias:
        bias = torch.randn((wl.heads, wl.d), generator=g, dtype=torch.float32) * 0.1
    dt = torch_dtype(wl.dtype)
    out = {"q": q.to(dt).contiguous(), "k": k.to(dt).contiguous(),
           "v": v.to(dt).contiguous(), "w": w.to(dt).contiguous(),
           "bias": None if bias is None else bias.to(dt).contiguous()}
    return out


def to_f64(t) -> np.ndarray | None:
    """Exact upcast of a stored tensor (fp32, bf16 or fp16) to a float64 numpy array."""
    if t is None:
        return None
    return t.detach().to("cpu").to(torch.float64).contiguous().numpy()

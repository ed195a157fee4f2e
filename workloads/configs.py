"""The five benchmark workloads and their seeded input generators.

Input recipe (all synthetic; the second parameter of N(.,.) is a variance):
  mlp            x1 ~ N(0,1), x2 ~ max(0, N(0,1)), dy ~ N(0, 0.01^2), fp32
  conv3x3        x ~ N(0,1), dy ~ N(0, 1e-4), fp32
  resnet20       x ~ N(0,1) (GroupNorm inputs too), dy ~ N(0, 1e-4), fp32
  resnet50       x ~ |N(0,1)| (post-ReLU), dy ~ N(0, 1e-4), rounded to bf16 (nearest-even)
  resnet50_nano  same tensors, micro-batch 1, per-layer clipping
One numpy Generator per (data seed, micro-step, layer) so any micro-step or layer
can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .layers import (GN, Layer, conv, resnet18_layers, resnet20_layers, resnet50_layers, resnet_bottleneck_layers,
                     tiny_mlp_layers)

WORKLOAD_NAMES = ("mlp", "conv3x3", "resnet20", "resnet50", "resnet50_nano",
                  # further layer sets for the same kernels (the paper's other networks)
                  "resnet50_gn", "resnet101_gn", "resnet18_gn")


@dataclass(frozen=True)
class Workload:
    name: str
    layers: Tuple[Layer, ...]
    n: int                      # examples per micro-step
    accum: int                  # micro-steps per optimiser step
    dtype: str                  # "f32" or "bf16": type of x and dy handed to the path
    clip_mode: str              # "global" or "per_layer"
    clip_c: float               # overall norm bound C
    sigma: float                # noise multiplier
    x_dist: Tuple[str, ...]     # per layer: "normal", "relu", "absnormal"
    dy_std: float
    data_seed: int
    philox_seed: int = 0
    step: int = 0

    @property
    def total_batch(self) -> int:
        return self.n * self.accum

    @property
    def group_of_layer(self) -> List[int]:
        if self.clip_mode == "global":
            return [0] * len(self.layers)
        return list(range(len(self.layers)))

    @property
    def n_groups(self) -> int:
        return 1 if self.clip_mode == "global" else len(self.layers)

    @property
    def n_params(self) -> int:
        return sum(l.pw + l.pb for l in self.layers)

    @property
    def flops_per_example(self) -> int:
        return sum(l.flops for l in self.layers)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def in_bytes_per_example(self) -> int:
        return sum(l.in_bytes(self.elem_bytes) for l in self.layers)


def get_workload(name: str, *, n: Optional[int] = None, accum: Optional[int] = None,
                 hw: Optional[int] = None) -> Workload:
    """Return one of the five workloads.  `n`, `accum` and `hw` (input resolution of the
    ResNet layer sets / the single conv layer) shrink it for tests without changing its structure."""
    if name == "mlp":
        layers = tuple(tiny_mlp_layers())
        wl = Workload(name, layers, 32, 1, "f32", "global", 1.0, 1.1, ("normal", "relu"), 0.01, 1001)
    elif name == "conv3x3":
        layers = (conv(64, 64, 3, 1, hw or 56, bias=True, name="conv"),)
        wl = Workload(name, layers, 16, 4, "f32", "per_layer", 1.0, 1.0, ("normal",), 0.01, 1002)
    elif name == "resnet20":
        layers = tuple(resnet20_layers(True, hw or 32))
        wl = Workload(name, layers, 256, 1, "f32", "global", 1.5, 1.2,
                      tuple("normal" for _ in layers), 0.01, 1003)
    elif name == "resnet50":
        layers = tuple(resnet50_layers(hw or 224))
        wl = Workload(name, layers, 32, 8, "bf16", "global", 1.0, 1.0,
                      tuple("absnormal" for _ in layers), 0.01, 1004)
    elif name == "resnet50_nano":
        layers = tuple(resnet50_layers(hw or 224))
        wl = Workload(name, layers, 1, 1024, "bf16", "per_layer", 1.0, 0.8,
                      tuple("absnormal" for _ in layers), 0.01, 1005)
    elif name in ("resnet50_gn", "resnet101_gn"):
        # bottleneck ResNets with GroupNorm(32) scale/shift gradients in the set (Table 3: ResNet-101-GN32)
        blocks = (3, 4, 6, 3) if name == "resnet50_gn" else (3, 4, 23, 3)
        layers = tuple(resnet_bottleneck_layers(blocks, hw or 224, 1000, 32))
        wl = Workload(name, layers, 32, 8, "bf16", "global", 1.0, 1.0,
                      tuple("normal" if l.kind == GN else "absnormal" for l in layers), 0.01, 1006)
    elif name == "resnet18_gn":
        # the CIFAR-10 / chest-CT network of Sections 3.2 and 3.6: ResNet-18 with GroupNorm, batch 32 x accumulation
        layers = tuple(resnet18_layers(hw or 32, 10, 32))
        wl = Workload(name, layers, 32, 8, "bf16", "global", 1.0, 1.0,
                      tuple("normal" if l.kind == GN else "absnormal" for l in layers), 0.01, 1007)
    else:
        raise KeyError(f"unknown workload {name!r}; choose from {WORKLOAD_NAMES}")
    if n is not None:
        wl = replace(wl, n=n)
    if accum is not None:
        wl = replace(wl, accum=accum)
    return wl


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the 16-bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (((u >> 16) & 1) + np.uint32(0x7FFF))
    return (rounded >> 16).astype(np.uint16)


def to_bf16_grid(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bf16."""
    bits = f32_to_bf16_bits(a).astype(np.uint32) << 16
    return bits.view(np.float32).reshape(a.shape)


def _draw(rng: np.random.Generator, shape, dist: str, std: float = 1.0) -> np.ndarray:
    a = rng.standard_normal(shape, dtype=np.float32)
    if dist == "relu":
        np.maximum(a, 0.0, out=a)
    elif dist == "absnormal":
        np.abs(a, out=a)
    elif dist != "normal":
        raise ValueError(dist)
    if std != 1.0:
        a *= np.float32(std)
    return a


def make_inputs(wl: Workload, micro_step: int = 0, layers: Optional[Sequence[int]] = None,
                n: Optional[int] = None):
    """Seeded (x, dy) pairs for one micro-step: a list over layers of
    (x [n, *x_shape], dy [n, *dy_shape]) fp32 arrays.  For bf16 workloads the values
    lie on the bf16 grid, so converting them to bf16 and to fp64 is exact on both sides."""
    n = wl.n if n is None else n
    out = []
    idxs = range(len(wl.layers)) if layers is None else layers
    for li in idxs:
        l = wl.layers[li]
        rng = np.random.default_rng([wl.data_seed, micro_step, li])
        x = _draw(rng, (n,) + tuple(l.x_shape), wl.x_dist[li])
        dy = _draw(rng, (n,) + tuple(l.dy_shape), "normal", wl.dy_std)
        if wl.dtype == "bf16":
            x = to_bf16_grid(x)
            dy = to_bf16_grid(dy)
        out.append((x, dy))
    return out

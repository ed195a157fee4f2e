"""Seeded synthetic workloads for the DPSGD gradient-privatisation path.

This module only describes layer shapes and draws random tensors.  It holds none
of the method's arithmetic (no gradients, norms, clipping or noise) and imports
neither the CPU oracle nor the HIP library, so both can be fed the same bits.

The paper (Section 3.1, Tables 1-4) measures ResNet-50/101/18 with GroupNorm on
ImageNet / CIFAR-10.  Those datasets are not available here and the path consumes
only (input activation, output gradient) pairs per layer, so tensors with the
networks' layer shapes and simple stated distributions stand in for them.
"""
from .layers import Layer, conv, dense, gn_affine, resnet20_layers, resnet50_layers, tiny_mlp_layers
from .configs import Workload, get_workload, WORKLOAD_NAMES, make_inputs, to_bf16_grid, f32_to_bf16_bits

__all__ = [
    "Layer", "conv", "dense", "gn_affine", "resnet20_layers", "resnet50_layers", "tiny_mlp_layers",
    "Workload", "get_workload", "WORKLOAD_NAMES", "make_inputs", "to_bf16_grid", "f32_to_bf16_bits",
]

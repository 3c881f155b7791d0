"""Seeded synthetic workloads: shapes, tensor order and random buffers.

This package holds no arithmetic of the method.  It fixes the shapes of the
workloads, the order of the trainable tensors along the chain (index 0 is the
input-most tensor), and draws every random buffer once on the host from a
fixed seed so that the CPU oracle and the HIP path consume identical bits.
"""
from .configs import MLPConfig, ViTConfig, ResNetConfig, VGGConfig, MobileNetConfig, CONFIGS, tensor_specs, mobilenet_blocks  # noqa: F401
from .gen import make_workload, bf16_round, Workload  # noqa: F401

"""Seeded buffers for the workloads.

Every buffer is drawn on the host with numpy's `default_rng`, one seed per
buffer (derived from the workload seed and the buffer's ordinal), and is
returned as float32.  For bf16 workloads the float32 values are rounded to
the nearest bf16 (ties to even) first, so converting them to bf16 on the
device, or widening them to float64 on the host, is exact.
"""
from dataclasses import dataclass
from typing import List

import numpy as np

from .configs import tensor_specs


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); result stays float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


@dataclass
class Workload:
    cfg: object
    names: List[str]
    weights: List[np.ndarray]    # float32, chain order; bf16-representable for bf16 configs
    snapshot: List[np.ndarray]   # weights + N(0, std 1e-3), same representation
    x: np.ndarray                # MLP: [B, dims[0]]; ViT: [B, tokens-1, patch_dim]; ResNet, VGG: [B, H, W, C]
    y: np.ndarray                # int32 labels, uniform over the classes


def _rng(seed: int, ordinal: int) -> np.random.Generator:
    return np.random.default_rng([seed, ordinal])


def _trunc_normal(rng, shape, std):
    """Normal(0, std) redrawn until inside +-2 std."""
    a = rng.standard_normal(shape)
    bad = np.abs(a) > 2.0
    while bad.any():
        a[bad] = rng.standard_normal(int(bad.sum()))
        bad = np.abs(a) > 2.0
    return a * std


def make_workload(cfg, seed: int = 0, init: str = "paper", batch: int = None) -> Workload:
    """Draw one workload.

    init="paper":  biases and LayerNorm shifts zero, LayerNorm gains one (the
                   benchmark configuration).
    init="random": biases/shifts N(0, 0.02) and gains 1 + N(0, 0.1), so that
                   parity cases exercise every term.
    batch overrides cfg.batch (used for bounded CPU timing samples).
    """
    specs = tensor_specs(cfg)
    B = cfg.batch if batch is None else batch
    quant = bf16_round if cfg.dtype == "bf16" else (lambda a: np.ascontiguousarray(a, dtype=np.float32))
    weights, snapshot, names = [], [], []
    for i, (name, shape) in enumerate(specs):
        rng = _rng(seed, 100 + i)
        if cfg.kind == "mlp":
            w = rng.standard_normal(shape) * np.sqrt(2.0 / shape[1])        # Kaiming normal, fan-in
        elif cfg.kind == "vgg":
            if name.endswith(".W"):                                          # He normal, fan-in
                w = rng.standard_normal(shape) * np.sqrt(2.0 / int(np.prod(shape[1:])))
            else:
                w = np.zeros(shape) if init == "paper" else 0.05 * rng.standard_normal(shape)
        elif cfg.kind in ("resnet", "mobilenet"):
            leaf = name.split(".")[-1]
            if leaf == "W":                                                  # He normal, fan-in
                w = rng.standard_normal(shape) * np.sqrt(2.0 / int(np.prod(shape[1:])))
            elif leaf == "g":
                # A folded BatchNorm gain carries the 1/sigma of the statistics it absorbed.  He-normal
                # kernels keep the second moment through convolution + ReLU, but every residual sum adds
                # the branch's to the stream's: the gains closing a ResNet block (last main convolution,
                # projection shortcut) are therefore below one, so that the stream stays O(1) through
                # the 16 blocks (0.25^2 + 0.9^2 ~ 0.9 where two zero-mean branches meet under a ReLU), and
                # the stem's gain brings the stream to a root mean square of about one (logits of a few
                # units, loss 6.6 at the full size).
                base = 1.0
                if cfg.kind == "resnet" and name.endswith("c3.g"):
                    base = 0.25
                elif cfg.kind == "resnet" and name.endswith("sc.g"):
                    base = 0.9
                elif cfg.kind == "resnet" and name == "stem.g":
                    base = 0.4
                w = base * (np.ones(shape) if init == "paper" else 1.0 + 0.1 * rng.standard_normal(shape))
            else:
                w = np.zeros(shape) if init == "paper" else 0.05 * rng.standard_normal(shape)
        else:
            leaf = name.split(".")[-1]
            if leaf == "W" or name in ("cls", "pos"):
                w = _trunc_normal(rng, shape, 0.02)
            elif leaf == "g":
                w = np.ones(shape) if init == "paper" else 1.0 + 0.1 * rng.standard_normal(shape)
            else:                                                            # biases, LayerNorm shifts
                w = np.zeros(shape) if init == "paper" else 0.02 * rng.standard_normal(shape)
        w = quant(w.astype(np.float32))
        s = quant((w.astype(np.float64) + 1e-3 * _rng(seed, 5000 + i).standard_normal(shape)).astype(np.float32))
        names.append(name)
        weights.append(w)
        snapshot.append(s)
    if cfg.kind == "mlp":
        x = _rng(seed, 1).standard_normal((B, cfg.dims[0])).astype(np.float32)
    elif cfg.kind in ("resnet", "vgg", "mobilenet"):
        x = quant(_rng(seed, 1).standard_normal((B, cfg.image, cfg.image, cfg.in_ch)).astype(np.float32))
    else:
        x = quant(_rng(seed, 1).standard_normal((B, cfg.tokens - 1, cfg.patch_dim)).astype(np.float32))
    y = _rng(seed, 2).integers(0, cfg.classes, size=B).astype(np.int32)
    return Workload(cfg, names, weights, snapshot, x, y)

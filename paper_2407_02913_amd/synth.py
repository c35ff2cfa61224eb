"""Seeded synthetic inputs for the SFC 3x3 convolution path.

This module only draws random numbers with the shapes and value distributions
of the workloads; it holds none of the method's arithmetic, so both the HIP
library's callers and the CPU oracle's callers may use it.

The paper evaluates on ImageNet with TorchVision ResNets (Sec. 6.1) and times
VGG-16 layers on an FPGA (Sec. 6.2).  Neither data nor weights are available
here, so ResNet-shaped stride-1 3x3 layers with post-ReLU-like int8
activations and Gaussian int8 weights stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20240702


@dataclass(frozen=True)
class LayerShape:
    name: str
    N: int
    Cin: int
    Cout: int
    H: int
    W: int
    dist: str  # "uniform" or "relu"
    per_channel_wscale: bool
    cfg: int  # seed group

    @property
    def direct_ops(self) -> int:
        """Direct-convolution-equivalent integer operations (2 per MAC)."""
        return 18 * self.N * self.H * self.W * self.Cin * self.Cout


#: The single-layer workloads.  "resnet56" is the one throughput is quoted on.
LAYERS = {
    "tiny32": LayerShape("tiny32", 1, 16, 16, 32, 32, "uniform", False, 1),
    "resnet56": LayerShape("resnet56", 32, 64, 64, 56, 56, "relu", True, 2),
    "resnet28": LayerShape("resnet28", 64, 128, 128, 28, 28, "relu", True, 3),
    "resnet14": LayerShape("resnet14", 128, 256, 256, 14, 14, "relu", True, 4),
    "resnet7": LayerShape("resnet7", 256, 512, 512, 7, 7, "relu", True, 5),
    # CIFAR-sized feature maps (powers of two): 4x4 tiles cover them exactly
    "cifar16": LayerShape("cifar16", 256, 128, 128, 16, 16, "relu", True, 6),
    "cifar8": LayerShape("cifar8", 512, 256, 256, 8, 8, "relu", True, 7),
}

#: ResNet-18-shaped stack of stride-1 3x3 layers at batch 64: (channels, spatial, count)
STACK_STAGES = ((64, 56, 4), (128, 28, 3), (256, 14, 3), (512, 7, 3))
STACK_BATCH = 64


def _rng(cfg: int, k: int, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng(BASE_SEED + 10 * cfg + k + 1000 * extra)


def activations(shape, dist: str, rng: np.random.Generator) -> np.ndarray:
    """int8 activations: uniform on [-128,127], or half-normal sigma=30 clipped to [0,127]."""
    if dist == "uniform":
        return rng.integers(-128, 128, size=shape, dtype=np.int64).astype(np.int8)
    if dist == "relu":
        a = np.abs(rng.normal(0.0, 30.0, size=shape))
        return np.clip(np.rint(a), 0, 127).astype(np.int8)
    raise ValueError(dist)


def weights(shape, dist: str, rng: np.random.Generator) -> np.ndarray:
    """int8 weights: uniform on [-128,127], or normal sigma=20 clipped to [-127,127]."""
    if dist == "uniform":
        return rng.integers(-128, 128, size=shape, dtype=np.int64).astype(np.int8)
    if dist == "relu":
        return np.clip(np.rint(rng.normal(0.0, 20.0, size=shape)), -127, 127).astype(np.int8)
    raise ValueError(dist)


def make_layer(shape: LayerShape, batch: int | None = None, extra: int = 0, kernel: int = 3):
    """Draw one layer's inputs.

    Returns a dict with ``x`` int8 [N,Cin,H,W], ``w`` int8 [Cout,Cin,kernel,kernel],
    ``x_scale`` (float), ``w_scale`` float32 [Cout] or [1], and ``x_calib``, a
    second activation tensor (4 images, different seed) for scale calibration.
    ``batch`` overrides N (for bounded CPU samples of the same workload).
    """
    n = shape.N if batch is None else batch
    x = activations((n, shape.Cin, shape.H, shape.W), shape.dist, _rng(shape.cfg, 0, extra))
    w = weights((shape.Cout, shape.Cin, kernel, kernel), shape.dist, _rng(shape.cfg, 1, extra))
    if shape.per_channel_wscale:
        ws = _rng(shape.cfg, 2, extra).uniform(0.005, 0.02, size=shape.Cout).astype(np.float32)
    else:
        ws = np.array([0.01], dtype=np.float32)
    xc = activations((min(n, 4), shape.Cin, shape.H, shape.W), shape.dist, _rng(shape.cfg, 3, extra))
    return {"x": x, "w": w, "x_scale": 0.02, "w_scale": ws, "x_calib": xc, "shape": shape}


def stack_layers(batch: int = STACK_BATCH):
    """The 13 stride-1 3x3 layer shapes of the ResNet-18-shaped stack, in order."""
    out = []
    idx = 0
    for c, hw, count in STACK_STAGES:
        for _ in range(count):
            out.append(LayerShape(f"stack{idx}_c{c}_s{hw}", batch, c, c, hw, hw, "relu", True, 6 + idx))
            idx += 1
    return out

"""Seeded synthetic inputs for the VGG19 path (images, parameters, labels).

This module only draws numbers; it holds none of the model's arithmetic and is
the one piece of code that both the CPU oracle's tests and the GPU library's
tests use, so that both sides see bit-identical fp32 inputs.

Recipe (stands in for ImageNet images and trained weights, which the paper's
section "VGG19 forward pass" used and which are not available offline):
  * one numpy Generator(PCG64(seed)) per call, draws in this fixed order:
    image batch, then for each layer in network order the weight tensor and
    then the bias, then the labels;
  * images  ~ U[0,1)   (or N(0,1) for the single-layer microbenchmark),
  * weights ~ N(0, 2/fan_in)  ("He-normal"; fan_in = 9*Cin for a 3x3
    convolution, In for a dense layer),
  * biases  = 0.01,
  * labels  ~ uniform integers in [0, classes);
  * everything is drawn in float64 and rounded once to float32.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

# (Cin, Cout) of the sixteen 3x3 convolutions; a 2x2 max-pool follows the
# layers whose index is in POOL_AFTER.
CONV_CHANNELS: Tuple[Tuple[int, int], ...] = (
    (3, 64), (64, 64),
    (64, 128), (128, 128),
    (128, 256), (256, 256), (256, 256), (256, 256),
    (256, 512), (512, 512), (512, 512), (512, 512),
    (512, 512), (512, 512), (512, 512), (512, 512),
)
POOL_AFTER: Tuple[int, ...] = (1, 3, 7, 11, 15)


@dataclass
class VGGInputs:
    """fp32 canonical-layout tensors: x [N,3,H,W]; conv_w[l] [Cout,Cin,3,3];
    fc_w[l] [Out,In] (the first dense layer's columns are in C,H,W flatten
    order); labels int32 [N]."""
    x: np.ndarray
    conv_w: List[np.ndarray] = field(default_factory=list)
    conv_b: List[np.ndarray] = field(default_factory=list)
    fc_w: List[np.ndarray] = field(default_factory=list)
    fc_b: List[np.ndarray] = field(default_factory=list)
    labels: np.ndarray | None = None


def _normal(rng: np.random.Generator, shape, std: float) -> np.ndarray:
    return (rng.standard_normal(shape) * std).astype(np.float32)


def conv_layer_inputs(N: int, H: int, W: int, Cin: int, Cout: int, seed: int = 0
                      ) -> Dict[str, np.ndarray]:
    """Single-layer microbenchmark inputs: x ~ N(0,1) [N,Cin,H,W], He-normal
    weights [Cout,Cin,3,3], bias 0.01, and an upstream gradient ~ N(0,1)
    [N,Cout,H,W] for backward tests."""
    rng = np.random.default_rng(np.random.PCG64(seed))
    x = _normal(rng, (N, Cin, H, W), 1.0)
    w = _normal(rng, (Cout, Cin, 3, 3), float(np.sqrt(2.0 / (9 * Cin))))
    b = np.full((Cout,), 0.01, dtype=np.float32)
    dy = _normal(rng, (N, Cout, H, W), 1.0)
    return {"x": x, "w": w, "b": b, "dy": dy}


def vgg19_inputs(N: int, H: int, W: int, fc_hidden: int, classes: int, seed: int = 0,
                 with_labels: bool = True) -> VGGInputs:
    """Whole-network inputs.  The flatten width is 512*(H/32)*(W/32)."""
    if H % 32 or W % 32:
        raise ValueError("H and W must be multiples of 32 (five 2x2 pools)")
    rng = np.random.default_rng(np.random.PCG64(seed))
    out = VGGInputs(x=rng.random((N, 3, H, W)).astype(np.float32))
    for cin, cout in CONV_CHANNELS:
        out.conv_w.append(_normal(rng, (cout, cin, 3, 3), float(np.sqrt(2.0 / (9 * cin)))))
        out.conv_b.append(np.full((cout,), 0.01, dtype=np.float32))
    flat = 512 * (H // 32) * (W // 32)
    dims = [(flat, fc_hidden), (fc_hidden, fc_hidden), (fc_hidden, classes)]
    for fin, fout in dims:
        out.fc_w.append(_normal(rng, (fout, fin), float(np.sqrt(2.0 / fin))))
        out.fc_b.append(np.full((fout,), 0.01, dtype=np.float32))
    if with_labels:
        out.labels = rng.integers(0, classes, size=(N,), dtype=np.int64).astype(np.int32)
    return out


def tiny_config(seed: int = 0) -> VGGInputs:
    """Batch 2, 3x32x32 images, classifier 512->512->512->10."""
    return vgg19_inputs(2, 32, 32, 512, 10, seed)


def full_config(N: int = 100, seed: int = 0, with_labels: bool = True) -> VGGInputs:
    """Batch N, 3x224x224 images, classifier 25088->4096->4096->1000."""
    return vgg19_inputs(N, 224, 224, 4096, 1000, seed, with_labels)
